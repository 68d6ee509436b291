// Runtime kernel selection (paper Section IV): a decision tree deployed as integer comparisons.
// Host only; no device access, no allocation.
#include "../../include/ks_gemm.h"

#include <limits.h>
#include <string.h>

#include "selector_table.inc"

namespace {

struct Deployed {
    ks_tree_node_t nodes[KS_MAX_TREE_NODES];
    int n;
    bool custom;
};
Deployed g_tree[2];

const ks_tree_node_t *builtin(int dtype, int *n) {
    if (dtype == KS_F32) {
        *n = (int)(sizeof(kTreeF32) / sizeof(kTreeF32[0]));
        return kTreeF32;
    }
    *n = (int)(sizeof(kTreeBf16) / sizeof(kTreeBf16[0]));
    return kTreeBf16;
}

const ks_tree_node_t *active(int dtype, int *n) {
    if (g_tree[dtype].custom) {
        *n = g_tree[dtype].n;
        return g_tree[dtype].nodes;
    }
    return builtin(dtype, n);
}

int64_t sat_mul(int64_t a, int64_t b) {
    if (a == 0 || b == 0) return 0;
    if (a > INT64_MAX / b) return INT64_MAX;
    return a * b;
}

}  // namespace

extern "C" int ks_features(int64_t M, int64_t N, int64_t K, int64_t batch, int transA, int transB,
                           int64_t *out) {
    if (!out) return KS_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || batch < 0) return KS_ERR_INVALID_ARG;
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return KS_ERR_INVALID_ARG;
    out[0] = M;
    out[1] = N;
    out[2] = K;
    out[3] = batch;
    out[4] = transA;
    out[5] = transB;
    out[6] = sat_mul(M, N);
    out[7] = sat_mul(out[6], K);
    out[8] = M < N ? M : N;
    out[9] = M < N ? N : M;
    return KS_OK;
}

extern "C" int ks_select(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch, int transA,
                         int transB) {
    if (dtype == KS_F16) dtype = KS_BF16;          // the fp16 form runs the 16-bit family with its tree
    if (dtype != KS_F32 && dtype != KS_BF16) return KS_ERR_INVALID_ARG;
    int64_t f[KS_NUM_FEATURES];
    const int rc = ks_features(M, N, K, batch, transA, transB, f);
    if (rc != KS_OK) return rc;
    int n = 0;
    const ks_tree_node_t *t = active(dtype, &n);
    int i = 0;
    // children always have larger indices than their parent, so the walk ends within n steps
    for (int step = 0; step < n; ++step) {
        if (t[i].feature < 0) return t[i].value;
        i = f[t[i].feature] <= t[i].threshold ? t[i].left : t[i].right;
    }
    return t[i].feature < 0 ? t[i].value : KS_ERR_INVALID_ARG;
}

extern "C" int ks_set_selector(int dtype, const ks_tree_node_t *nodes, int n) {
    if (dtype != KS_F32 && dtype != KS_BF16) return KS_ERR_INVALID_ARG;
    if (n == 0) {
        g_tree[dtype].custom = false;
        return KS_OK;
    }
    if (!nodes || n < 0 || n > KS_MAX_TREE_NODES) return KS_ERR_INVALID_ARG;
    const int nk = ks_num_kernels(dtype);
    for (int i = 0; i < n; ++i) {
        if (nodes[i].feature < 0) {
            if (nodes[i].value < 0 || nodes[i].value >= nk) return KS_ERR_INVALID_ARG;
        } else {
            if (nodes[i].feature >= KS_NUM_FEATURES) return KS_ERR_INVALID_ARG;
            if (nodes[i].left <= i || nodes[i].left >= n) return KS_ERR_INVALID_ARG;
            if (nodes[i].right <= i || nodes[i].right >= n) return KS_ERR_INVALID_ARG;
        }
    }
    memcpy(g_tree[dtype].nodes, nodes, sizeof(ks_tree_node_t) * (size_t)n);
    g_tree[dtype].n = n;
    g_tree[dtype].custom = true;
    return KS_OK;
}

extern "C" int ks_get_selector(int dtype, ks_tree_node_t *nodes, int cap) {
    if (dtype != KS_F32 && dtype != KS_BF16) return KS_ERR_INVALID_ARG;
    int n = 0;
    const ks_tree_node_t *t = active(dtype, &n);
    if (!nodes || cap < n) return KS_ERR_INVALID_ARG;
    memcpy(nodes, t, sizeof(ks_tree_node_t) * (size_t)n);
    return n;
}

extern "C" const char *ks_status_string(int status) {
    switch (status) {
        case KS_OK: return "success";
        case KS_ERR_INVALID_ARG: return "invalid argument";
        case KS_ERR_UNSUPPORTED: return "unsupported size";
        case KS_ERR_LAUNCH: return "HIP launch failed or no device";
        case KS_ERR_WORKSPACE: return "split-K workspace missing or too small";
        default: return status > 0 ? "not a status (non-negative value)" : "unknown status";
    }
}
