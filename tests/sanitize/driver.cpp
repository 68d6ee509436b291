// Host-only driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the C oracle and of
// the library's host code (offline tuner, selector): walks their entry points over seeded data with
// exactly-sized heap buffers, ragged sizes, padded leading dimensions, batches, empty dimensions and
// the tuner's edge cases, so that any out-of-bounds access or undefined operation aborts the run.
// Results are only sanity-checked here; their values are the business of the other tests.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/ks_gemm.h"

extern "C" {
int oracle_gemm_f32(int, int, int64_t, int64_t, int64_t, float, const float *, int64_t, const float *, int64_t, float,
                    float *, int64_t, int64_t, int64_t, int64_t, int64_t);
int oracle_gemm_bias_f32(int, int, int64_t, int64_t, int64_t, float, const float *, int64_t, const float *, int64_t,
                         float, float *, int64_t, int64_t, int64_t, int64_t, int64_t, const float *);
int oracle_gemm_bf16(int, int, int64_t, int64_t, int64_t, float, const uint16_t *, int64_t, const uint16_t *, int64_t,
                     float, float *, int64_t, int64_t, int64_t, int64_t, int64_t);
int oracle_gemm_out_bf16(int, int, int, int64_t, int64_t, int64_t, float, const void *, int64_t, const void *, int64_t,
                         float, uint16_t *, int64_t, int64_t, int64_t, int64_t, int64_t, const float *);
int oracle_gemm_f32_entries(int, int, int64_t, int64_t, int64_t, float, const float *, int64_t, const float *, int64_t,
                            float, const float *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, const int64_t *,
                            const int64_t *, const int64_t *, float *);
uint16_t oracle_round_to_bf16(double);
double oracle_widen_f16(uint16_t);
}

// The registry lives in the HIP translation unit, which is not part of this host-only build; the
// selector only needs the family sizes, counted here from the same instance list.
static const int kCountF32 = 0
#define KS_F32_INSTANCE(...) +1
#define KS_F32_INSTANCE_KW(...) +1
#include "../../paper_2003_06795_amd/csrc/instances.def"
#undef KS_F32_INSTANCE
#undef KS_F32_INSTANCE_KW
    ;
static const int kCountBf16 = 0
#define KS_BF16_INSTANCE(...) +1
#include "../../paper_2003_06795_amd/csrc/instances.def"
#undef KS_BF16_INSTANCE
    ;
extern "C" int ks_num_kernels(int dtype) { return dtype == KS_F32 ? kCountF32 : (dtype == KS_BF16 || dtype == KS_F16) ? kCountBf16 : KS_ERR_INVALID_ARG; }

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double rnd() {
    g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
    return (double)(g_state >> 11) / 9007199254740992.0;
}
#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "driver: %s failed at line %d\n", #c, __LINE__); exit(2); } } while (0)

static void oracle_cases() {
    const int shapes[][4] = {{1, 1, 1, 1}, {7, 5, 3, 2}, {33, 17, 40, 1}, {0, 5, 4, 1}, {5, 0, 4, 2}, {6, 4, 0, 3}, {9, 9, 9, 0}};
    for (auto &sh : shapes)
        for (int tA = 0; tA < 2; ++tA)
            for (int tB = 0; tB < 2; ++tB) {
                const int64_t M = sh[0], N = sh[1], K = sh[2], batch = sh[3];
                const int64_t rowsA = tA ? K : M, colsA = tA ? M : K, rowsB = tB ? N : K, colsB = tB ? K : N;
                const int64_t lda = colsA + 3, ldb = colsB + 1, ldc = N + 2;
                const int64_t sA = rowsA * lda + 5, sB = 0 /* broadcast */, sC = M * ldc + 7;
                // exactly as many elements as the call may touch
                std::vector<float> A((size_t)(batch > 0 ? (batch - 1) * sA + (rowsA ? (rowsA - 1) * lda + colsA : 0) : 0));
                std::vector<float> B((size_t)(rowsB ? (rowsB - 1) * ldb + colsB : 0));
                std::vector<float> C((size_t)(batch > 0 ? (batch - 1) * sC + (M ? (M - 1) * ldc + N : 0) : 0));
                std::vector<float> bias((size_t)N);
                for (auto &v : A) v = (float)(2 * rnd() - 1);
                for (auto &v : B) v = (float)(2 * rnd() - 1);
                for (auto &v : C) v = (float)(2 * rnd() - 1);
                for (auto &v : bias) v = (float)rnd();
                std::vector<float> C0 = C;
                REQUIRE(oracle_gemm_f32(tA, tB, M, N, K, 1.5f, A.data(), lda, B.data(), ldb, -0.5f, C.data(), ldc, batch, sA, sB, sC) == 0);
                C = C0;
                REQUIRE(oracle_gemm_bias_f32(tA, tB, M, N, K, 1.0f, A.data(), lda, B.data(), ldb, 0.0f, C.data(), ldc, batch, sA, sB, sC, bias.data()) == 0);
                for (auto v : C) REQUIRE(isfinite(v) || M * N == 0);
                if (M > 0 && N > 0 && batch > 0) {
                    const int64_t bb[2] = {0, batch - 1}, ii[2] = {0, M - 1}, jj[2] = {0, N - 1};
                    float out[2];
                    REQUIRE(oracle_gemm_f32_entries(tA, tB, M, N, K, 1.0f, A.data(), lda, B.data(), ldb, 0.5f, C0.data(), ldc, batch, sA, sB, sC, 2, bb, ii, jj, out) == 0);
                }
                // 16-bit operands and 16-bit output
                std::vector<uint16_t> A16(A.size()), B16(B.size()), C16(C.size());
                for (size_t i = 0; i < A.size(); ++i) A16[i] = oracle_round_to_bf16(A[i]);
                for (size_t i = 0; i < B.size(); ++i) B16[i] = oracle_round_to_bf16(B[i]);
                for (size_t i = 0; i < C.size(); ++i) C16[i] = oracle_round_to_bf16(C0[i]);
                C = C0;
                REQUIRE(oracle_gemm_bf16(tA, tB, M, N, K, 1.0f, A16.data(), lda, B16.data(), ldb, 0.25f, C.data(), ldc, batch, sA, sB, sC) == 0);
                REQUIRE(oracle_gemm_out_bf16(1, tA, tB, M, N, K, 1.0f, A16.data(), lda, B16.data(), ldb, 1.0f, C16.data(), ldc, batch, sA, sB, sC, bias.data()) == 0);
            }
    for (unsigned b = 0; b < 65536; b += 7) (void)oracle_widen_f16((uint16_t)b);
    REQUIRE(oracle_round_to_bf16(1.0) == 0x3F80);
}

static void tuner_cases() {
    const int dims[][3] = {{1, 1, 1}, {5, 3, 6}, {64, 17, 10}, {200, 24, 10}};
    for (auto &d : dims) {
        const int rows = d[0], cols = d[1], nf = d[2];
        std::vector<double> P((size_t)rows * cols), Ph(P.size());
        std::vector<int64_t> X((size_t)rows * nf);
        for (int s = 0; s < rows; ++s) {
            const int64_t M = 8 + (int64_t)(rnd() * 4000), N = 8 + (int64_t)(rnd() * 4000), K = 8 + (int64_t)(rnd() * 4000);
            int64_t f[KS_NUM_FEATURES];
            REQUIRE(ks_features(M, N, K, s % 5 == 0 ? 1024 : 1, s & 1, (s >> 1) & 1, f) == KS_OK);
            for (int j = 0; j < nf; ++j) X[(size_t)s * nf + j] = f[j];
            for (int c = 0; c < cols; ++c) P[(size_t)s * cols + c] = 1e9 * (0.1 + rnd() + (c == (int)(M % cols) ? 1.0 : 0.0));
        }
        REQUIRE(ks_tune_normalise(P.data(), rows, cols, Ph.data()) == KS_OK);
        for (int leaves : {1, 2, 8, 64}) {
            std::vector<int32_t> kept((size_t)leaves);
            std::vector<ks_tree_node_t> reg((size_t)2 * leaves - 1);
            int nodes = 0;
            const int nk = ks_tune_prune_tree(X.data(), nf, Ph.data(), rows, cols, leaves, 1, kept.data(), reg.data(), &nodes);
            REQUIRE(nk >= 1 && nk <= leaves && nodes >= 1 && nodes <= 2 * leaves - 1);
            double ach = 0;
            REQUIRE(ks_tune_achievable(Ph.data(), rows, cols, kept.data(), nk, &ach) == KS_OK && ach > 0 && ach <= 1.0 + 1e-12);
            for (int msl : {1, 4}) {
                std::vector<ks_tree_node_t> tree(KS_MAX_TREE_NODES);
                const int tn = ks_tune_fit_selector(X.data(), nf, P.data(), rows, cols, kept.data(), nk, 12, msl, nullptr, tree.data(), KS_MAX_TREE_NODES);
                REQUIRE(tn >= 1);
                std::vector<int32_t> chosen((size_t)rows);
                REQUIRE(ks_tune_predict(tree.data(), tn, X.data(), nf, rows, chosen.data()) == KS_OK);
                double sc = 0;
                REQUIRE(ks_tune_selector_score(Ph.data(), rows, cols, chosen.data(), &sc) == KS_OK && sc <= ach + 1e-12);
                // deploy, walk, restore
                if (nf >= KS_NUM_RAW_FEATURES) {
                    bool ids_ok = true;
                    for (int i = 0; i < tn; ++i) if (tree[i].feature < 0 && tree[i].value >= kCountBf16) ids_ok = false;
                    if (ids_ok && ks_set_selector(KS_BF16, tree.data(), tn) == KS_OK) {
                        for (int s = 0; s < rows; ++s) {
                            const int64_t *x = &X[(size_t)s * nf];
                            REQUIRE(ks_select(KS_BF16, x[0], x[1], x[2], x[3], (int)x[4], (int)x[5]) == chosen[s]);
                        }
                        std::vector<ks_tree_node_t> back((size_t)tn);
                        REQUIRE(ks_get_selector(KS_BF16, back.data(), tn) == tn);
                        REQUIRE(ks_get_selector(KS_BF16, back.data(), tn - 1) < 0 || tn == 1);
                        REQUIRE(ks_set_selector(KS_BF16, nullptr, 0) == KS_OK);
                    }
                }
            }
            std::vector<int32_t> k2((size_t)leaves);
            REQUIRE(ks_tune_prune_top_n(Ph.data(), rows, cols, leaves, k2.data()) >= 1);
            if (leaves <= rows) {
                REQUIRE(ks_tune_prune_kmeans(Ph.data(), rows, cols, leaves, 0, 50, k2.data()) >= 1);
                const int pd = cols < 3 ? cols : 3;
                REQUIRE(ks_tune_prune_kmeans(Ph.data(), rows, cols, leaves, pd, 50, k2.data()) >= 1);
            }
        }
        if (rows >= 5) {
            std::vector<int32_t> kh((size_t)cols), lab((size_t)rows);
            for (int mcs : {2, 5, 40})
                REQUIRE(ks_tune_prune_hdbscan(Ph.data(), rows, cols, mcs, mcs < 5 ? 1 : mcs, kh.data(), cols, lab.data()) >= 1);
            REQUIRE(ks_tune_prune_hdbscan(Ph.data(), rows, cols, 1, 1, kh.data(), cols, nullptr) < 0);
        }
        std::vector<double> ratio((size_t)cols);
        // a table without variance (one row, or one column of ones) is refused, anything else is not
        REQUIRE(ks_tune_pca_variance(Ph.data(), rows, cols, ratio.data()) == (rows > 1 && cols > 1 ? KS_OK : KS_ERR_INVALID_ARG));
    }
    // the compiled-in trees over a spread of sizes, and the error paths
    for (int i = 0; i < 20000; ++i) {
        const int64_t M = (int64_t)exp(rnd() * 28), N = (int64_t)exp(rnd() * 28), K = (int64_t)exp(rnd() * 28);
        const int a = ks_select(KS_F32, M, N, K, 1 + (int64_t)(rnd() * 5000), i & 1, (i >> 1) & 1);
        const int b = ks_select(KS_BF16, M, N, K, 1, i & 1, (i >> 1) & 1);
        REQUIRE(a >= 0 && a < 64 && b >= 0 && b < 64);
    }
    REQUIRE(ks_select(KS_F32, -1, 1, 1, 1, 0, 0) < 0 && ks_select(9, 1, 1, 1, 1, 0, 0) < 0);
    REQUIRE(ks_tune_normalise(nullptr, 1, 1, nullptr) < 0);
    REQUIRE(ks_status_string(KS_ERR_WORKSPACE) != nullptr && ks_status_string(-99) != nullptr);
}

int main() {
    oracle_cases();
    tuner_cases();
    printf("sanitize driver: ok\n");
    return 0;
}
