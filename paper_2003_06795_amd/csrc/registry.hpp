// Host-side registry of the kernel family: launch-function tables filled by the instance shards.
#pragma once
#include "ks_common.hpp"

namespace ks {

// variant index = akc*4 + bkc*2 + vec
typedef void (*LaunchFn)(const GemmParams &p, int grid, int variant, hipStream_t stream);

struct InstanceDesc {
    int id, core, bm, bn, bk, p1, p2, threads, splitK, ldsBytes, kw;
    int band = 8;        // tile rows per band of the one-dimensional tile order
    int sk = 0;          // > 0: has a balanced persistent form of 256 * sk work-groups
};

// Pruned library (paper Sections I and II-B: every instantiation costs binary size and build time,
// which is what the pruning of Section III is for).  With -DKS_KEPT_ONLY only the members the
// deployed trees can return (kept_set.inc, written with the trees) and the four bring-up tiles are
// compiled; the launch table entries of the others stay null and ks_kernel_info reports them absent.
#include "kept_set.inc"
constexpr int kKeptF32[] = KS_KEPT_F32;
constexpr int kKeptBf16[] = KS_KEPT_BF16;
template <int N>
constexpr bool id_in(const int (&list)[N], int id) {
    for (int i = 0; i < N; ++i)
        if (list[i] == id) return true;
    return false;
}
#ifdef KS_KEPT_ONLY
constexpr bool compiled_f32(int id) { return id_in(kKeptF32, id); }
constexpr bool compiled_bf16(int id) { return id_in(kKeptBf16, id); }
#else
constexpr bool compiled_f32(int) { return true; }
constexpr bool compiled_bf16(int) { return true; }
#endif

constexpr int kNumF32 = 64;
constexpr int kNumBf16 = 48;
constexpr int kShards = 16;

}  // namespace ks
