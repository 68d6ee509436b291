// One shard of the bf16 instantiations (see instances_f32.hip for the sharding scheme).
#include "gemm_bf16.hpp"
#include "registry.hpp"

#ifndef KS_SHARD
#error "compile with -DKS_SHARD=<n>"
#endif
#define KS_CAT2(a, b) a##b
#define KS_CAT(a, b) KS_CAT2(a, b)

namespace ks {

template <int F, int BM, int BN, int BK, int WM, int WN, bool SPLIT>
static void launch_bf16_fixed(const GemmParams &p, int grid, int variant, hipStream_t s) {
    constexpr int NT = 64 * (BM / WM) * (BN / WN);
    const dim3 g = launch_grid(p, grid), b(NT);
    // variant bit 4: the operands are IEEE binary16 instead of bf16
#define KS_V(A, B, V)                                                                                        \
    do {                                                                                                     \
        if (variant & 16)                                                                                    \
            hipLaunchKernelGGL((gemm_bf16_kernel<F, BM, BN, BK, WM, WN, SPLIT, A, B, V, true>), g, b, 0, s, p);  \
        else                                                                                                 \
            hipLaunchKernelGGL((gemm_bf16_kernel<F, BM, BN, BK, WM, WN, SPLIT, A, B, V, false>), g, b, 0, s, p); \
    } while (0)
    switch (variant & 7) {
        case 0: KS_V(false, false, false); break;
        case 1: KS_V(false, false, true); break;
        case 2: KS_V(false, true, false); break;
        case 3: KS_V(false, true, true); break;
        case 4: KS_V(true, false, false); break;
        case 5: KS_V(true, false, true); break;
        case 6: KS_V(true, true, false); break;
        default: KS_V(true, true, true); break;
    }
#undef KS_V
}

// SPLITMODE 0: never split-K; 1: always; 2: decided per call (variant bit 3), both forms compiled
template <int F, int BM, int BN, int BK, int WM, int WN, int SPLITMODE>
static void launch_bf16(const GemmParams &p, int grid, int variant, hipStream_t s) {
    if constexpr (SPLITMODE == 2) {
        if (variant & 8) launch_bf16_fixed<F, BM, BN, BK, WM, WN, true>(p, grid, variant & 23, s);
        else launch_bf16_fixed<F, BM, BN, BK, WM, WN, false>(p, grid, variant & 23, s);
    } else {
        launch_bf16_fixed<F, BM, BN, BK, WM, WN, SPLITMODE == 1>(p, grid, variant & 23, s);
    }
}

template <int SHARD>
static void fill(LaunchFn *table) {
#define KS_BF16_INSTANCE(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK) \
    if constexpr ((id) % kShards == SHARD && compiled_bf16(id)) table[id] = &launch_bf16<F, BM, BN, BK, WM, WN, ((SPLITK) == 0 ? 2 : (SPLITK) > 1 ? 1 : 0)>;
#include "instances.def"
#undef KS_BF16_INSTANCE
}

void KS_CAT(register_bf16_shard_, KS_SHARD)(LaunchFn *table) { fill<KS_SHARD>(table); }

}  // namespace ks
