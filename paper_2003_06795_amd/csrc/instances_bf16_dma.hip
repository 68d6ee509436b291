// One shard of the direct-to-LDS bf16 instantiations (see instances_f32.hip for the sharding scheme).
#include "gemm_bf16_pp.hpp"
#include "registry.hpp"

#ifndef KS_SHARD
#error "compile with -DKS_SHARD=<n>"
#endif
#define KS_CAT2(a, b) a##b
#define KS_CAT(a, b) KS_CAT2(a, b)

namespace ks {

// The eight-wave 256 x 256 x 64 members (128 x 64 of output per wave) and the eight-wave
// 128 x 128 x 128 members on 16x16x32 fragments run in the form with two groups of waves
// alternating between memory and MFMA slots (gemm_bf16_pp.hpp).
template <int F, int BM, int BN, int BK, int WM, int WN, int STAGES>
constexpr bool kTwoGroups = bf16_two_groups(F, BM, BN, BK, WM, WN, STAGES);

// variant = akc * 2 + bkc
template <int F, int BM, int BN, int BK, int WM, int WN, int STAGES, bool SPLIT>
static void launch_bf16_dma_fixed(const GemmParams &p, int grid, int variant, hipStream_t s) {
    constexpr int NT = 64 * (BM / WM) * (BN / WN);
    const dim3 g = launch_grid(p, grid), b(NT);
    // variant bit 4: the operands are IEEE binary16 instead of bf16
#define KS_V(A, B)                                                                                                  \
    do {                                                                                                            \
        if constexpr (kTwoGroups<F, BM, BN, BK, WM, WN, STAGES>) {                                                  \
            if (variant & 16) hipLaunchKernelGGL((gemm_bf16_pp_kernel<F, SPLIT, A, B, true, 0, BM, BK>), g, b, 0, s, p);  \
            else hipLaunchKernelGGL((gemm_bf16_pp_kernel<F, SPLIT, A, B, false, 0, BM, BK>), g, b, 0, s, p);        \
        } else if (variant & 16)                                                                                    \
            hipLaunchKernelGGL((gemm_bf16_dma_kernel<F, BM, BN, BK, WM, WN, STAGES, SPLIT, A, B, true>), g, b, 0, s, p);  \
        else                                                                                                        \
            hipLaunchKernelGGL((gemm_bf16_dma_kernel<F, BM, BN, BK, WM, WN, STAGES, SPLIT, A, B, false>), g, b, 0, s, p); \
    } while (0)
    switch (variant & 3) {
        case 0: KS_V(false, false); break;
        case 1: KS_V(false, true); break;
        case 2: KS_V(true, false); break;
        default: KS_V(true, true); break;
    }
#undef KS_V
}

// SPLITMODE 0: never split-K; 1: always; 2: decided per call (variant bit 3), both forms compiled
template <int F, int BM, int BN, int BK, int WM, int WN, int STAGES, int SPLITMODE>
static void launch_bf16_dma(const GemmParams &p, int grid, int variant, hipStream_t s) {
    if constexpr (SPLITMODE == 2) {
        if (variant & 8) launch_bf16_dma_fixed<F, BM, BN, BK, WM, WN, STAGES, true>(p, grid, variant & 19, s);
        else launch_bf16_dma_fixed<F, BM, BN, BK, WM, WN, STAGES, false>(p, grid, variant & 19, s);
    } else {
        launch_bf16_dma_fixed<F, BM, BN, BK, WM, WN, STAGES, SPLITMODE == 1>(p, grid, variant & 19, s);
    }
}

template <int SHARD>
static void fill(LaunchFn *table) {
#define KS_BF16_INSTANCE(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK) \
    if constexpr ((id) % kShards == SHARD && compiled_bf16(id)) table[id] = &launch_bf16_dma<F, BM, BN, BK, WM, WN, STAGES, ((SPLITK) == 0 ? 2 : (SPLITK) > 1 ? 1 : 0)>;
#include "instances.def"
#undef KS_BF16_INSTANCE
}

void KS_CAT(register_bf16_dma_shard_, KS_SHARD)(LaunchFn *table) { fill<KS_SHARD>(table); }

}  // namespace ks
