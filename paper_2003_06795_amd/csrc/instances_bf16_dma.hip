// One shard of the direct-to-LDS bf16 instantiations (see instances_f32.hip for the sharding scheme).
#include "gemm_bf16_dma.hpp"
#include "registry.hpp"

#ifndef KS_SHARD
#error "compile with -DKS_SHARD=<n>"
#endif
#define KS_CAT2(a, b) a##b
#define KS_CAT(a, b) KS_CAT2(a, b)

namespace ks {

// variant = akc * 2 + bkc
template <int F, int BM, int BN, int BK, int WM, int WN, int STAGES, bool SPLIT>
static void launch_bf16_dma(const GemmParams &p, int grid, int variant, hipStream_t s) {
    constexpr int NT = 64 * (BM / WM) * (BN / WN);
    const dim3 g((unsigned)grid), b(NT);
#define KS_V(A, B) hipLaunchKernelGGL((gemm_bf16_dma_kernel<F, BM, BN, BK, WM, WN, STAGES, SPLIT, A, B>), g, b, 0, s, p)
    switch (variant) {
        case 0: KS_V(false, false); break;
        case 1: KS_V(false, true); break;
        case 2: KS_V(true, false); break;
        default: KS_V(true, true); break;
    }
#undef KS_V
}

template <int SHARD>
static void fill(LaunchFn *table) {
#define KS_BF16_INSTANCE(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK) \
    if constexpr ((id) % kShards == SHARD) table[id] = &launch_bf16_dma<F, BM, BN, BK, WM, WN, STAGES, ((SPLITK) > 1)>;
#include "instances.def"
#undef KS_BF16_INSTANCE
}

void KS_CAT(register_bf16_dma_shard_, KS_SHARD)(LaunchFn *table) { fill<KS_SHARD>(table); }

}  // namespace ks
