// One shard of the fp32 instantiations: compiled KS_NSHARDS times with -DKS_SHARD=0..KS_NSHARDS-1
// so the family builds in parallel.  Each shard fills its ids of the launch table.
#include "gemm_f32.hpp"
#include "gemm_f32_direct.hpp"
#include "gemm_f32_kslice.hpp"
#include "registry.hpp"

#ifndef KS_SHARD
#error "compile with -DKS_SHARD=<n>"
#endif
#define KS_CAT2(a, b) a##b
#define KS_CAT(a, b) KS_CAT2(a, b)

namespace ks {

template <int CORE, int BM, int BN, int BK, int P1, int P2, bool SPLIT, int KW>
static void launch_f32_fixed(const GemmParams &p, int grid, int variant, hipStream_t s) {
    constexpr int NT = F32Shape<CORE, BM, BN, P1, P2>::threads * KW;
    // the multi-tile form exists beside the single-tile one and runs when the host asks for it
    constexpr bool MULTI_OK = !SPLIT && f32_multi_tile(CORE, BM, BN, P1, P2, KW);
    const dim3 g = launch_grid(p, grid), b(NT);
#define KS_V(A, B, V)                                                                                   \
    do {                                                                                                \
        if constexpr (CORE == CORE_KSLICE)                                                              \
            hipLaunchKernelGGL((gemm_f32_kslice_kernel<BM, BN, BK, P1, P2, SPLIT, A, B, V>), g, b, 0, s, p); \
        else if constexpr (CORE == CORE_DIRECT)                                                         \
            hipLaunchKernelGGL((gemm_f32_direct_kernel<BM, BN, BK, P1, P2, SPLIT, A, B, V>), g, b, 0, s, p); \
        else if constexpr (MULTI_OK) {                                                                  \
            if (p.tilesPerWG > 1)                                                                       \
                hipLaunchKernelGGL((gemm_f32_kernel<CORE, BM, BN, BK, P1, P2, SPLIT, A, B, V, KW, true>), g, b, 0, s, p); \
            else                                                                                        \
                hipLaunchKernelGGL((gemm_f32_kernel<CORE, BM, BN, BK, P1, P2, SPLIT, A, B, V, KW>), g, b, 0, s, p); \
        } else                                                                                          \
            hipLaunchKernelGGL((gemm_f32_kernel<CORE, BM, BN, BK, P1, P2, SPLIT, A, B, V, KW>), g, b, 0, s, p);  \
    } while (0)
    switch (variant) {
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
template <int CORE, int BM, int BN, int BK, int P1, int P2, int SPLITMODE, int KW>
static void launch_f32(const GemmParams &p, int grid, int variant, hipStream_t s) {
    if constexpr (SPLITMODE == 2) {
        if (variant & 8) launch_f32_fixed<CORE, BM, BN, BK, P1, P2, true, KW>(p, grid, variant & 7, s);
        else launch_f32_fixed<CORE, BM, BN, BK, P1, P2, false, KW>(p, grid, variant & 7, s);
    } else {
        launch_f32_fixed<CORE, BM, BN, BK, P1, P2, SPLITMODE == 1, KW>(p, grid, variant & 7, s);
    }
}

// Members with a balanced persistent form: that form (two kernels) when the host set it up,
// otherwise the plain member of the same tiles.
template <int CORE, int BM, int BN, int BK, int P1, int P2>
static void launch_f32_sk(const GemmParams &p, int grid, int variant, hipStream_t s) {
    if (p.skGroups <= 0) {
        launch_f32_fixed<CORE, BM, BN, BK, P1, P2, false, 1>(p, grid, variant & 7, s);
        return;
    }
    constexpr int NT = F32Shape<CORE, BM, BN, P1, P2>::threads;
    const dim3 g((unsigned)p.skGroups), b(NT);
#define KS_V(A, B, V) \
    hipLaunchKernelGGL((gemm_f32_kernel<CORE, BM, BN, BK, P1, P2, false, A, B, V, 1, false, true>), g, b, 0, s, p)
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
    if (p.skTailTiles > 0)
        hipLaunchKernelGGL((gemm_f32_sk_fixup_kernel<BM, BN, BK, P1, P2>), dim3((unsigned)p.skTailTiles, NT / 64),
                           dim3(64), 0, s, p);
}

template <int SHARD>
static void fill(LaunchFn *table) {
#define KS_F32_INSTANCE_SK(id, CORE, BM, BN, BK, P1, P2, PERCU) \
    if constexpr ((id) % kShards == SHARD && compiled_f32(id)) table[id] = &launch_f32_sk<CORE_##CORE, BM, BN, BK, P1, P2>;
#define KS_F32_INSTANCE_KW(id, CORE, BM, BN, BK, P1, P2, SPLITK, KW) \
    if constexpr ((id) % kShards == SHARD && compiled_f32(id)) table[id] = &launch_f32<CORE_##CORE, BM, BN, BK, P1, P2, ((SPLITK) == 0 ? 2 : (SPLITK) > 1 ? 1 : 0), KW>;
#define KS_F32_INSTANCE(id, CORE, BM, BN, BK, P1, P2, SPLITK) KS_F32_INSTANCE_KW(id, CORE, BM, BN, BK, P1, P2, SPLITK, 1)
#include "instances.def"
#undef KS_F32_INSTANCE
#undef KS_F32_INSTANCE_KW
#undef KS_F32_INSTANCE_SK
}

void KS_CAT(register_f32_shard_, KS_SHARD)(LaunchFn *table) { fill<KS_SHARD>(table); }

}  // namespace ks
