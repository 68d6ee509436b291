// 256 x 256 x 64 and 128 x 128 x 128 members of the 16-bit family (paper Section II: one work-group
// tile, wave tile and K-step of the templated kernel) in their "two groups of waves" form for
// gfx950.  The description below uses the numbers of the 256 x 256 x 64 tile; the 128 x 128 x 128
// tile (TILE = 128, BK = 128: 64-row halves of the same 16 KB, 32 x 16 blocks per wave and quadrant,
// 16x16x32 fragments only, 256 matrix-pipe clocks per compute slot) runs the same schedule.
//
// The eight waves of a work-group form two groups of four; a SIMD holds one wave of each group.
// Every K-step is cut into two pairs of slots, a memory slot (LDS -> register fragment reads and
// the issue of direct-to-LDS global loads) followed by a compute slot (sixteen 32x32x16 or
// thirty-two 16x16x32 MFMAs, 512 clocks of the matrix pipe), each slot closed by s_barrier.  The
// second group runs one slot behind the first, so on every SIMD one wave streams MFMAs while the
// other feeds the memory pipes, and the matrix pipe never waits for an LDS read or a load issue.
//
// Tile decomposition: the 256 x 256 tile is four 128 x 128 quadrants (i, j); wave (wr, wc) of the
// 2 x 4 wave grid owns the 64 x 32 block at rows wr*64, columns wc*32 of each quadrant (128 x 64
// entries per wave in all).  The operand tiles live in LDS as halves A0, A1 (rows 0..127 /
// 128..255 of the A tile) and B0, B1, two stages each (128 KB); a half is released by the barrier
// behind the second group's slot that reads it and is refilled at once with the K-step after
// next, so loads run 1.5 K-steps ahead of their use although there are only two stages.
//
// Slots of K-step t (stage s = t & 1), per wave:
//   M0  read A0, B0, B1 fragments   issue A1(t+1) -> stage s^1             wait: A1(t) landed
//   C0  quadrants (0,0), (0,1)
//   M1  read A1 fragments           issue A0, B0, B1 (t+2) -> stage s      wait: A0, B0, B1 (t+1) landed
//   C1  quadrants (1,1), (1,0)
// A memory slot ends with the wave's own LDS reads complete (so the half may be overwritten after
// the barrier) and with the wave's own part of the half read next complete (s_waitcnt vmcnt); the
// barrier then publishes both to the work-group.  Loads are issued in the fixed order
// [A0 B0 B1](u), A1(u), [A0 B0 B1](u+1), ... so each wait leaves exactly the eight youngest loads
// in flight.  Past the end of the K range the same loads are issued on the last K-step's
// addresses into halves nobody reads any more: every step is the same straight-line code.
// Preconditions are those of gemm_bf16_dma.hpp.
#pragma once
#include "gemm_bf16_dma.hpp"

namespace ks {

// Per-lane source offsets (bytes from the tile origin, row0 / col0 at this K-step) of the two
// direct-to-LDS loads a wave contributes to one 128-row half of an operand tile.
template <bool KC, int HALF = 128, int BK = 64, int F = 32>
struct PpPlan {
    static_assert(HALF * BK == 8192, "a half tile is 16 KB: sixteen 1 KB loads, two per wave");
    unsigned off[2];
    __device__ __forceinline__ void init(int wave, int lane, long long ld, int row0, int half, int limit) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int L = (wave + j * 8) * 64 + lane;            // 16-byte slot in the LDS half
            if constexpr (KC) {
                constexpr int CPR = BK / 8, RP = 16 / CPR;       // as in Bf16Lds<BK>::chunk
                const int r = L / CPR, pos = L % CPR;
                const int c = pos ^ ((r / RP) & (CPR - 1));
                const int row = min(row0 + half * HALF + r, limit - 1) - row0;
                off[j] = (unsigned)(((long long)row * ld + c * 8) * 2);
            } else {
                constexpr int CPK = HALF / 8;                    // 16-byte chunks per k row
                const int k = L / CPK, pos = L % CPK;
                const int c = pos ^ (2 * Bf16LdsT<HALF, F>::swz(k));
                const int row = min(row0 + half * HALF + c * 8, limit - 8) - row0;
                off[j] = (unsigned)(((long long)k * ld + row) * 2);
            }
        }
    }
    // tile: wave-uniform address of the tile origin at this K-step; lds: the LDS half (wave-uniform).
    // Written as one instruction sequence so that the load keeps the form "scalar base + 32-bit
    // lane offset" and so that the compiler, which cannot tell which LDS half an in-flight load
    // fills once control flow merges, does not guard every LDS read with a full vmcnt wait: the
    // waits for these loads are the explicit ones in the K loop.  M0 (the LDS destination) is
    // written here and read by nothing else in this kernel.
    __device__ __forceinline__ void issue(const char *tile, char *lds, int wave) const {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const unsigned dst = (unsigned)(uintptr_t)(lds_void_ptr)(lds + (wave + j * 8) * 1024);
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :
                         : "v"(off[j]), "s"(tile), "s"(dst)
                         : "memory");
        }
    }
};

// ABLATE != 0 exists for measurement only (ks_bf16_ablation): bit 0 leaves out the direct-to-LDS
// loads after the first two K-steps (LDS keeps their contents), bit 1 the LDS fragment reads after
// the first two K-steps (the registers keep theirs), so that the cost of each data path can be read
// off against the full kernel on the same operand values (the result is then not a GEMM).  Bit 2
// changes nothing in the computation: the first lane of work-group 0 reads the shader cycle counter
// and the 100 MHz reference counter at both ends of its K loop and leaves the differences in
// pp_probe_clocks, which gives the clock the device holds while this kernel runs.
static __device__ unsigned long long pp_probe_clocks[2];

template <int F, bool SPLIT, bool AKC, bool BKC, bool F16 = false, int ABLATE = 0, int TILE = 256, int BK = 64>
__global__ __launch_bounds__(512) void gemm_bf16_pp_kernel(const GemmParams p) {
    static_assert((TILE == 256 && BK == 64) || (TILE == 128 && BK == 128 && F == 16), "tiles of this form");
    constexpr int BM = TILE, BN = TILE, HALF = TILE / 2;
    constexpr int WBM = HALF / 2, WBN = HALF / 4;            // a wave's block of one quadrant: 64 x 32 or 32 x 16
    constexpr int FM = WBM / F, FN = WBN / F;                // its fragments
    constexpr int KSTEP = F == 32 ? 16 : 32, NSUB = BK / KSTEP;
    constexpr int HB = HALF * BK * 2;                        // bytes of one half tile
    __shared__ __attribute__((aligned(1024))) char A00[HB];  // A<stage><half>
    __shared__ __attribute__((aligned(1024))) char A01[HB];
    __shared__ __attribute__((aligned(1024))) char A10[HB];
    __shared__ __attribute__((aligned(1024))) char A11[HB];
    __shared__ __attribute__((aligned(1024))) char B00[HB];
    __shared__ __attribute__((aligned(1024))) char B01[HB];
    __shared__ __attribute__((aligned(1024))) char B10[HB];
    __shared__ __attribute__((aligned(1024))) char B11[HB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 2, wc = wave & 3;
    const TileCoord tc = tile_of_block(p);
    const int row0 = tc.tm * BM, col0 = tc.tn * BN;
    const int kBegin = tc.split * p.kChunk;
    const int kEnd = min(p.K, kBegin + p.kChunk);
    const int nk = (kEnd - kBegin) / BK;
    const uint16_t *Ab = static_cast<const uint16_t *>(p.A) + (long long)tc.batch * p.strideA;
    const uint16_t *Bb = static_cast<const uint16_t *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    // measurement only (ABLATE bit 3): every work-group fetches the operand panels of tile (0, 0),
    // so all loads hit in L2 and nothing crosses the fabric; the result is then not a GEMM
    const int lrow0 = (ABLATE & 8) ? 0 : row0, lcol0 = (ABLATE & 8) ? 0 : col0;
    const char *aTile = reinterpret_cast<const char *>(AKC ? Ab + (long long)lrow0 * p.lda + kBegin
                                                            : Ab + (long long)kBegin * p.lda + lrow0);
    const char *bTile = reinterpret_cast<const char *>(BKC ? Bb + (long long)lcol0 * p.ldb + kBegin
                                                            : Bb + (long long)kBegin * p.ldb + lcol0);
    const long long aStep = AKC ? BK * 2LL : BK * 2LL * p.lda;
    const long long bStep = BKC ? BK * 2LL : BK * 2LL * p.ldb;

    PpPlan<AKC, HALF, BK, F> pa0, pa1;
    PpPlan<BKC, HALF, BK, F> pb0, pb1;
    pa0.init(wave, lane, p.lda, lrow0, 0, p.M);
    pa1.init(wave, lane, p.lda, lrow0, 1, p.M);
    pb0.init(wave, lane, p.ldb, lcol0, 0, p.N);
    pb1.init(wave, lane, p.ldb, lcol0, 1, p.N);

    // acc[i][j]: the wave's block of quadrant (i, j)
    floatx4 acc16[2][2][F == 16 ? FM : 1][F == 16 ? FN : 1];
    floatx16 acc32[2][2][F == 32 ? FM : 1][F == 32 ? FN : 1];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int m = 0; m < FM; ++m)
#pragma unroll
            for (int n = 0; n < FN; ++n) {
                if constexpr (F == 16) acc16[q >> 1][q & 1][m][n] = floatx4{0.f, 0.f, 0.f, 0.f};
                else
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc32[q >> 1][q & 1][m][n][e] = 0.f;
            }

    bf16x8 a[FM][NSUB], b0[FN][NSUB], b1[FN][NSUB];

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    auto lds_a = [&](auto s, auto h) -> char * {
        constexpr int S = decltype(s)::value, H = decltype(h)::value;
        return S == 0 ? (H == 0 ? A00 : A01) : (H == 0 ? A10 : A11);
    };
    auto lds_b = [&](auto s, auto h) -> char * {
        constexpr int S = decltype(s)::value, H = decltype(h)::value;
        return S == 0 ? (H == 0 ? B00 : B01) : (H == 0 ? B10 : B11);
    };
    auto read_a = [&](const char *half) {
#pragma unroll
        for (int m = 0; m < FM; ++m)
#pragma unroll
            for (int ks = 0; ks < NSUB; ++ks)
                a[m][ks] = read_fragment<F, HALF, BK, AKC>(half, wr * WBM + m * F, ks * KSTEP, lane);
    };
    auto read_b = [&](const char *half, bf16x8 (&b)[FN][NSUB]) {
#pragma unroll
        for (int n = 0; n < FN; ++n)
#pragma unroll
            for (int ks = 0; ks < NSUB; ++ks)
                b[n][ks] = read_fragment<F, HALF, BK, BKC>(half, wc * WBN + n * F, ks * KSTEP, lane);
    };
    auto mma = [&](auto qi, auto qj, const bf16x8 (&b)[FN][NSUB]) {
        constexpr int QI = decltype(qi)::value, QJ = decltype(qj)::value;
#pragma unroll
        for (int ks = 0; ks < NSUB; ++ks)
#pragma unroll
            for (int m = 0; m < FM; ++m)
#pragma unroll
                for (int n = 0; n < FN; ++n) {
                    if constexpr (F == 16)
                        acc16[QI][QJ][m][n] = mfma_16x16x32<F16>(a[m][ks], b[n][ks], acc16[QI][QJ][m][n]);
                    else
                        acc32[QI][QJ][m][n] = mfma_32x32x16<F16>(a[m][ks], b[n][ks], acc32[QI][QJ][m][n]);
                }
    };
    // end of a slot: nothing moves across it, then the work-group barrier
    auto slot_end = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    // end of a memory slot: at most the eight youngest loads of this wave still in flight and all
    // of its LDS reads returned (vmcnt(8), lgkmcnt(0); the export counter is left alone)
    auto memory_slot_end = [&]() {
        wait_vmcnt<8>();
        __builtin_amdgcn_s_waitcnt(0xC07F);
        slot_end();
    };

    auto step = [&](int t, auto s) {
        constexpr int S = decltype(s)::value;
        using SC = std::integral_constant<int, S>;
        using SN = std::integral_constant<int, S ^ 1>;
        const int t1 = min(t + 1, nk - 1), t2 = min(t + 2, nk - 1);
        const bool reads = (ABLATE & 2) == 0 || t < 2;
        // M0
        if (reads) {
            read_a(lds_a(SC{}, I0{}));
            read_b(lds_b(SC{}, I0{}), b0);
            read_b(lds_b(SC{}, I1{}), b1);
        }
        if constexpr ((ABLATE & 1) == 0) pa1.issue(aTile + t1 * aStep, lds_a(SN{}, I1{}), wave);
        memory_slot_end();
        // C0: the wave that is issuing MFMAs goes ahead of the one issuing memory instructions
        __builtin_amdgcn_s_setprio(1);
        mma(I0{}, I0{}, b0);
        mma(I0{}, I1{}, b1);
        __builtin_amdgcn_s_setprio(0);
        slot_end();
        // M1
        if (reads) read_a(lds_a(SC{}, I1{}));
        if constexpr ((ABLATE & 1) == 0) {
            pa0.issue(aTile + t2 * aStep, lds_a(SC{}, I0{}), wave);
            pb0.issue(bTile + t2 * bStep, lds_b(SC{}, I0{}), wave);
            pb1.issue(bTile + t2 * bStep, lds_b(SC{}, I1{}), wave);
        }
        memory_slot_end();
        // C1
        __builtin_amdgcn_s_setprio(1);
        mma(I1{}, I1{}, b1);
        mma(I1{}, I0{}, b0);
        __builtin_amdgcn_s_setprio(0);
        slot_end();
    };

    // A work-group whose K partition is empty (possible for the last split-K partition) only
    // writes zeros; the branch is uniform over the work-group, so the barriers stay matched.
    unsigned long long probeC = 0, probeR = 0;
    if constexpr ((ABLATE & 4) != 0) {
        if (blockIdx.x == 0 && tid == 0) { probeC = __builtin_amdgcn_s_memtime(); probeR = __builtin_amdgcn_s_memrealtime(); }
    }
    if (nk > 0) {
        // prologue: K-steps 0 and 1 except A1(1), in the order the waits count on
        const int s1 = min(1, nk - 1);
        pa0.issue(aTile, lds_a(I0{}, I0{}), wave);
        pb0.issue(bTile, lds_b(I0{}, I0{}), wave);
        pb1.issue(bTile, lds_b(I0{}, I1{}), wave);
        pa1.issue(aTile, lds_a(I0{}, I1{}), wave);
        pa0.issue(aTile + s1 * aStep, lds_a(I1{}, I0{}), wave);
        pb0.issue(bTile + s1 * bStep, lds_b(I1{}, I0{}), wave);
        pb1.issue(bTile + s1 * bStep, lds_b(I1{}, I1{}), wave);
        wait_vmcnt<8>();
        slot_end();
        if (wr == 1) slot_end();                             // the second group starts one slot later

        int t = 0;
        for (; t + 2 <= nk; t += 2) {
            step(t, I0{});
            step(t + 1, I1{});
        }
        if (t < nk) step(t, I0{});
        // the loads issued past the end must have landed before this work-group's LDS is given away
        wait_vmcnt<0>();
        if (wr == 0) slot_end();                             // pairs with the second group's last slot
    }
    if constexpr ((ABLATE & 4) != 0) {
        if (blockIdx.x == 0 && tid == 0) {
            pp_probe_clocks[0] = __builtin_amdgcn_s_memtime() - probeC;
            pp_probe_clocks[1] = __builtin_amdgcn_s_memrealtime() - probeR;
        }
    }

#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int i = q >> 1, j = q & 1;
        if constexpr (F == 16)
            write_tile_mfma16<SPLIT, FM, FN>(p, tc, Cb, row0 + i * HALF + wr * WBM, col0 + j * HALF + wc * WBN, lane,
                                             acc16[i][j]);
        else
            write_tile_mfma32<SPLIT, FM, FN>(p, tc, Cb, row0 + i * HALF + wr * WBM, col0 + j * HALF + wc * WBN, lane,
                                             acc32[i][j]);
    }
}

}  // namespace ks
