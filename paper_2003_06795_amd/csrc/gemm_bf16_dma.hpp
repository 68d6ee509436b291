// bf16 fast path of the tiled GEMM family (paper Section II): the same instantiations as
// gemm_bf16.hpp (work-group tile BM x BN, K-step BK, wave tile WM x WN, fragment F), but the
// operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, 16 bytes per
// lane, no staging registers) one K-step ahead of the MFMAs.
//
// Preconditions (checked by the host, which otherwise launches the generic kernel):
//   16-byte aligned operands, leading dimensions and contiguous extents multiples of 8,
//   K a multiple of BK, tile-relative byte offsets below 2^31.
// Rows beyond M / N are clamped to the last valid row (the results they feed are never stored).
//
// LDS layouts
//   K-contiguous operand (A not transposed, B transposed):  tile[row][BK]; the 16-byte chunk c of
//     row r sits at chunk position c ^ swz(r) (Bf16Lds), read with ds_read_b128.
//   row-contiguous operand (A transposed, B not transposed): tile[k][ROWS] exactly as in memory;
//     32-byte units are XOR-swizzled by k.  The MFMA operand (8 consecutive k of one row per
//     lane) is produced by the transposing LDS read ds_read_b64_tr_b16: inside each group of 16
//     lanes, lane s supplies the address of 4 consecutive rows at k = kb + s/4, and lane l
//     receives the 4 values k = kb .. kb+3 of row l.
//
// A direct-to-LDS load writes LDS_base(wave-uniform) + lane * 16, i.e. one instruction fills 1 KiB
// of the tile; the swizzle is applied by choosing which global chunk each lane fetches.
#pragma once
#include <type_traits>

#include "gemm_bf16.hpp"

namespace ks {

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;

// F: fragment edge of the MFMAs that read the tile (the unit swizzle of narrow tiles depends on it)
template <int ROWS, int F = 32>
struct Bf16LdsT {
    static constexpr int CPR = ROWS / 8;                    // 16-byte chunks per k row
    static constexpr int UPR = ROWS / 16;                   // 32-byte units per k row
    // XOR applied to the 32-byte unit index of k row `k`.  A transposing read touches, per group of
    // sixteen lanes, one or two units of four consecutive k rows, and two such groups (k and k + 8
    // with 16 x 16 fragments, the next sixteen tile rows with 32 x 32 fragments) are served
    // together: bits 0, 1 and 3 of k pick the unit, so that all eight land in different banks.
    __device__ __forceinline__ static int swz(int k) {
        if constexpr (UPR >= 8) return (k & 3) | ((k >> 1) & 4);
        // narrower tiles: 16 x 16 fragments read k and k + 8 in the same pass, and a k row of 128 or
        // 64 bytes already puts k and k + 1 into different banks: the units tell k from k + 2 and
        // from k + 8.  32 x 32 fragments read two units of four consecutive k rows per pass and
        // keep the pairing that measured fastest for them (the other one cost them 5 - 20 %).
        else if constexpr (UPR == 4) return F == 16 ? ((k & 2) | ((k >> 3) & 1)) : ((k >> 1) & 3);
        else if constexpr (UPR == 2) return F == 16 ? ((k >> 3) & 1) : ((k >> 2) & 1);
        else return 0;
    }
    // byte offset of element (k, row) for row a multiple of 4
    __device__ __forceinline__ static int byte_of(int k, int row) {
        return k * (ROWS * 2) + ((((row >> 4) ^ swz(k)) << 5) | ((row & 15) << 1));
    }
};

// Per-lane source offsets of the direct-to-LDS loads of one operand tile.
template <int ROWS, int BK, int NW, bool KC, int F = 32>
struct DmaPlan {
    static constexpr int TOTAL = ROWS * BK / 512;            // 1 KiB instructions per tile
    static constexpr int PER_WAVE = (TOTAL + NW - 1) / NW;
    unsigned off[PER_WAVE];                                  // byte offset from the tile origin

    // origin: element (row0, k = 0) of the operand; limit = number of valid rows from row 0
    __device__ __forceinline__ void init(int wave, int lane, long long ld, int row0, int limit) {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int L = (wave + j * NW) * 64 + lane;       // chunk slot in the LDS tile
            if constexpr (KC) {
                constexpr int CPR = BK / 8;
                const int r = L / CPR, pos = L % CPR;
                const int c = pos ^ ((r / (16 / CPR)) & (CPR - 1));
                const int row = min(row0 + r, limit - 1) - row0;
                off[j] = (unsigned)(((long long)row * ld + c * 8) * 2);
            } else {
                constexpr int CPR = ROWS / 8;
                const int k = L / CPR, pos = L % CPR;
                const int c = pos ^ (2 * Bf16LdsT<ROWS, F>::swz(k));
                const int row = min(row0 + c * 8, limit - 8) - row0;
                off[j] = (unsigned)(((long long)k * ld + row) * 2);
            }
        }
    }

    // tile: global address of the tile origin at this K-step (wave-uniform); lds: stage base
    __device__ __forceinline__ void issue(const char *tile, char *lds, int wave) const {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int i = wave + j * NW;
            if (TOTAL % NW == 0 || i < TOTAL)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(tile + off[j]),
                    (lds_void_ptr)(lds + i * 1024), 16, 0, 0);
        }
    }
};

// vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// LDS -> registers: the MFMA operand of one fragment, i.e. for lane l the eight consecutive k
// starting at kk + 8*(l / F) of tile row rowBase + l % F.  KC tiles ([row][BK], swizzled chunks)
// need one ds_read_b128; row-contiguous tiles ([k][ROWS]) two transposing ds_read_b64_tr_b16, in
// which lane s of a 16-lane group addresses rows 4*(s%4).. of k row s/4 and lane l receives the
// four k values of row l.
template <int F, int ROWS, int BK, bool KC>
__device__ __forceinline__ bf16x8 read_fragment(const char *tile, int rowBase, int kk, int lane) {
    const int lgrp = lane / F;
    if constexpr (KC) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uintx4 *>(
            tile + 16 * Bf16Lds<BK>::chunk(rowBase + lane % F, kk / 8 + lgrp)));
    } else {
        typedef short shortx8 __attribute__((ext_vector_type(8)));
        using LT = Bf16LdsT<ROWS, F>;
        const int trRow = 4 * (lane & 3) + (F == 32 ? 16 * ((lane >> 4) & 1) : 0);
        const int kb = kk + 8 * lgrp + ((lane & 15) >> 2);
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) shortx4 *)(lds_void_ptr)(tile + LT::byte_of(kb, rowBase + trRow)));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) shortx4 *)(lds_void_ptr)(tile + LT::byte_of(kb + 4, rowBase + trRow)));
        const shortx8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    }
}

// Scheduling hint for one k-substep: NM MFMAs with NR LDS reads spread evenly between them.
template <int M, int NM, int NR>
struct InterleaveHint {
    __device__ __forceinline__ static void emit() {
        if constexpr (M < NM) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
            // all reads go behind the first NM-2 MFMAs; the last two cover the read latency
            constexpr int SLOTS = NM > 2 ? NM - 2 : 1;
            constexpr int reads = M < SLOTS ? (NR * (M + 1)) / SLOTS - (NR * M) / SLOTS : 0;
            if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);   // LDS reads
            InterleaveHint<M + 1, NM, NR>::emit();
        }
    }
};

template <int F, int BM, int BN, int BK, int WM, int WN, int STAGES, bool SPLIT, bool AKC, bool BKC,
          bool F16 = false>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_bf16_dma_kernel(const GemmParams p) {
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int FM = WM / F, FN = WN / F;
    constexpr int KSTEP = F == 32 ? 16 : 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static_assert(STAGES >= 2 && STAGES <= 4, "stages");
    // one __shared__ object per stage: the compiler can then tell that the stage being filled by
    // the in-flight loads is not the stage the ds_reads touch, and does not serialise them
    __shared__ __attribute__((aligned(1024))) char As0[A_BYTES];
    __shared__ __attribute__((aligned(1024))) char As1[A_BYTES];
    __shared__ __attribute__((aligned(1024))) char As2[STAGES > 2 ? A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char As3[STAGES > 3 ? A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char Bs0[B_BYTES];
    __shared__ __attribute__((aligned(1024))) char Bs1[B_BYTES];
    __shared__ __attribute__((aligned(1024))) char Bs2[STAGES > 2 ? B_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) char Bs3[STAGES > 3 ? B_BYTES : 16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TileCoord tc = tile_of_block(p);
    const int row0 = tc.tm * BM, col0 = tc.tn * BN;
    const int kBegin = tc.split * p.kChunk;
    const int kEnd = min(p.K, kBegin + p.kChunk);
    const int nk = (kEnd - kBegin) / BK;
    const uint16_t *Ab = static_cast<const uint16_t *>(p.A) + (long long)tc.batch * p.strideA;
    const uint16_t *Bb = static_cast<const uint16_t *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    // tile origins at k = kBegin and their advance per K-step, in bytes
    const char *aTile = reinterpret_cast<const char *>(AKC ? Ab + (long long)row0 * p.lda + kBegin
                                                            : Ab + (long long)kBegin * p.lda + row0);
    const char *bTile = reinterpret_cast<const char *>(BKC ? Bb + (long long)col0 * p.ldb + kBegin
                                                            : Bb + (long long)kBegin * p.ldb + col0);
    const long long aStep = AKC ? BK * 2LL : BK * 2LL * p.lda;
    const long long bStep = BKC ? BK * 2LL : BK * 2LL * p.ldb;

    DmaPlan<BM, BK, NW, AKC, F> pa;
    DmaPlan<BN, BK, NW, BKC, F> pb;
    pa.init(wave, lane, p.lda, row0, p.M);
    pb.init(wave, lane, p.ldb, col0, p.N);

    const int subM = (wave / (BN / WN)) * WM, subN = (wave % (BN / WN)) * WN;

    floatx4 acc16[F == 16 ? FM : 1][F == 16 ? FN : 1];
    floatx16 acc32[F == 32 ? FM : 1][F == 32 ? FN : 1];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            if constexpr (F == 16) acc16[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
            else
#pragma unroll
                for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
        }

    // LDS -> register fragments of one k-substep (KSTEP values of k) for this wave's tile
    auto load_frags = [&](const char *as, const char *bs, int kk, bf16x8 (&a)[FM], bf16x8 (&b)[FN]) {
#pragma unroll
        for (int i = 0; i < FM; ++i) a[i] = read_fragment<F, BM, BK, AKC>(as, subM + i * F, kk, lane);
#pragma unroll
        for (int j = 0; j < FN; ++j) b[j] = read_fragment<F, BN, BK, BKC>(bs, subN + j * F, kk, lane);
    };

    // One K-step on a landed stage.  The fragments of k-substep s+1 are fetched while the MFMAs of
    // substep s run (two register sets), and the scheduler is told to issue one LDS read after
    // every MFMA instead of batching reads behind a wait.
    constexpr int NSUB = BK / KSTEP;
    constexpr int NREAD = (AKC ? FM : 2 * FM) + (BKC ? FN : 2 * FN);   // LDS reads per substep
    constexpr int NMFMA = FM * FN;
    auto compute = [&](const char *as, const char *bs) {
        bf16x8 a[2][FM], b[2][FN];
        load_frags(as, bs, 0, a[0], b[0]);
        __builtin_amdgcn_sched_group_barrier(0x100, NREAD, 0);
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) {
            const int cur = sub & 1;
            if (sub + 1 < NSUB) load_frags(as, bs, (sub + 1) * KSTEP, a[cur ^ 1], b[cur ^ 1]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    if constexpr (F == 16)
                        acc16[i][j] = mfma_16x16x32<F16>(a[cur][i], b[cur][j], acc16[i][j]);
                    else
                        acc32[i][j] = mfma_32x32x16<F16>(a[cur][i], b[cur][j], acc32[i][j]);
                }
            if (sub + 1 < NSUB) InterleaveHint<0, NMFMA, NREAD>::emit();
            else InterleaveHint<0, NMFMA, 0>::emit();
        }
    };

    // Software pipeline over K-steps with a ring of STAGES LDS stages.  K-step t lives in stage
    // t % STAGES.  Before computing step t a wave waits until at most the loads of the younger
    // steps (t+1 .. t+STAGES-2) are still in flight, i.e. its own part of step t has landed; the
    // barrier then (a) publishes every wave's part of step t and (b) proves that everyone has
    // finished reading step t-1, whose stage is refilled right away with step t+STAGES-1.
    constexpr int LOADS = DmaPlan<BM, BK, NW, AKC>::PER_WAVE + DmaPlan<BN, BK, NW, BKC>::PER_WAVE;
    static_assert((STAGES - 2) * LOADS < 64, "vmcnt range");
    auto issue = [&](int t, auto stage) {
        constexpr int S = decltype(stage)::value;
        char *as = S == 0 ? As0 : S == 1 ? As1 : S == 2 ? As2 : As3;
        char *bs = S == 0 ? Bs0 : S == 1 ? Bs1 : S == 2 ? Bs2 : Bs3;
        pa.issue(aTile + t * aStep, as, wave);
        pb.issue(bTile + t * bStep, bs, wave);
    };
    auto step = [&](int t, auto stage) {
        constexpr int S = decltype(stage)::value;
        const int younger = min(nk - 1 - t, STAGES - 2);     // steps after t whose loads were issued
        if (younger >= 2) wait_vmcnt<(STAGES > 3 ? 2 : 0) * LOADS>();
        else if (younger == 1) wait_vmcnt<(STAGES > 2 ? 1 : 0) * LOADS>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (t + STAGES - 1 < nk) issue(t + STAGES - 1, std::integral_constant<int, (S + STAGES - 1) % STAGES>{});
        __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the MFMAs they overlap
        const char *as = S == 0 ? As0 : S == 1 ? As1 : S == 2 ? As2 : As3;
        const char *bs = S == 0 ? Bs0 : S == 1 ? Bs1 : S == 2 ? Bs2 : Bs3;
        // waves that are issuing MFMAs go ahead of waves that are still issuing loads or waiting
        __builtin_amdgcn_s_setprio(3);
        compute(as, bs);
        __builtin_amdgcn_s_setprio(0);
    };

    if (nk > 0) issue(0, std::integral_constant<int, 0>{});
    if (STAGES > 2 && nk > 1) issue(1, std::integral_constant<int, 1>{});
    if (STAGES > 3 && nk > 2) issue(2, std::integral_constant<int, 2>{});
    int t = 0;
    for (; t + STAGES <= nk; t += STAGES) {
        step(t, std::integral_constant<int, 0>{});
        step(t + 1, std::integral_constant<int, 1>{});
        if constexpr (STAGES > 2) step(t + 2, std::integral_constant<int, 2>{});
        if constexpr (STAGES > 3) step(t + 3, std::integral_constant<int, 3>{});
    }
    if (t < nk) step(t, std::integral_constant<int, 0>{});
    if (t + 1 < nk) step(t + 1, std::integral_constant<int, 1>{});
    if constexpr (STAGES > 2) { if (t + 2 < nk) step(t + 2, std::integral_constant<int, 2>{}); }

    if constexpr (F == 16)
        write_tile_mfma16<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc16);
    else
        write_tile_mfma32<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc32);
}

}  // namespace ks
