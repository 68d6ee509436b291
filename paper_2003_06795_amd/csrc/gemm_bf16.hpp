// bf16-input, fp32-accumulate members of the tiled GEMM family (paper Section II), MFMA only.
//
// An instantiation fixes the work-group tile BM x BN, the K-step BK (multiple of 32), the wave
// tile WM x WN and the MFMA fragment F (32: v_mfma_f32_32x32x16_bf16, 16: v_mfma_f32_16x16x32_bf16).
// Both operand tiles are staged in LDS K-contiguous, tile[row][BK], in 16-byte chunks of eight
// consecutive k, because every lane of these MFMAs consumes eight consecutive k of one row.
// Chunk positions inside a row are XOR-swizzled so that the 16 lanes of one ds_read_b128 phase,
// which read the same k-chunk of 16 consecutive rows, fall into 16 different bank groups.
//
//   AKC / BKC  operand is K-contiguous in memory (A: transA == 0, B: transB == 1): chunks are
//              copied straight through.  Otherwise an 8(k) x 8(row) block is loaded along the
//              contiguous row direction and transposed in registers before it is written.
//   VEC        16-byte global accesses are legal (alignment, leading dimension and contiguous
//              extent multiples of 8); otherwise scalar.  Every access is edge-predicated.
#pragma once
#include "ks_common.hpp"

namespace ks {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// The 16-bit members move bit patterns; only the MFMA instruction knows whether they are bf16 or
// IEEE binary16 (F16: v_mfma_f32_16x16x32_f16 / v_mfma_f32_32x32x16_f16).
template <bool F16>
__device__ __forceinline__ floatx4 mfma_16x16x32(bf16x8 a, bf16x8 b, floatx4 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
template <bool F16>
__device__ __forceinline__ floatx16 mfma_32x32x16(bf16x8 a, bf16x8 b, floatx16 c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

template <int BK>
struct Bf16Lds {
    static constexpr int CPR = BK / 8;            // 16-byte chunks per tile row
    static constexpr int RP = 16 / CPR;           // tile rows per 256 bytes of LDS
    static_assert(CPR == 4 || CPR == 8 || CPR == 16, "BK must be 32, 64 or 128");
    // index (in 16-byte units) of k-chunk c of tile row r
    __device__ __forceinline__ static int chunk(int r, int c) {
        return r * CPR + (c ^ ((r / RP) & (CPR - 1)));
    }
};

template <int ROWS, int BK, int NT, bool KC, bool VEC>
struct Bf16TileLoader {
    using L = Bf16Lds<BK>;
    static constexpr int CPR = BK / 8;
    // KC: units are chunks, INNER = CPR along k.  !KC: units are 8x8 blocks, INNER = ROWS/8 along rows.
    static constexpr int INNER = KC ? CPR : ROWS / 8;
    static constexpr int OUTER = KC ? ROWS : CPR;
    static constexpr int UNITS = INNER * OUTER;
    static constexpr int ITERS = (UNITS + NT - 1) / NT;
    static constexpr int REGS = KC ? 1 : 8;
    static_assert((INNER <= NT && NT % INNER == 0) || (INNER > NT && INNER % NT == 0), "walk");

    uintx4 reg[ITERS][REGS];

    __device__ __forceinline__ static void unit(int tid, int it, int &inner, int &outer) {
        if constexpr (INNER <= NT) {
            inner = tid % INNER;
            outer = tid / INNER + it * (NT / INNER);
        } else {
            inner = tid + (it % (INNER / NT)) * NT;
            outer = it / (INNER / NT);
        }
    }

    // eight consecutive bf16 starting at src; element e is valid while e < nValid
    __device__ __forceinline__ static uintx4 load8(const uint16_t *src, int nValid) {
        uintx4 v = {0u, 0u, 0u, 0u};
        if constexpr (VEC) {
            if (nValid > 0) v = *reinterpret_cast<const uintx4 *>(src);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                unsigned x = e < nValid ? (unsigned)src[e] : 0u;
                v[e >> 1] |= x << (16 * (e & 1));
            }
        }
        return v;
    }

    __device__ __forceinline__ void load(const uint16_t *base, long long ld, int row0, int rowLimit,
                                         int k0, int kEnd, int tid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int inner, outer;
            unit(tid, it, inner, outer);
            const bool live = UNITS % NT == 0 || outer < OUTER;
            if constexpr (KC) {
                const int r = row0 + outer, k = k0 + inner * 8;
                const int nValid = (live && r < rowLimit) ? (kEnd - k) : 0;
                reg[it][0] = load8(base + (long long)r * ld + k, nValid);
            } else {
                const int r = row0 + inner * 8;
                const int nValid = live ? (rowLimit - r) : 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = k0 + outer * 8 + j;
                    reg[it][j] = load8(base + (long long)k * ld + r, k < kEnd ? nValid : 0);
                }
            }
        }
    }

    __device__ __forceinline__ void store(uintx4 *lds, int tid) const {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int inner, outer;
            unit(tid, it, inner, outer);
            if (UNITS % NT != 0 && outer >= OUTER) continue;
            if constexpr (KC) {
                lds[L::chunk(outer, inner)] = reg[it][0];
            } else {
                // reg[it][j] holds k = 8*outer + j, rows 8*inner .. +7; emit one chunk per row
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uintx4 o;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const unsigned lo = (reg[it][2 * d][i >> 1] >> (16 * (i & 1))) & 0xffffu;
                        const unsigned hi = (reg[it][2 * d + 1][i >> 1] >> (16 * (i & 1))) & 0xffffu;
                        o[d] = lo | (hi << 16);
                    }
                    lds[L::chunk(inner * 8 + i, outer)] = o;
                }
            }
        }
    }
};

template <int F, int BM, int BN, int BK, int WM, int WN, bool SPLIT, bool AKC, bool BKC, bool VEC,
          bool F16 = false>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_bf16_kernel(const GemmParams p) {
    constexpr int NT = 64 * (BM / WM) * (BN / WN);
    constexpr int FM = WM / F, FN = WN / F;
    constexpr int KSTEP = F == 32 ? 16 : 32;          // k consumed by one MFMA
    constexpr int LGRP = F == 32 ? 2 : 4;             // lane groups along k
    using L = Bf16Lds<BK>;
    __shared__ __attribute__((aligned(16))) uintx4 As[2][BM * BK / 8];
    __shared__ __attribute__((aligned(16))) uintx4 Bs[2][BN * BK / 8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TileCoord tc = tile_of_block(p);
    const int row0 = tc.tm * BM, col0 = tc.tn * BN;
    const uint16_t *Ab = static_cast<const uint16_t *>(p.A) + (long long)tc.batch * p.strideA;
    const uint16_t *Bb = static_cast<const uint16_t *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    const int kBegin = tc.split * p.kChunk;
    const int kEnd = min(p.K, kBegin + p.kChunk);
    const int nk = (kEnd - kBegin + BK - 1) / BK;
    const int subM = (wave / (BN / WN)) * WM, subN = (wave % (BN / WN)) * WN;
    const int lrow = lane % F, lgrp = lane / F;

    Bf16TileLoader<BM, BK, NT, AKC, VEC> la;
    Bf16TileLoader<BN, BK, NT, BKC, VEC> lb;

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

    if (nk > 0) {
        la.load(Ab, p.lda, row0, p.M, kBegin, kEnd, tid);
        lb.load(Bb, p.ldb, col0, p.N, kBegin, kEnd, tid);
        la.store(As[0], tid);
        lb.store(Bs[0], tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) {
            const int k0 = kBegin + (kt + 1) * BK;
            la.load(Ab, p.lda, row0, p.M, k0, kEnd, tid);
            lb.load(Bb, p.ldb, col0, p.N, k0, kEnd, tid);
        }
        const uintx4 *as = As[cur], *bs = Bs[cur];
#pragma unroll
        for (int kk = 0; kk < BK; kk += KSTEP) {
            const int c = kk / 8 + lgrp;              // this lane's k-chunk
            bf16x8 a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                a[i] = __builtin_bit_cast(bf16x8, as[L::chunk(subM + i * F + lrow, c)]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                b[j] = __builtin_bit_cast(bf16x8, bs[L::chunk(subN + j * F + lrow, c)]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    if constexpr (F == 16)
                        acc16[i][j] = mfma_16x16x32<F16>(a[i], b[j], acc16[i][j]);
                    else
                        acc32[i][j] = mfma_32x32x16<F16>(a[i], b[j], acc32[i][j]);
                }
        }
        if (more) {
            la.store(As[cur ^ 1], tid);
            lb.store(Bs[cur ^ 1], tid);
        }
        __syncthreads();
    }
    (void)LGRP;

    if constexpr (F == 16)
        write_tile_mfma16<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc16);
    else
        write_tile_mfma32<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc32);
}

}  // namespace ks
