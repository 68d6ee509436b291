// fp32 "direct" members of the tiled GEMM family (paper Section II): small tiles for problems that
// are bound by latency and occupancy rather than by the matrix pipe.  Every wave owns a WM x WN
// tile of C made of 16x16x4 MFMA fragments and fetches its operands from global memory straight
// into the registers the MFMAs read - no LDS staging, no barrier, so the waves of a work-group
// (BM x BN = its waves' tiles side by side) never wait for each other, and the loads of K-step
// t+1 are in flight while the MFMAs of K-step t run.
//
// Operand mapping.  The 16x16x4 MFMA takes from lane l one value A[l%16][k] and one value
// B[k][l%16] with k = l/16 (four k per instruction).  A lane here holds four consecutive k,
// k0 + 4*(l/16) + j, j = 0..3, of its row (one float4 when the operand is K-contiguous in
// memory), and MFMA j of a group of four consumes element j of both operands; the sum over the
// 16 k of the group is the same set of products, in another order.
//
//   BK        k consumed per pipeline step (multiple of 16)
//   AKC/BKC   operand is K-contiguous in memory (A: transA == 0, B: transB == 1)
//   VEC       16-byte accesses are legal (see gemm_f32.hpp); otherwise scalar loads
// Rows / columns beyond M / N are clamped to the last valid one (their results are never stored);
// k beyond the end of the K range reads as zero.
#pragma once
#include "ks_common.hpp"

#ifndef KS_F32_DIRECT_SETS
// Two sets (one K-step in flight) for every tile: three and four sets were measured 1 - 5 % slower
// on the small-problem workload (more registers, fewer resident waves) and much slower for the
// 16-wave K-sliced members, whose register budget is 128 per lane.
#define KS_F32_DIRECT_SETS(regs) 2
#endif

namespace ks {

template <bool KC, bool VEC>
__device__ __forceinline__ floatx4 direct_fetch(const float *base, long long ld, int idx, int k, int kEnd) {
    floatx4 v = {0.f, 0.f, 0.f, 0.f};
    if constexpr (KC && VEC) {
        if (k < kEnd) v = *reinterpret_cast<const floatx4 *>(base + (long long)idx * ld + k);
    } else if constexpr (KC) {
        const float *src = base + (long long)idx * ld + k;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (k + j < kEnd) v[j] = src[j];
    } else {
        const float *src = base + (long long)k * ld + idx;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (k + j < kEnd) v[j] = src[(long long)j * ld];
    }
    return v;
}

// The same four values when the whole K-step is known to lie inside the K range: no predicate,
// so nothing between the loads of a step makes the wave wait for an earlier one.  `lanePtr` is the
// lane's element at k = 0 (KC: &op[idx][kLane]; otherwise &op[kLane][idx]); k is wave-uniform.
template <bool KC, bool VEC>
__device__ __forceinline__ floatx4 direct_fetch_full(const float *lanePtr, long long ld, int k) {
    floatx4 v;
    if constexpr (KC && VEC) {
        v = *reinterpret_cast<const floatx4 *>(lanePtr + k);
    } else if constexpr (KC) {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = lanePtr[k + j];
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = lanePtr[(long long)(k + j) * ld];
    }
    return v;
}

template <int BM, int BN, int BK, int WM, int WN, bool SPLIT, bool AKC, bool BKC, bool VEC>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN)) void gemm_f32_direct_kernel(const GemmParams p) {
    constexpr int FM = WM / 16, FN = WN / 16, NG = BK / 16;       // fragments per wave; k-groups per step
    static_assert(BK % 16 == 0 && WM % 16 == 0 && WN % 16 == 0, "direct core shape");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TileCoord tc = tile_of_block(p);
    const int row0 = tc.tm * BM + (wave / (BN / WN)) * WM;
    const int col0 = tc.tn * BN + (wave % (BN / WN)) * WN;
    const float *Ab = static_cast<const float *>(p.A) + (long long)tc.batch * p.strideA;
    const float *Bb = static_cast<const float *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    const int kBegin = tc.split * p.kChunk;
    const int kEnd = min(p.K, kBegin + p.kChunk);
    const int nk = (kEnd - kBegin + BK - 1) / BK;
    const int kLane = 4 * (lane >> 4);

    int rowIdx[FM], colIdx[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) rowIdx[i] = min(row0 + i * 16 + (lane & 15), p.M - 1);
#pragma unroll
    for (int j = 0; j < FN; ++j) colIdx[j] = min(col0 + j * 16 + (lane & 15), p.N - 1);

    floatx4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // register sets = K-steps in flight + the one being consumed; small sets afford more
    [[maybe_unused]] constexpr int SET_REGS = 4 * NG * (FM + FN);
    constexpr int S = KS_F32_DIRECT_SETS(SET_REGS);
    floatx4 a[S][NG][FM], b[S][NG][FN];
    // the lane's element at k = 0 of each fragment row / column, computed once
    const float *aLane[FM], *bLane[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
        aLane[i] = AKC ? Ab + (long long)rowIdx[i] * p.lda + kLane : Ab + (long long)kLane * p.lda + rowIdx[i];
#pragma unroll
    for (int j = 0; j < FN; ++j)
        bLane[j] = BKC ? Bb + (long long)colIdx[j] * p.ldb + kLane : Bb + (long long)kLane * p.ldb + colIdx[j];
    // A K-step wholly inside the range (all lanes agree) is fetched without predicates; only the
    // step that the range cuts tests every element.
    auto fetch = [&](int set, int k0) {
        if (k0 + BK <= kEnd) {
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    a[set][g][i] = direct_fetch_full<AKC, VEC>(aLane[i], p.lda, k0 + g * 16);
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    b[set][g][j] = direct_fetch_full<BKC, VEC>(bLane[j], p.ldb, k0 + g * 16);
            }
        } else {
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    a[set][g][i] = direct_fetch<AKC, VEC>(Ab, p.lda, rowIdx[i], k0 + g * 16 + kLane, kEnd);
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    b[set][g][j] = direct_fetch<BKC, VEC>(Bb, p.ldb, colIdx[j], k0 + g * 16 + kLane, kEnd);
            }
        }
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[set][g][i][e], b[set][g][j][e],
                                                                         acc[i][j], 0, 0, 0);
    };

#pragma unroll
    for (int d = 0; d < S - 1; ++d)
        if (d < nk) fetch(d, kBegin + d * BK);
    // step t lives in set t % S; while it is consumed, the set that step t - 1 left is refilled
    // with step t + S - 1
    for (int t0 = 0; t0 < nk; t0 += S) {
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const int t = t0 + u;
            if (t >= nk) break;
            if (t + S - 1 < nk) fetch((u + S - 1) % S, kBegin + (t + S - 1) * BK);
            mfmas(u);
        }
    }

    write_tile_mfma16<SPLIT, FM, FN>(p, tc, Cb, row0, col0, lane, acc);
}

}  // namespace ks
