// fp32 "K-sliced" members of the tiled GEMM family (paper Section II): one BM x BN tile of C per
// work-group, made of W x W wave tiles, and the K range of the work-group cut into KW slices; a
// wave owns one wave tile on one slice (work-group = KW * (BM/W) * (BN/W) waves).  Every wave
// runs the register-fed 16x16x4 MFMA pipeline of gemm_f32_direct.hpp on its slice, so a small
// problem with a long K - a latency chain of K / BK dependent steps in the other members - becomes
// KW chains that are KW times shorter and run side by side.  The partial tiles meet in LDS and
// are added in slice order 0 .. KW-1 (the same order every time), then scaled and stored once:
// no workspace and no second kernel, unlike the split-K members that partition K over
// work-groups.  Both forms of splitting combine (SPLIT: this work-group's K range is one of
// p.splitK partitions and its tile goes to the workspace).
//
// Slice length: the K range divided by KW, rounded up to a multiple of 16 (one group of four
// 16x16x4 MFMAs, and a whole number of 16-byte accesses); trailing slices may be empty.
#pragma once
#include "gemm_f32_direct.hpp"

namespace ks {

template <int BM, int BN, int BK, int KW, int W, bool SPLIT, bool AKC, bool BKC, bool VEC>
__global__ __launch_bounds__(64 * KW * (BM / W) * (BN / W)) void gemm_f32_kslice_kernel(const GemmParams p) {
    constexpr int FM = W / 16, FN = W / 16, NG = BK / 16;
    constexpr int TW = (BM / W) * (BN / W);                   // wave tiles per work-group tile
    constexpr int NF = TW * FM * FN;                          // 16x16 fragments per work-group tile
    static_assert(BK % 16 == 0 && W % 16 == 0 && BM % W == 0 && BN % W == 0 && KW >= 2 && KW * TW <= 16,
                  "k-slice shape");
    __shared__ floatx4 part[KW][NF][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) / TW, tw = (tid >> 6) % TW;
    const TileCoord tc = tile_of_block(p);
    const int row0 = tc.tm * BM + (tw / (BN / W)) * W, col0 = tc.tn * BN + (tw % (BN / W)) * W;
    const float *Ab = static_cast<const float *>(p.A) + (long long)tc.batch * p.strideA;
    const float *Bb = static_cast<const float *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    const int kLo = tc.split * p.kChunk;
    const int kHi = min(p.K, kLo + p.kChunk);
    const int slice = (((kHi - kLo + KW - 1) / KW) + 15) & ~15;
    const int kBegin = kLo + wave * slice;
    const int kEnd = min(kHi, kBegin + slice);
    const int nk = kEnd > kBegin ? (kEnd - kBegin + BK - 1) / BK : 0;
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

    // every wave publishes its partial wave tile; the fragments of the work-group tile are then
    // dealt out over all waves, each summed over the slices in order and stored
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) part[wave][(tw * FM + i) * FN + j][lane] = acc[i][j];
    __syncthreads();
    const int tileRow = tc.tm * BM, tileCol = tc.tn * BN;
#pragma unroll
    for (int f0 = 0; f0 < NF; f0 += KW * TW) {
        const int f = f0 + (tid >> 6);
        if (f < NF) {
            floatx4 sum[1][1];
            sum[0][0] = part[0][f][lane];
#pragma unroll
            for (int s = 1; s < KW; ++s) sum[0][0] += part[s][f][lane];
            const int t = f / (FM * FN), i = (f / FN) % FM, j = f % FN;
            write_tile_mfma16<SPLIT, 1, 1>(p, tc, Cb, tileRow + (t / (BN / W)) * W + i * 16,
                                           tileCol + (t % (BN / W)) * W + j * 16, lane, sum);
        }
    }
}

}  // namespace ks
