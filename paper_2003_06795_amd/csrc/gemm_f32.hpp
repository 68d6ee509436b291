// fp32 members of the tiled GEMM family (paper Section II).
//
// One kernel template; an instantiation fixes
//   BM x BN   work-group tile of C, staged operand tiles live in LDS (double buffered)
//   BK        K-step per stage (the paper's accumulator step, at work-group granularity)
//   CORE      inner-product engine:
//               FMA     each lane owns a TM x TN register tile and does outer-product FMAs;
//                       work-group = (BM/TM) x (BN/TN) lanes  (the paper's per-work-item tile)
//               MFMA16  each wave owns WM x WN built from 16x16x4 fp32 MFMA fragments
//               MFMA32  each wave owns WM x WN built from 32x32x2 fp32 MFMA fragments
//   P1 x P2   TM x TN for FMA, WM x WN for the MFMA cores
//   SPLIT     the instantiation is a split-K member: partial sums go to the workspace
//   AKC/BKC   whether op(A)/op(B) is K-contiguous in memory (A: transA == 0, B: transB == 1);
//             decides the coalescing direction of the global loads
//   VEC       operands are 16-byte aligned with leading dimensions and contiguous extents that
//             are multiples of 4, so global accesses are float4; otherwise scalar.  Both forms
//             predicate every access against the matrix edges and zero-fill.
//
// LDS layout (both operands): tile[k][m or n] with the row padded by 4 floats.  All cores read
// "one k, many m/n", so rows of consecutive m/n are conflict-free for them.
#pragma once
#include "ks_common.hpp"

namespace ks {

// Staging-register sets (K-steps in flight) as a function of the registers one set takes and the
// work-group size.  Measured on the small-problem workload: depth 4 gains 5 - 8 % for 8-register
// sets and 2 - 3 % for 16-register sets of four-wave work-groups, but costs 2 % for the eight-wave
// 128 x 128 x 32 tile, which already has two waves per SIMD to cover the latency; odd depths lose
// (the LDS buffer of a step is then no longer fixed inside the unrolled body).
#ifndef KS_F32_PREFETCH
#define KS_F32_PREFETCH(regs, threads) \
    ((regs) <= 8 || ((regs) <= 16 && (threads) <= 256) ? 4 : (regs) <= 32 ? 2 : 1)
#endif

// Waves per SIMD the register allocation must leave room for (0 = no demand).  The multi-tile
// forms keep the next tile's staging registers alive across the epilogue; the four-wave members
// with 64 x 32 wave tiles then drift a few registers past the budget of three waves per SIMD (168
// with the accumulators) that they met before, and lose a resident work-group.
#ifndef KS_F32_MIN_WAVES
#define KS_F32_MIN_WAVES(multi, core, bm, bn, bk, p1, p2) ((multi) && ((bm) / (p1)) * ((bn) / (p2)) <= 4 ? 3 : 0)
#endif
// The balanced persistent form counts on a fixed number of resident work-groups per compute unit:
// two of eight waves (four waves per SIMD, 128 registers) or three of four waves (three per SIMD),
// which is what the plain forms of those members reach.
#ifndef KS_F32_SK_MIN_WAVES
#define KS_F32_SK_MIN_WAVES(bm, bn, p1, p2) (((bm) / (p1)) * ((bn) / (p2)) >= 8 ? 4 : 3)
#endif

// Row padding of the row-contiguous operand's LDS tile when the other operand is K-contiguous and
// both are fetched as float4 (NN and TT layouts): the padding of its partner instead of its own 4
// for the members named below.  With unequal row lengths (130 and 132 floats at BK = 32) the
// compiler keeps separate sets of fragment addresses for the two tiles, 23 - 28 registers.  The
// balanced persistent form of the 128 x 128 x 32 member does not have them inside its budget of 128
// (it spilled 13 - 14 and ran 16 % slower in NN than in NT / TN; with equal rows it needs 110), and
// the sixteen-wave 64 x 64 x 32 member on 16 x 16 wave tiles loses its second resident work-group
// (75 registers against 52).  The tile is then written with 8-byte stores, which costs elsewhere:
// measured on the NN and TT rows of the tuning set, the three members on 16 x 16 wave tiles with
// square tiles, K-step 32 and at least 512 threads gain 2.5 - 9 %, every other member is level or
// loses 1 - 9 % (among them the four-wave 64 x 64 x 32 balanced member), so only those get it.
// -1 = no override.
constexpr int f32_pad_of_partner(bool sk, int core, int bm, int bn, int p1, int p2, int kw, bool kc, bool partnerKc,
                                 bool vec, int bk, int threads) {
    const bool balancedLarge = sk && threads >= 512;
    const bool squareOn16 = core == 1 && bm == bn && p1 == 16 && p2 == 16 && bk == 32 && threads * kw >= 512;
    return (balancedLarge || squareOn16) && vec && !kc && partnerKc && bk <= 32 && (64 / bk) % 2 == 0 ? 64 / bk : -1;
}

enum { CORE_FMA = 0, CORE_MFMA16 = 1, CORE_MFMA32 = 2, CORE_DIRECT = 3, CORE_KSLICE = 4 };

template <int CORE, int BM, int BN, int P1, int P2>
struct F32Shape {
    static constexpr int threads =
        CORE == CORE_FMA ? (BM / P1) * (BN / P2) : CORE == CORE_KSLICE ? 64 * P1 * (BM / P2) * (BN / P2) : 64 * (BM / P1) * (BN / P2);
    static constexpr int frag = CORE == CORE_MFMA16 ? 16 : 32;
};

// ---- global -> registers -> LDS staging of one ROWS x BK operand tile ------------------------
// KC:  memory is [row][k] (k contiguous);  !KC: memory is [k][row] (row contiguous).
// Units are float4 (VEC) or single floats walked so that consecutive lanes touch consecutive
// addresses.  INNER = units along the contiguous direction, OUTER = the other direction.
// PAD >= 0 overrides the row padding chosen below (see f32_pad_of_partner).
template <int ROWS, int BK, int NT, bool KC, bool VEC, int PAD = -1>
struct TileLoader {
    static constexpr int W = VEC ? 4 : 1;
    static constexpr int INNER = (KC ? BK : ROWS) / W;
    static constexpr int OUTER = KC ? ROWS : BK;
    static constexpr int UNITS = INNER * OUTER;
    static constexpr int ITERS = (UNITS + NT - 1) / NT;
    // Row padding of the LDS tile.  A K-contiguous operand fetched as float4 is written as four
    // scalars to rows k .. k+3; a wave's lanes then differ in k by multiples of 4 (BK/4 lanes)
    // and in the row, and land in 64 different banks when 4 * LDS_LD = 256/BK (mod 64), i.e. a
    // padding of 64/BK floats.  The other forms write along a row and take the padding of 4 that
    // keeps their 16-byte writes aligned.  (Measured: bank-conflict cycles of the 128 x 128 x 32
    // member fell to a third and the BK = 32 / 64 members gained 2 - 20 % on long K; giving the
    // lane groups of an MFMA read rows 4 or 8 apart instead of adjacent ones changed nothing.)
    static constexpr int LDS_LD = ROWS + (PAD >= 0 ? PAD : (KC && VEC) ? (BK >= 64 ? 1 : 64 / BK) : 4);
    static_assert(!(VEC && !KC) || LDS_LD % 2 == 0, "row-contiguous vector writes need 8-byte alignment");
    static_assert((INNER <= NT && NT % INNER == 0) || (INNER > NT && INNER % NT == 0), "walk");

    float reg[ITERS][W];

    __device__ __forceinline__ static void unit(int tid, int it, int &inner, int &outer) {
        if constexpr (INNER <= NT) {
            inner = tid % INNER;
            outer = tid / INNER + it * (NT / INNER);
        } else {
            inner = tid + (it % (INNER / NT)) * NT;
            outer = it / (INNER / NT);
        }
    }

    // rowLimit: number of valid rows from row0 on; k runs from k0, valid while < kEnd.
    __device__ __forceinline__ void load(const float *base, long long ld, int row0, int rowLimit,
                                         int k0, int kEnd, int tid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int inner, outer;
            unit(tid, it, inner, outer);
            const int r = KC ? outer : inner * W;
            const int k = KC ? inner * W : outer;
            const bool ok = (UNITS % NT == 0 || outer < OUTER) && (row0 + r < rowLimit) && (k0 + k < kEnd);
            const float *src = KC ? base + (long long)(row0 + r) * ld + (k0 + k)
                                  : base + (long long)(k0 + k) * ld + (row0 + r);
            if constexpr (VEC) {
                floatx4 v = {0.f, 0.f, 0.f, 0.f};
                if (ok) v = *reinterpret_cast<const floatx4 *>(src);
                reg[it][0] = v.x; reg[it][1] = v.y; reg[it][2] = v.z; reg[it][3] = v.w;
            } else {
                reg[it][0] = ok ? *src : 0.f;
            }
        }
    }

    __device__ __forceinline__ void store(float *lds, int tid) const {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int inner, outer;
            unit(tid, it, inner, outer);
            if (UNITS % NT != 0 && outer >= OUTER) continue;
            const int r = KC ? outer : inner * W;
            const int k = KC ? inner * W : outer;
            if constexpr (VEC && !KC && LDS_LD % 4 == 0) {
                floatx4 v = {reg[it][0], reg[it][1], reg[it][2], reg[it][3]};
                *reinterpret_cast<floatx4 *>(lds + k * LDS_LD + r) = v;
            } else if constexpr (VEC && !KC) {
                typedef float floatx2 __attribute__((ext_vector_type(2)));
                floatx2 *dst = reinterpret_cast<floatx2 *>(lds + k * LDS_LD + r);
                dst[0] = floatx2{reg[it][0], reg[it][1]};
                dst[1] = floatx2{reg[it][2], reg[it][3]};
            } else if constexpr (VEC) {
#pragma unroll
                for (int j = 0; j < 4; ++j) lds[(k + j) * LDS_LD + r] = reg[it][j];
            } else {
                lds[k * LDS_LD + r] = reg[it][0];
            }
        }
    }
};

// KW > 1 (MFMA cores): the work-group holds KW groups of waves, each a complete copy of the
// BM x BN wave arrangement with its own LDS stages, and each takes one slice of the work-group's
// K range (rounded to whole K-steps).  The groups run the same number of K-steps in lock-step (a
// short slice pads with zero tiles), then add their accumulators through LDS in group order.
// More waves per compute unit for the same number of tiles, without a workspace.
//
// MULTI (members for which f32_multi_tile holds, never split-K): the work-group walks
// GemmParams::tilesPerWG consecutive logical tiles.  The single-tile form of the same member is a
// separate instantiation: the flattened loop costs it about 6 % on ordinary shapes.
//
// SK (32x32 MFMA members, single K group, never split-K): the balanced persistent form.  The launch
// holds a fixed number of work-groups (a few per compute unit, all resident at once).  Each first
// computes GemmParams::skRounds whole tiles, then an equal share of the K-steps of the tiles that
// are left over when the tile count is not a multiple of the work-group count: those tiles are
// flattened into one sequence of (tile, K-step) units and cut into contiguous shares, so every
// compute unit gets the same number of K-steps however unevenly the tiles divide.  A share that
// covers a whole tile is written to C as usual; a share that covers part of a tile goes to the
// workspace as a raw accumulator tile (at most two per work-group: the head and the tail of its
// share), and gemm_f32_sk_fixup_kernel adds the parts of every divided tile in K order and applies
// the epilogue.  No work-group waits for another, so there is nothing to deadlock on.
template <int CORE, int BM, int BN, int BK, int P1, int P2, bool SPLIT, bool AKC, bool BKC, bool VEC,
          int KW = 1, bool MULTI = false, bool SK = false>
__global__ __launch_bounds__((F32Shape<CORE, BM, BN, P1, P2>::threads * KW), (SK ? KS_F32_SK_MIN_WAVES(BM, BN, P1, P2) : KS_F32_MIN_WAVES(MULTI, CORE, BM, BN, BK, P1, P2))) void gemm_f32_kernel(
    const GemmParams p) {
    static_assert(!MULTI || (f32_multi_tile(CORE, BM, BN, P1, P2, KW) && !SPLIT), "multi-tile form");
    static_assert(!SK || (CORE == CORE_MFMA32 && KW == 1 && !SPLIT && !MULTI), "balanced persistent form");
    using Shape = F32Shape<CORE, BM, BN, P1, P2>;
    constexpr int NT = Shape::threads;                        // threads of one group
    static_assert(KW == 1 || CORE != CORE_FMA, "K groups need an MFMA core");
    constexpr int PADA = f32_pad_of_partner(SK, CORE, BM, BN, P1, P2, KW, AKC, BKC, VEC, BK, NT);
    constexpr int PADB = f32_pad_of_partner(SK, CORE, BM, BN, P1, P2, KW, BKC, AKC, VEC, BK, NT);
    constexpr int LDA = TileLoader<BM, BK, NT, AKC, VEC, PADA>::LDS_LD, LDB = TileLoader<BN, BK, NT, BKC, VEC, PADB>::LDS_LD;
    __shared__ __attribute__((aligned(16))) float AsAll[KW][2][BK * LDA];
    __shared__ __attribute__((aligned(16))) float BsAll[KW][2][BK * LDB];

    const int grp = KW == 1 ? 0 : (int)threadIdx.x / NT;
    const int tid = KW == 1 ? (int)threadIdx.x : (int)threadIdx.x % NT;
    float (*As)[BK * LDA] = AsAll[grp];
    float (*Bs)[BK * LDB] = BsAll[grp];
    // the (first) tile of this work-group
    const TileCoord tc = MULTI && !p.grid3d ? tile_of_logical(p, logical_of_block() * (unsigned)p.tilesPerWG)
                                            : tile_of_block(p);
    const int row0 = tc.tm * BM, col0 = tc.tn * BN;
    const float *Ab = static_cast<const float *>(p.A) + (long long)tc.batch * p.strideA;
    const float *Bb = static_cast<const float *>(p.B) + (long long)tc.batch * p.strideB;
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    const int kLo = tc.split * p.kChunk, kHi = min(p.K, kLo + p.kChunk);
    const int slice = KW == 1 ? p.kChunk : ((((kHi - kLo) + KW - 1) / KW + BK - 1) / BK) * BK;
    const int kBegin = kLo + grp * slice;
    const int kEnd = min(kHi, kBegin + slice);               // may lie below kBegin: an empty slice
    const int nk = (min(slice, kHi - kLo) + BK - 1) / BK;     // steps of the longest slice, for all groups

    // K-steps in flight between global memory and LDS (each in its own set of staging registers):
    // small tiles are latency-bound - few waves per compute unit, short MFMA runs per K-step - and
    // afford several; large tiles hide the latency behind their MFMAs and keep the registers.
    using LoaderA = TileLoader<BM, BK, NT, AKC, VEC, PADA>;
    using LoaderB = TileLoader<BN, BK, NT, BKC, VEC, PADB>;
    constexpr int STAGE_REGS = (LoaderA::ITERS + LoaderB::ITERS) * LoaderA::W;
    constexpr int PF = KS_F32_PREFETCH(STAGE_REGS, NT);
    LoaderA la[PF];
    LoaderB lb[PF];

    // accumulators
    constexpr int FR = Shape::frag;
    constexpr int FM = CORE == CORE_FMA ? 1 : P1 / FR, FN = CORE == CORE_FMA ? 1 : P2 / FR;
    float accF[CORE == CORE_FMA ? P1 : 1][CORE == CORE_FMA ? P2 : 1];
    floatx4 acc16[CORE == CORE_MFMA16 ? FM : 1][CORE == CORE_MFMA16 ? FN : 1];
    floatx16 acc32[CORE == CORE_MFMA32 ? FM : 1][CORE == CORE_MFMA32 ? FN : 1];
    if constexpr (CORE == CORE_FMA) {
#pragma unroll
        for (int i = 0; i < P1; ++i)
#pragma unroll
            for (int j = 0; j < P2; ++j) accF[i][j] = 0.f;
    } else if constexpr (CORE == CORE_MFMA16) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) acc16[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    } else {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
    }

    // lane -> sub-tile origin inside the work-group tile
    const int lane = tid & 63, wave = tid >> 6;
    int subM, subN;
    if constexpr (CORE == CORE_FMA) {
        subM = (tid / (BN / P2)) * P1;
        subN = (tid % (BN / P2)) * P2;
    } else {
        subM = (wave / (BN / P2)) * P1;
        subN = (wave % (BN / P2)) * P2;
    }

    // one K-step of MFMAs / FMAs on a landed LDS stage
    auto compute_step = [&](const float *as, const float *bs) {
        if constexpr (CORE == CORE_FMA) {
#pragma unroll
            for (int kk = 0; kk < BK; ++kk) {
                float a[P1], b[P2];
#pragma unroll
                for (int i = 0; i < P1; ++i) a[i] = as[kk * LDA + subM + i];
#pragma unroll
                for (int j = 0; j < P2; ++j) b[j] = bs[kk * LDB + subN + j];
#pragma unroll
                for (int i = 0; i < P1; ++i)
#pragma unroll
                    for (int j = 0; j < P2; ++j) accF[i][j] = fmaf(a[i], b[j], accF[i][j]);
            }
        } else if constexpr (CORE == CORE_MFMA16) {
            // 16x16x4: lane l feeds A[l%16][l/16] and B[l/16][l%16]
#pragma unroll
            for (int kk = 0; kk < BK; kk += 4) {
                const int kr = kk + (lane >> 4);
                float a[FM], b[FN];
#pragma unroll
                for (int i = 0; i < FM; ++i) a[i] = as[kr * LDA + subM + i * 16 + (lane & 15)];
#pragma unroll
                for (int j = 0; j < FN; ++j) b[j] = bs[kr * LDB + subN + j * 16 + (lane & 15)];
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc16[i][j], 0, 0, 0);
            }
        } else {
            // 32x32x2: lane l feeds A[l%32][l/32] and B[l/32][l%32]
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                const int kr = kk + (lane >> 5);
                float a[FM], b[FN];
#pragma unroll
                for (int i = 0; i < FM; ++i) a[i] = as[kr * LDA + subM + i * 32 + (lane & 31)];
#pragma unroll
                for (int j = 0; j < FN; ++j) b[j] = bs[kr * LDB + subN + j * 32 + (lane & 31)];
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc32[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc32[i][j], 0, 0, 0);
            }
        }
    };

    if constexpr (MULTI) {
        // The work-group walks nTiles consecutive logical tiles as ONE sequence of K-steps: the
        // loads run PF steps ahead of the MFMAs across tile boundaries, so the first steps of the
        // next tile are requested before the finished tile's C is stored (the vector memory path
        // of a compute unit is in order: loads issued behind 64 KB of stores to a busy HBM wait
        // for them), and tiles after the first pay no work-group launch and no pipeline fill.
        // All tiles of a launch with tilesPerWG > 1 share one K range (the host grants it only
        // without split-K); a range without steps still runs one step of zero tiles.
        unsigned firstTile = 0;
        int nTiles = 1;
        if (!p.grid3d) {
            const unsigned total = (unsigned)p.tilesM * (unsigned)p.tilesN * (unsigned)(p.batch * p.splitK);
            firstTile = logical_of_block() * (unsigned)p.tilesPerWG;
            nTiles = (int)min((unsigned)p.tilesPerWG, total - firstTile);
        }
        const int nkT = max(nk, 1);
        const int G = nTiles * nkT;
        // load stream
        TileCoord tcL = tc;
        int iL = 0, kL = 0, rowL = row0, colL = col0;
        const float *AbL = Ab, *BbL = Bb;
        auto issue_load = [&](LoaderA &a, LoaderB &b) {
            a.load(AbL, p.lda, rowL, p.M, kBegin + kL * BK, kEnd, tid);
            b.load(BbL, p.ldb, colL, p.N, kBegin + kL * BK, kEnd, tid);
            if (++kL == nkT) {
                kL = 0;
                if (++iL < nTiles) {
                    tcL = tile_of_logical(p, firstTile + (unsigned)iL);
                    rowL = tcL.tm * BM; colL = tcL.tn * BN;
                    AbL = static_cast<const float *>(p.A) + (long long)tcL.batch * p.strideA;
                    BbL = static_cast<const float *>(p.B) + (long long)tcL.batch * p.strideB;
                }
            }
        };
        // compute stream
        TileCoord tcC = tc;
        int iC = 0, kC = 0;
#pragma unroll
        for (int d = 0; d < PF; ++d)
            if (d < G) issue_load(la[d], lb[d]);
        la[0].store(As[0], tid);
        lb[0].store(Bs[0], tid);
        __syncthreads();
        for (int g0 = 0; g0 < G; g0 += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int g = g0 + u;
                if (g >= G) break;
                const int cur = g & 1;
                if (g + PF < G) issue_load(la[u], lb[u]);
                compute_step(As[cur], Bs[cur]);
                if (g + 1 < G) {
                    la[(u + 1) % PF].store(As[cur ^ 1], tid);
                    lb[(u + 1) % PF].store(Bs[cur ^ 1], tid);
                }
                if (++kC == nkT) {
                    kC = 0;
                    float *Cc = p.C + (long long)tcC.batch * p.strideC;
                    write_tile_mfma32_lean<SPLIT, FM, FN>(p, tcC, Cc, tcC.tm * BM + subM, tcC.tn * BN + subN, lane, acc32);
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
                    if (++iC < nTiles) tcC = tile_of_logical(p, firstTile + (unsigned)iC);
                }
                __syncthreads();
            }
        }
        return;
    }

    if constexpr (SK) {
        // Everything that describes the share is the same for all lanes; the integer divisions run
        // on the vector unit, so their results are moved to scalar registers explicitly.
        auto uni = [](long long v) -> long long {
            const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)v);
            const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)v >> 32));
            return (long long)(((unsigned long long)hi << 32) | lo);
        };
        const unsigned lw = (unsigned)__builtin_amdgcn_readfirstlane((int)logical_of_block());
        const long long groups = (long long)gridDim.x;
        const int nkT = (p.K + BK - 1) / BK;
        const long long units = (long long)p.skTailTiles * nkT;
        const long long ub = uni(sk_share_begin(lw, units, groups)), ue = uni(sk_share_begin(lw + 1, units, groups));
        const long long t0 = uni(ub / nkT);                  // first left-over tile of the share
        const int r0 = (int)(ub - t0 * nkT);                  // and the K-step it starts at
        const int tailSegs = ue > ub ? (int)(uni((ue - 1) / nkT) - t0) + 1 : 0;
        const int nSeg = p.skRounds + tailSegs;
        for (int sg = 0; sg < nSeg; ++sg) {
            unsigned logical;
            int ks0 = 0, ks1 = nkT;
            if (sg < p.skRounds) {
                logical = (unsigned)sg * (unsigned)groups + lw;
            } else {
                const long long t = t0 + (sg - p.skRounds);
                logical = (unsigned)p.skRounds * (unsigned)groups + (unsigned)t;
                ks0 = sg == p.skRounds ? r0 : 0;
                ks1 = (int)min((long long)nkT, ue - t * nkT);
            }
            TileCoord tcS = tile_of_logical(p, logical);
            tcS.batch = __builtin_amdgcn_readfirstlane(tcS.batch);
            tcS.tm = __builtin_amdgcn_readfirstlane(tcS.tm);
            tcS.tn = __builtin_amdgcn_readfirstlane(tcS.tn);
            tcS.split = 0;
            const int rowS = tcS.tm * BM, colS = tcS.tn * BN;
            const float *AbS = static_cast<const float *>(p.A) + (long long)tcS.batch * p.strideA;
            const float *BbS = static_cast<const float *>(p.B) + (long long)tcS.batch * p.strideB;
            const int kB = ks0 * BK, kE = min(p.K, ks1 * BK), nkS = ks1 - ks0;
            // every staging set is (re)defined here, so none stays alive across the epilogue of the
            // previous tile; steps past the end of the range are zero tiles that touch no memory
#pragma unroll
            for (int d = 0; d < PF; ++d) {
                la[d].load(AbS, p.lda, rowS, p.M, kB + d * BK, kE, tid);
                lb[d].load(BbS, p.ldb, colS, p.N, kB + d * BK, kE, tid);
            }
            la[0].store(As[0], tid);
            lb[0].store(Bs[0], tid);
            __syncthreads();
            for (int kt0 = 0; kt0 < nkS; kt0 += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int kt = kt0 + u;
                    if (kt >= nkS) break;
                    const int cur = kt & 1;
                    if (kt + PF < nkS) {
                        const int k0 = kB + (kt + PF) * BK;
                        la[u].load(AbS, p.lda, rowS, p.M, k0, kE, tid);
                        lb[u].load(BbS, p.ldb, colS, p.N, k0, kE, tid);
                    }
                    compute_step(As[cur], Bs[cur]);
                    if (kt + 1 < nkS) {
                        la[(u + 1) % PF].store(As[cur ^ 1], tid);
                        lb[(u + 1) % PF].store(Bs[cur ^ 1], tid);
                    }
                    __syncthreads();
                }
            }
            // the lane's output offsets are recomputed for every tile (the compiler would otherwise
            // keep them in registers across the K loop, which has none to spare)
            int laneE = lane;
            asm volatile("" : "+v"(laneE));
            if (ks0 == 0 && ks1 == nkT) {
                float *CbS = p.C + (long long)tcS.batch * p.strideC;
                write_tile_mfma32<false, FM, FN>(p, tcS, CbS, rowS + subM, colS + subN, laneE, acc32);
            } else {
                // raw accumulators, in register order: float4 unit (wave, i, j, chunk) of lane l
                floatx4 *part = reinterpret_cast<floatx4 *>(p.ws) +
                                ((long long)lw * 2 + (sg == p.skRounds ? 0 : 1)) * (BM * BN / 4);
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            part[(((wave * FM + i) * FN + j) * 4 + c) * 64 + laneE] =
                                floatx4{acc32[i][j][4 * c], acc32[i][j][4 * c + 1], acc32[i][j][4 * c + 2],
                                        acc32[i][j][4 * c + 3]};
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
        }
        return;
    }

#pragma unroll
    for (int d = 0; d < PF; ++d)
        if (d < nk) {
            la[d].load(Ab, p.lda, row0, p.M, kBegin + d * BK, kEnd, tid);
            lb[d].load(Bb, p.ldb, col0, p.N, kBegin + d * BK, kEnd, tid);
        }
    if (nk > 0) {
        la[0].store(As[0], tid);
        lb[0].store(Bs[0], tid);
    }
    __syncthreads();

    // K-step kt sits in LDS buffer kt & 1 and came through staging set kt % PF; while it is being
    // consumed, that set is refilled with step kt + PF and step kt + 1 moves from its set to LDS.
    for (int kt0 = 0; kt0 < nk; kt0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int kt = kt0 + u;
            if (kt >= nk) break;
            const int cur = kt & 1;
            if (kt + PF < nk) {
                const int k0 = kBegin + (kt + PF) * BK;
                la[u].load(Ab, p.lda, row0, p.M, k0, kEnd, tid);
                lb[u].load(Bb, p.ldb, col0, p.N, k0, kEnd, tid);
            }
            const float *as = As[cur], *bs = Bs[cur];
            compute_step(as, bs);
            if (kt + 1 < nk) {
                la[(u + 1) % PF].store(As[cur ^ 1], tid);
                lb[(u + 1) % PF].store(Bs[cur ^ 1], tid);
            }
            __syncthreads();
        }
    }

    // epilogue
    if constexpr (CORE == CORE_FMA) {
        write_tile<SPLIT>(p, tc, Cb, [&](auto emit) {
#pragma unroll
            for (int i = 0; i < P1; ++i)
#pragma unroll
                for (int j = 0; j < P2; ++j) emit(row0 + subM + i, col0 + subN + j, accF[i][j]);
        });
    } else if constexpr (KW > 1) {
        // every wave publishes its accumulators as float4 units [group][wave][i][j][chunk][lane];
        // the units are then dealt out over all threads, summed in group order and stored
        constexpr int CH = CORE == CORE_MFMA32 ? 4 : 1;       // float4 chunks per fragment and lane
        constexpr int FRG = CORE == CORE_MFMA32 ? 32 : 16;
        constexpr int UNITS = (NT / 64) * FM * FN * CH * 64;
        __shared__ floatx4 part[KW][UNITS];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int base = (((wave * FM + i) * FN + j) * CH) * 64 + lane;
                if constexpr (CORE == CORE_MFMA16) {
                    part[grp][base] = acc16[i][j];
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        part[grp][base + c * 64] = floatx4{acc32[i][j][4 * c], acc32[i][j][4 * c + 1],
                                                           acc32[i][j][4 * c + 2], acc32[i][j][4 * c + 3]};
                }
            }
        __syncthreads();
        const OutTarget o = out_target<SPLIT>(p, tc, Cb);
        for (int u = (int)threadIdx.x; u < UNITS; u += NT * KW) {
            floatx4 sum = part[0][u];
#pragma unroll
            for (int g = 1; g < KW; ++g) sum += part[g][u];
            const int ul = u & 63;
            int q = __builtin_amdgcn_readfirstlane(u >> 6);
            const int c = q % CH; q /= CH;
            const int j = q % FN; q /= FN;
            const int i = q % FM;
            const int w = q / FM;
            const int fr0 = row0 + (w / (BN / P2)) * P1 + i * FRG, fc0 = col0 + (w % (BN / P2)) * P2 + j * FRG;
            const bool full = fr0 + FRG <= o.M && fc0 + FRG <= o.N;
            const float v[4] = {sum[0], sum[1], sum[2], sum[3]};
            if constexpr (CORE == CORE_MFMA16)
                store_lane_column<SPLIT, 4>(o, fr0 + 4 * (ul >> 4), fc0 + (ul & 15), full, v, [](int e) { return e; });
            else
                store_lane_column<SPLIT, 4>(o, fr0 + 8 * c + 4 * (ul >> 5), fc0 + (ul & 31), full, v,
                                            [](int e) { return e; });
        }
    } else if constexpr (CORE == CORE_MFMA16) {
        write_tile_mfma16<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc16);
    } else {
        write_tile_mfma32<SPLIT, FM, FN>(p, tc, Cb, row0 + subM, col0 + subN, lane, acc32);
    }
}

// Second kernel of the balanced persistent form: one single-wave work-group per left-over tile and
// wave tile (blockIdx.x = tile, blockIdx.y = wave of the first kernel's work-group).  A tile that
// one share covered whole was written by the first kernel and is skipped; for a divided tile the
// raw accumulator tiles of its shares are added in K order (ascending work-group, a fixed order:
// results are reproducible) and stored through the usual epilogue.  Lanes map to accumulator
// elements exactly as in gemm_f32_kernel.
template <int BM, int BN, int BK, int P1, int P2>
__global__ __launch_bounds__(64) void gemm_f32_sk_fixup_kernel(const GemmParams p) {
    constexpr int FM = P1 / 32, FN = P2 / 32;
    const long long groups = p.skGroups;
    const int nkT = (p.K + BK - 1) / BK;
    const long long units = (long long)p.skTailTiles * nkT;
    const long long t = blockIdx.x, u0 = t * nkT, u1 = u0 + nkT;
    // first work-group whose share reaches into this tile
    long long w = (u0 * groups) / units;
    while (w > 0 && sk_share_begin(w, units, groups) > u0) --w;
    while (sk_share_begin(w + 1, units, groups) <= u0) ++w;
    if (sk_share_begin(w, units, groups) <= u0 && sk_share_begin(w + 1, units, groups) >= u1) return;

    const int lane = (int)threadIdx.x, wave = (int)blockIdx.y;
    floatx16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    // the parts are fetched four shares at a time (all loads of a batch are independent) and
    // added in share order
    constexpr int PB = 4;
    bool more = true;
    do {
        const floatx4 *part[PB];
        bool have[PB];
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            have[q] = false;
            part[q] = nullptr;
            while (more) {
                if (w >= groups) { more = false; break; }
                const long long b = sk_share_begin(w, units, groups), e = sk_share_begin(w + 1, units, groups);
                if (b >= u1) { more = false; break; }
                const long long cur = w++;
                if (e <= b) continue;                        // an empty share wrote nothing
                part[q] = reinterpret_cast<const floatx4 *>(p.ws) + (cur * 2 + (b / nkT == t ? 0 : 1)) * (BM * BN / 4) +
                          (long long)wave * (FM * FN * 4 * 64) + lane;
                have[q] = true;
                break;
            }
        }
        floatx4 v[PB][FM * FN * 4];
#pragma unroll
        for (int q = 0; q < PB; ++q)
            if (have[q]) {
#pragma unroll
                for (int f = 0; f < FM * FN * 4; ++f) v[q][f] = part[q][f * 64];
            }
#pragma unroll
        for (int q = 0; q < PB; ++q)
            if (have[q]) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
#pragma unroll
                            for (int x = 0; x < 4; ++x) acc[i][j][4 * c + x] += v[q][(i * FN + j) * 4 + c][x];
            }
    } while (more);
    const TileCoord tc = tile_of_logical(p, (unsigned)p.skRounds * (unsigned)groups + (unsigned)t);
    float *Cb = p.C + (long long)tc.batch * p.strideC;
    const int subM = (wave / (BN / P2)) * P1, subN = (wave % (BN / P2)) * P2;
    write_tile_mfma32<false, FM, FN>(p, tc, Cb, tc.tm * BM + subM, tc.tn * BN + subN, lane, acc);
}

}  // namespace ks
