// Shared device-side pieces of the tiled GEMM family (paper Section II): launch parameters,
// work-group -> tile mapping, and the alpha/beta epilogue.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ks {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmParams {
    const void *A;
    const void *B;
    float *C;
    float *ws;                       // split-K partial sums: [split][batch][M][N], dense
    const float *bias;               // N values added to every row of C after alpha / beta, or null
    long long lda, ldb, ldc;
    long long strideA, strideB, strideC;
    int M, N, K, batch;
    int tilesM, tilesN;
    int splitK, kChunk;              // K range of split s is [s*kChunk, min(K, (s+1)*kChunk))
    int grid3d;                      // 1: launched as (tilesN, tilesM, batch*splitK) work-groups
    int tilesPerWG;                  // consecutive logical tiles one work-group walks (members that
                                     // support it; 1 everywhere else and on 3-D launches)
    int bandRows;                    // tile rows per band of the one-dimensional tile order (8 unless the
                                     // member says otherwise)
    int out16;                       // 1: C holds bf16 (2-byte elements; ldc in elements); strideC is
                                     //    then 0 and the batch stride, in elements, is strideC16
    long long strideC16;
    float alpha, beta;
    // balanced persistent form (fp32 members that have one; 0 everywhere else): the launch holds
    // skGroups work-groups; each computes skRounds whole tiles (logical tiles round * skGroups + its
    // own logical id) and then an equal share of the K-steps of the skTailTiles tiles that are left
    int skGroups, skRounds, skTailTiles;
    // a launch over part of the tiles (the split tail of a hybrid launch, see dispatch.hip): logical
    // ids 0 .. tileSpan * splitK - 1 stand for the tiles tileBase .. tileBase + tileSpan - 1 of the
    // one-dimensional order, partition-major, and partial sums go to the workspace as compact
    // bm x bn tiles [partition][tile - tileBase].  tileSpan == 0 everywhere else.
    int tileBase, tileSpan, bm, bn;
};

// K-steps [first, last) of the left-over tiles (flattened as tile * steps-per-tile + step) that
// work-group `w` of `groups` computes in the balanced persistent form; shares differ by at most one
__host__ __device__ inline long long sk_share_begin(long long w, long long units, long long groups) {
    return (w * units) / groups;
}

// bf16 <-> fp32 for an output kept in bf16: widening is exact, narrowing rounds to nearest even
// (NaN stays NaN)
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __builtin_bit_cast(float, (unsigned)b << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
// C[idx] = alpha * acc + beta * C[idx] + bias with C in bf16 (element index idx from the batch
// item's origin)
__device__ __forceinline__ void store_bf16_out(float *Cb, long long idx, float acc, float alpha, float beta,
                                               float biasv) {
    uint16_t *c = reinterpret_cast<uint16_t *>(Cb) + idx;
    float x = alpha * acc;
    if (beta != 0.0f) x = fmaf(beta, bf16_bits_to_float(*c), x);
    *c = float_to_bf16_bits(x + biasv);
}

// fp32 LDS-staged members that also exist in a form whose work-groups walk several tiles
// (GemmParams::tilesPerWG): 32x32 MFMA members (core 2) with large tiles of at least 128 columns
// (the 128 x 64 member measured slower in that form), wave tiles of at most 2048 entries (the form
// holds staging registers across the epilogue) and a single K group.
constexpr bool f32_multi_tile(int core, int bm, int bn, int p1, int p2, int kw) {
    return core == 2 && bm * bn >= 8192 && bn >= 128 && p1 * p2 <= 2048 && kw == 1;
}

// 16-bit members whose direct-to-LDS path runs in the form with two groups of waves alternating
// between memory and MFMA slots: the eight-wave 256 x 256 x 64 members (128 x 64 of output per wave)
// with either fragment shape, and the eight-wave 128 x 128 x 128 members on 16x16x32 fragments
// (64 x 32 of output per wave).
constexpr bool bf16_two_groups(int f, int bm, int bn, int bk, int wm, int wn, int stages) {
    return ((f == 32 || f == 16) && bm == 256 && bn == 256 && bk == 64 && wm == 128 && wn == 64 && stages == 2) ||
           (f == 16 && bm == 128 && bn == 128 && bk == 128 && wm == 64 && wn == 32 && stages == 2);
}

// launch shape that tile_of_block expects
inline dim3 launch_grid(const GemmParams &p, int grid) {
    return p.grid3d ? dim3((unsigned)p.tilesN, (unsigned)p.tilesM, (unsigned)(p.batch * p.splitK))
                    : dim3((unsigned)grid);
}

struct TileCoord {
    int batch, split, tm, tn;
};

// MI355X has 8 XCDs with private L2s and hands consecutive work-group ids to them round-robin.
// Renumber so that each XCD owns one contiguous run of logical tile ids, then walk tiles in
// bands of a few tile-rows (8 by default; a tunable axis of the 16-bit family), column-major inside
// a band, so the tiles resident on one XCD form a compact block that shares A row-panels and B
// column-panels in that XCD's L2.
// Small grids (where a handful of integer divisions is a visible part of a 3 us kernel and L2
// locality is not at stake) are launched three-dimensional instead and read their tile directly.
__device__ __forceinline__ unsigned logical_of_block() {
    const unsigned total = gridDim.x, id = blockIdx.x;
    const unsigned q = total >> 3, r = total & 7u, x = id & 7u;
    return x * q + (x < r ? x : r) + (id >> 3);
}

// tile with logical id `logical` of a one-dimensional launch: units (batch item, K partition) in
// order, inside a unit bands of p.bandRows tile-rows walked column-major
__device__ __forceinline__ TileCoord tile_of_logical(const GemmParams &p, unsigned logical) {
    const unsigned per = p.tileSpan ? (unsigned)p.tileSpan : (unsigned)p.tilesM * (unsigned)p.tilesN;
    const unsigned unit = logical / per, t = logical - unit * per + (unsigned)p.tileBase;
    TileCoord c;
    c.batch = (int)(unit / (unsigned)p.splitK);
    c.split = (int)(unit - (unsigned)c.batch * (unsigned)p.splitK);
    const unsigned h = (unsigned)p.bandRows;
    const unsigned band = h * (unsigned)p.tilesN;
    const unsigned g = t / band, in = t - g * band;
    const unsigned first = g * h;
    const unsigned rows = ((unsigned)p.tilesM - first) < h ? ((unsigned)p.tilesM - first) : h;
    c.tn = (int)(in / rows);
    c.tm = (int)(first + (in - (unsigned)c.tn * rows));
    return c;
}

// inverse of the tile walk above: position of tile (tm, tn) in the one-dimensional order of a unit
__device__ __forceinline__ unsigned logical_of_tile(const GemmParams &p, int tm, int tn) {
    const unsigned h = (unsigned)p.bandRows;
    const unsigned g = (unsigned)tm / h, first = g * h;
    const unsigned rows = ((unsigned)p.tilesM - first) < h ? ((unsigned)p.tilesM - first) : h;
    return g * h * (unsigned)p.tilesN + (unsigned)tn * rows + ((unsigned)tm - first);
}

// Where a split-K instantiation puts its partial sums and with which row length: the dense
// [partition][batch][M][N] array, or, in a launch over part of the tiles, the compact tile
// [partition][tile - tileBase] (the returned base is shifted so that base + row * ld + col with
// the absolute row and column lands inside that tile).
__device__ __forceinline__ float *partial_base(const GemmParams &p, const TileCoord &tc, long long &ld) {
    if (p.tileSpan) {
        ld = p.bn;
        const long long tileElems = (long long)p.bm * p.bn;
        const long long rel = (long long)logical_of_tile(p, tc.tm, tc.tn) - p.tileBase;
        return p.ws + ((long long)tc.split * p.tileSpan + rel) * tileElems -
               ((long long)tc.tm * p.bm * p.bn + (long long)tc.tn * p.bn);
    }
    ld = p.N;
    return p.ws + ((long long)tc.split * p.batch + tc.batch) * (long long)p.M * p.N;
}

__device__ __forceinline__ TileCoord tile_of_block(const GemmParams &p) {
    if (p.grid3d) {
        TileCoord c;
        c.tn = (int)blockIdx.x;
        c.tm = (int)blockIdx.y;
        const unsigned unit = blockIdx.z;
        if (p.splitK == 1) {
            c.batch = (int)unit; c.split = 0;
        } else {
            c.batch = (int)(unit / (unsigned)p.splitK);
            c.split = (int)(unit - (unsigned)c.batch * (unsigned)p.splitK);
        }
        return c;
    }
    return tile_of_logical(p, logical_of_block());
}

// Epilogue.  `visit(f)` calls f(row, col, acc) for every accumulator element this lane owns
// (tile-relative to the matrix, i.e. absolute row / col).  The three output modes are separated
// outside the element loops so the per-element code is a bounds test and one store:
//   SPLIT (a split-K instantiation): raw partial sum to this split's slice of the workspace;
//   beta == 0: C = alpha * acc (C is never read);
//   otherwise: C = alpha * acc + beta * C;
//   with a bias vector, bias[col] is added last (a split-K instantiation leaves that to the
//   reduction pass).
template <bool SPLIT, class Visit>
__device__ __forceinline__ void write_tile(const GemmParams &p, const TileCoord &tc, float *Cb,
                                           Visit visit) {
    const int M = p.M, N = p.N;
    if constexpr (SPLIT) {
        long long wld;
        float *w = partial_base(p, tc, wld);
        visit([&](int row, int col, float acc) {
            if (row < M && col < N) w[(long long)row * wld + col] = acc;
        });
    } else if (p.out16) {
        const float alpha = p.alpha, beta = p.beta;
        const float *bias = p.bias;
        const long long ldc = p.ldc;
        visit([&](int row, int col, float acc) {
            if (row < M && col < N)
                store_bf16_out(Cb, (long long)tc.batch * p.strideC16 + (long long)row * ldc + col, acc, alpha,
                               beta, bias ? bias[col] : 0.0f);
        });
    } else if (p.bias != nullptr) {
        const float alpha = p.alpha, beta = p.beta;
        const float *bias = p.bias;
        const long long ldc = p.ldc;
        visit([&](int row, int col, float acc) {
            if (row < M && col < N) {
                float *c = Cb + (long long)row * ldc + col;
                float v = alpha * acc;
                if (beta != 0.0f) v = fmaf(beta, *c, v);
                *c = v + bias[col];
            }
        });
    } else if (p.beta == 0.0f) {
        const float alpha = p.alpha;
        const long long ldc = p.ldc;
        visit([&](int row, int col, float acc) {
            if (row < M && col < N) Cb[(long long)row * ldc + col] = alpha * acc;
        });
    } else {
        const float alpha = p.alpha, beta = p.beta;
        const long long ldc = p.ldc;
        visit([&](int row, int col, float acc) {
            if (row < M && col < N) {
                float *c = Cb + (long long)row * ldc + col;
                *c = fmaf(beta, *c, alpha * acc);
            }
        });
    }
}

// Where an accumulator tile goes: the matrix C (alpha, beta applied) or, in a split-K
// instantiation, this partition's slice of the workspace (raw partial sums, dense rows of N).
struct OutTarget {
    float *base;
    const float *bias;               // added after alpha / beta; null in split-K instantiations
    long long ld;
    float alpha, beta;
    int M, N;
    int out16;                       // C is bf16 (never set in split-K instantiations)
    long long off16;                 // element offset of the batch item in a bf16 C
};

template <bool SPLIT>
__device__ __forceinline__ OutTarget out_target(const GemmParams &p, const TileCoord &tc, float *Cb) {
    OutTarget o;
    o.M = p.M; o.N = p.N;
    if constexpr (SPLIT) {
        o.base = partial_base(p, tc, o.ld);
        o.alpha = 1.0f; o.beta = 0.0f; o.bias = nullptr; o.out16 = 0; o.off16 = 0;
    } else {
        o.base = Cb; o.ld = p.ldc; o.alpha = p.alpha; o.beta = p.beta; o.bias = p.bias; o.out16 = p.out16;
        o.off16 = (long long)tc.batch * p.strideC16;
    }
    return o;
}

// One lane's share of an MFMA fragment: NE values in one column `col`, at rows r0 + rowOff(e).
// `full` (the same for every lane of the wave) says the whole fragment lies inside the matrix:
// then there is no per-element test, and with beta != 0 all the old values are fetched before the
// first one is needed.  Edge fragments test every element.
template <bool SPLIT, int NE, class RowOff>
__device__ __forceinline__ void store_lane_column(const OutTarget &o, int r0, int col, bool full,
                                                  const float (&v)[NE], RowOff rowOff) {
    if (!SPLIT && o.out16) {
        // bf16 output: one form for interior and edge fragments
        if (col < o.N) {
            const float bv = o.bias ? o.bias[col] : 0.0f;
#pragma unroll
            for (int e = 0; e < NE; ++e)
                if (r0 + rowOff(e) < o.M)
                    store_bf16_out(o.base, o.off16 + (long long)(r0 + rowOff(e)) * o.ld + col, v[e], o.alpha,
                                   o.beta, bv);
        }
        return;
    }
    float *ptr = o.base + (long long)r0 * o.ld + col;
    if (!SPLIT && o.bias != nullptr) {
        // bias form: the lane's column is fixed, so one bias value serves all its elements
        if (col < o.N) {
            const float bv = o.bias[col];
            float old[NE];
#pragma unroll
            for (int e = 0; e < NE; ++e)
                old[e] = (o.beta != 0.0f && r0 + rowOff(e) < o.M) ? ptr[(long long)rowOff(e) * o.ld] : 0.0f;
#pragma unroll
            for (int e = 0; e < NE; ++e)
                if (r0 + rowOff(e) < o.M) {
                    float x = o.alpha * v[e];
                    if (o.beta != 0.0f) x = fmaf(o.beta, old[e], x);
                    ptr[(long long)rowOff(e) * o.ld] = x + bv;
                }
        }
    } else if (full) {
        if (SPLIT) {
#pragma unroll
            for (int e = 0; e < NE; ++e) ptr[(long long)rowOff(e) * o.ld] = v[e];
        } else if (o.beta == 0.0f) {
#pragma unroll
            for (int e = 0; e < NE; ++e) ptr[(long long)rowOff(e) * o.ld] = o.alpha * v[e];
        } else {
            float old[NE];
#pragma unroll
            for (int e = 0; e < NE; ++e) old[e] = ptr[(long long)rowOff(e) * o.ld];
#pragma unroll
            for (int e = 0; e < NE; ++e) ptr[(long long)rowOff(e) * o.ld] = fmaf(o.beta, old[e], o.alpha * v[e]);
        }
    } else if (col < o.N) {
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (r0 + rowOff(e) < o.M) {
                float *c = ptr + (long long)rowOff(e) * o.ld;
                if (SPLIT) *c = v[e];
                else if (o.beta == 0.0f) *c = o.alpha * v[e];
                else *c = fmaf(o.beta, *c, o.alpha * v[e]);
            }
        }
    }
}

// accumulator register e of lane l of a 16x16 MFMA fragment holds C[4*(l/16) + e][l%16]
template <bool SPLIT, int FM, int FN, class Acc>
__device__ __forceinline__ void write_tile_mfma16(const GemmParams &p, const TileCoord &tc, float *Cb,
                                                  int rowBase, int colBase, int lane, const Acc &acc) {
    const OutTarget o = out_target<SPLIT>(p, tc, Cb);
    const int rb = __builtin_amdgcn_readfirstlane(rowBase), cb = __builtin_amdgcn_readfirstlane(colBase);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const bool full = rb + i * 16 + 16 <= o.M && cb + j * 16 + 16 <= o.N;
            const float v[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
            store_lane_column<SPLIT, 4>(o, rb + i * 16 + 4 * (lane >> 4), cb + j * 16 + (lane & 15), full, v,
                                        [](int e) { return e; });
        }
}

// accumulator register e of lane l of a 32x32 MFMA fragment holds C[8*(e/4) + 4*(l/32) + e%4][l%32]
template <bool SPLIT, int FM, int FN, class Acc>
__device__ __forceinline__ void write_tile_mfma32(const GemmParams &p, const TileCoord &tc, float *Cb,
                                                  int rowBase, int colBase, int lane, const Acc &acc) {
    const OutTarget o = out_target<SPLIT>(p, tc, Cb);
    const int rb = __builtin_amdgcn_readfirstlane(rowBase), cb = __builtin_amdgcn_readfirstlane(colBase);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const bool full = rb + i * 32 + 32 <= o.M && cb + j * 32 + 32 <= o.N;
            float v[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
            store_lane_column<SPLIT, 16>(o, rb + i * 32 + 4 * (lane >> 5), cb + j * 32 + (lane & 31), full, v,
                                         [](int e) { return 8 * (e >> 2) + (e & 3); });
        }
}

// The same fragment layout written in four chunks of four rows with the scheduler kept from
// merging them: fewer addresses and old values alive at once, for kernels that hold other
// registers (the next tile's operands) across the epilogue.
template <bool SPLIT, int FM, int FN, class Acc>
__device__ __forceinline__ void write_tile_mfma32_lean(const GemmParams &p, const TileCoord &tc, float *Cb,
                                                       int rowBase, int colBase, int lane, const Acc &acc) {
    const OutTarget o = out_target<SPLIT>(p, tc, Cb);
    const int rb = __builtin_amdgcn_readfirstlane(rowBase), cb = __builtin_amdgcn_readfirstlane(colBase);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const bool full = rb + i * 32 + 32 <= o.M && cb + j * 32 + 32 <= o.N;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float v[4] = {acc[i][j][4 * c], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2], acc[i][j][4 * c + 3]};
                store_lane_column<SPLIT, 4>(o, rb + i * 32 + 8 * c + 4 * (lane >> 5), cb + j * 32 + (lane & 31), full, v,
                                            [](int e) { return e; });
                __builtin_amdgcn_sched_barrier(0);
            }
        }
}

}  // namespace ks
