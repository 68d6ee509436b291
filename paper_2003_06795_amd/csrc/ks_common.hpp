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
    long long lda, ldb, ldc;
    long long strideA, strideB, strideC;
    int M, N, K, batch;
    int tilesM, tilesN;
    int splitK, kChunk;              // K range of split s is [s*kChunk, min(K, (s+1)*kChunk))
    float alpha, beta;
};

struct TileCoord {
    int batch, split, tm, tn;
};

// MI355X has 8 XCDs with private L2s and hands consecutive work-group ids to them round-robin.
// Renumber so that each XCD owns one contiguous run of logical tile ids, then walk tiles in
// bands of 8 tile-rows (column-major inside a band) so the tiles resident on one XCD form a
// compact block that shares A row-panels and B column-panels in that XCD's L2.
__device__ __forceinline__ TileCoord tile_of_block(const GemmParams &p) {
    const unsigned total = gridDim.x, id = blockIdx.x;
    const unsigned q = total >> 3, r = total & 7u, x = id & 7u;
    const unsigned logical = x * q + (x < r ? x : r) + (id >> 3);
    const unsigned per = (unsigned)p.tilesM * (unsigned)p.tilesN;
    const unsigned unit = logical / per, t = logical - unit * per;
    TileCoord c;
    c.batch = (int)(unit / (unsigned)p.splitK);
    c.split = (int)(unit - (unsigned)c.batch * (unsigned)p.splitK);
    const unsigned band = 8u * (unsigned)p.tilesN;
    const unsigned g = t / band, in = t - g * band;
    const unsigned first = g * 8u;
    const unsigned rows = ((unsigned)p.tilesM - first) < 8u ? ((unsigned)p.tilesM - first) : 8u;
    c.tn = (int)(in / rows);
    c.tm = (int)(first + (in - (unsigned)c.tn * rows));
    return c;
}

// One output entry.  splitK > 1: raw partial sum to the workspace slice of this split.
__device__ __forceinline__ void store_entry(const GemmParams &p, const TileCoord &tc, float *Cb,
                                            int row, int col, float acc) {
    if (row >= p.M || col >= p.N) return;
    if (p.splitK > 1) {
        p.ws[(((long long)tc.split * p.batch + tc.batch) * p.M + row) * (long long)p.N + col] = acc;
    } else {
        float *c = Cb + (long long)row * p.ldc + col;
        float v = p.alpha * acc;
        if (p.beta != 0.0f) v = fmaf(p.beta, *c, v);
        *c = v;
    }
}

}  // namespace ks
