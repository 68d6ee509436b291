// Host side of the C ABI: argument validation, registry, launch geometry, timing helper.
// Every compute step runs in the HIP kernels of this library; there is no CPU fallback.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/ks_gemm.h"
#include "registry.hpp"

#ifndef KS_GRID3D_MAX
#define KS_GRID3D_MAX 2048      // work-groups up to which the grid is launched three-dimensional
#endif
#ifndef KS_GRID3D_BYTES
#define KS_GRID3D_BYTES (4 << 20)   // ... and bytes of A and B together
#endif

namespace ks {

#define KS_DECL(n)                              \
    void register_f32_shard_##n(LaunchFn *);    \
    void register_bf16_shard_##n(LaunchFn *);   \
    void register_bf16_dma_shard_##n(LaunchFn *);
KS_DECL(0) KS_DECL(1) KS_DECL(2) KS_DECL(3) KS_DECL(4) KS_DECL(5) KS_DECL(6) KS_DECL(7)
KS_DECL(8) KS_DECL(9) KS_DECL(10) KS_DECL(11) KS_DECL(12) KS_DECL(13) KS_DECL(14) KS_DECL(15)
#undef KS_DECL

namespace {

constexpr int threads_of(int core, int bm, int bn, int p1, int p2) {
    return core == KS_CORE_FMA ? (bm / p1) * (bn / p2) : core == KS_CORE_KSLICE ? 64 * p1 * (bm / p2) * (bn / p2) : 64 * (bm / p1) * (bn / p2);
}

constexpr int KS_CORE_OF_FMA = KS_CORE_FMA, KS_CORE_OF_MFMA16 = KS_CORE_MFMA16,
              KS_CORE_OF_MFMA32 = KS_CORE_MFMA32, KS_CORE_OF_DIRECT = KS_CORE_DIRECT,
              KS_CORE_OF_KSLICE = KS_CORE_KSLICE;

const InstanceDesc kF32[kNumF32] = {
// kw: K groups inside the work-group (K-sliced members: waves along K); LDS-staged members with
// K groups also hold the float4 units through which the groups' accumulators are added
#define KS_F32_INSTANCE_KW(id, CORE, BM, BN, BK, P1, P2, SPLITK, KW)                                     \
    {id, KS_CORE_OF_##CORE, BM, BN, BK, P1, P2, threads_of(KS_CORE_OF_##CORE, BM, BN, P1, P2) * (KW), SPLITK, \
     KS_CORE_OF_##CORE == KS_CORE_DIRECT   ? 0                                                          \
     : KS_CORE_OF_##CORE == KS_CORE_KSLICE ? P1 * BM * BN * 4                                           \
                                           : (KW) * 2 * BK * ((BM + (BK < 16 ? 64 / BK : 4)) + (BN + (BK < 16 ? 64 / BK : 4))) * 4 + \
                                                 ((KW) > 1 ? (KW) * BM * BN * 4 : 0),                     \
     KS_CORE_OF_##CORE == KS_CORE_KSLICE ? P1 : (KW)},
#define KS_F32_INSTANCE(id, CORE, BM, BN, BK, P1, P2, SPLITK) KS_F32_INSTANCE_KW(id, CORE, BM, BN, BK, P1, P2, SPLITK, 1)
#define KS_F32_INSTANCE_SK(id, CORE, BM, BN, BK, P1, P2, PERCU)                                          \
    {id, KS_CORE_OF_##CORE, BM, BN, BK, P1, P2, threads_of(KS_CORE_OF_##CORE, BM, BN, P1, P2), 1,         \
     2 * BK * ((BM + (BK < 16 ? 64 / BK : 4)) + (BN + (BK < 16 ? 64 / BK : 4))) * 4, 1, 8, PERCU},
#include "instances.def"
#undef KS_F32_INSTANCE
#undef KS_F32_INSTANCE_KW
#undef KS_F32_INSTANCE_SK
};

const InstanceDesc kBf16[kNumBf16] = {
#define KS_BF16_INSTANCE_BAND(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK, BAND)                \
    {id, (F) == 16 ? KS_CORE_MFMA16 : KS_CORE_MFMA32, BM, BN, BK, WM, WN, 64 * (BM / WM) * (BN / WN), \
     SPLITK, STAGES * BK * (BM + BN) * 2, 1, BAND},
#define KS_BF16_INSTANCE(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK) \
    KS_BF16_INSTANCE_BAND(id, F, BM, BN, BK, WM, WN, STAGES, SPLITK, 8)
#include "instances.def"
#undef KS_BF16_INSTANCE
#undef KS_BF16_INSTANCE_BAND
};

LaunchFn g_f32[kNumF32];
LaunchFn g_bf16[kNumBf16];
LaunchFn g_bf16_dma[kNumBf16];
std::once_flag g_once;

void init_tables() {
    register_f32_shard_0(g_f32); register_f32_shard_1(g_f32); register_f32_shard_2(g_f32);
    register_f32_shard_3(g_f32); register_f32_shard_4(g_f32); register_f32_shard_5(g_f32);
    register_f32_shard_6(g_f32); register_f32_shard_7(g_f32); register_f32_shard_8(g_f32);
    register_f32_shard_9(g_f32); register_f32_shard_10(g_f32); register_f32_shard_11(g_f32);
    register_f32_shard_12(g_f32); register_f32_shard_13(g_f32); register_f32_shard_14(g_f32);
    register_f32_shard_15(g_f32);
    register_bf16_shard_0(g_bf16); register_bf16_shard_1(g_bf16); register_bf16_shard_2(g_bf16);
    register_bf16_shard_3(g_bf16); register_bf16_shard_4(g_bf16); register_bf16_shard_5(g_bf16);
    register_bf16_shard_6(g_bf16); register_bf16_shard_7(g_bf16); register_bf16_shard_8(g_bf16);
    register_bf16_shard_9(g_bf16); register_bf16_shard_10(g_bf16); register_bf16_shard_11(g_bf16);
    register_bf16_shard_12(g_bf16); register_bf16_shard_13(g_bf16); register_bf16_shard_14(g_bf16);
    register_bf16_shard_15(g_bf16);
    register_bf16_dma_shard_0(g_bf16_dma); register_bf16_dma_shard_1(g_bf16_dma);
    register_bf16_dma_shard_2(g_bf16_dma); register_bf16_dma_shard_3(g_bf16_dma);
    register_bf16_dma_shard_4(g_bf16_dma); register_bf16_dma_shard_5(g_bf16_dma);
    register_bf16_dma_shard_6(g_bf16_dma); register_bf16_dma_shard_7(g_bf16_dma);
    register_bf16_dma_shard_8(g_bf16_dma); register_bf16_dma_shard_9(g_bf16_dma);
    register_bf16_dma_shard_10(g_bf16_dma); register_bf16_dma_shard_11(g_bf16_dma);
    register_bf16_dma_shard_12(g_bf16_dma); register_bf16_dma_shard_13(g_bf16_dma);
    register_bf16_dma_shard_14(g_bf16_dma); register_bf16_dma_shard_15(g_bf16_dma);
}

int g_forceGeneric = 0;
int g_tilesPerWG = 0;        // 0: chosen per call (multi_tiles); n >= 1: forced
int g_skPerCU = 0;           // 0: the member's own count of work-groups per compute unit; n >= 1: forced
int g_tailSplit = -1;        // -1: chosen per call (tail_split); 0: never; n >= 2: forced where it can run
int g_splitForced = 0;       // 0: per-call split members take auto_split's count; n >= 1: forced (at least two K-steps each)
void *g_ws = nullptr;
size_t g_wsBytes = 0;

// K partitions for an instance whose split is chosen per call.  Work-groups run in rounds of
// `slots` (256 compute units times the work-groups that fit one); a work-group costs its K-steps
// plus a fixed prologue/epilogue, and splitting adds the reduction pass.  The cheapest count wins
// (the smaller one on ties); never more than 64 (fp32) or 256 (16-bit), never more than fills one
// round (16-bit) or four (fp32), and at least two K-steps per partition.
//   fp32 members: twelve waves per compute unit, cost in K-steps as measured on the tuning set.
//   16-bit members: their LDS stages (up to 144 KB) limit a compute unit to one to four
//   work-groups, and a partition's tile of partial sums (written, then read by the reduction
//   pass) is charged in units of one K-step's operand traffic, 4 BM BN / ((BM + BN) BK).
int64_t split_slots(const InstanceDesc *d, bool f32) {
    const int64_t waves = d->threads / 64;
    int64_t perCU = 12 / waves > 0 ? 12 / waves : 1;
    if (!f32) {
        const int64_t byLds = d->ldsBytes > 0 ? (160 * 1024) / d->ldsBytes : perCU;
        perCU = byLds < perCU ? (byLds > 0 ? byLds : 1) : perCU;
    }
    return 256 * perCU;
}

int64_t auto_split_max(const InstanceDesc *d, int64_t tiles, bool f32) {
    const int64_t slots = split_slots(d, f32);
    int64_t s = (slots + tiles - 1) / (tiles > 0 ? tiles : 1);
    // fp32: up to four rounds of partitions.  A count that overfills one round can still end
    // sooner, e.g. 152 tiles in 5 partitions are three rounds of a fifth of K where unsplit tiles
    // are one round of all of it; the cost estimate below matched the measured order of the counts
    // on every shape tried.
    if (f32 && tiles > 0 && 4 * slots / tiles > s) s = 4 * slots / tiles;
    const int64_t cap = f32 ? 64 : 256;
    return s < 1 ? 1 : (s > cap ? cap : s);
}

int64_t auto_split(const InstanceDesc *d, int64_t tiles, int64_t kTiles, bool f32) {
    const int64_t slots = split_slots(d, f32);
    const int64_t partial = f32 ? 0 : (4LL * d->bm * d->bn) / ((int64_t)(d->bm + d->bn) * d->bk);
    int64_t best = 1, bestCost = -1;
    const int64_t smax = auto_split_max(d, tiles, f32);
    // kTiles counts the steps of the work-group.  The K groups of an LDS-staged member share the
    // compute unit's matrix pipe, so one of its steps lasts as many K-steps as it has groups; the
    // waves of a K-sliced member wait on memory side by side and a step lasts one.
    const int64_t stepCost = d->core != KS_CORE_KSLICE && d->kw > 1 ? d->kw : 1;
    for (int64_t s = 1; s <= smax && (s == 1 || 2 * s <= kTiles); ++s) {
        const int64_t rounds = (tiles * s + slots - 1) / slots;
        const int64_t cost = rounds * (stepCost * ((kTiles + s - 1) / s) + 6 + (s > 1 ? partial : 0)) + (s > 1 ? 10 : 0);
        if (bestCost < 0 || cost < bestCost) { bestCost = cost; best = s; }
    }
    return best;
}

// K partitions for the last, partly filled round of work-groups of a 16-bit member whose split is
// chosen per call (0 = launch every tile whole).  With `slots` work-groups resident at once, T
// tiles take ceil(T / slots) rounds although the last one may hold only a few tiles; cutting the
// K range of just those left-over tiles into s = slots / left-over partitions fills that round
// with work-groups that are s times shorter.  Same cost units as auto_split; the partitioned round
// also pays its tiles of partial sums and a third launch.  Only with at least one whole round
// before it (otherwise auto_split decides), and only when it saves 3 % of the call.
bool tail_split_member(const InstanceDesc *d) {
    // members whose LDS stages leave room for one work-group per compute unit: their round is 256
    // work-groups for certain (smaller members share a unit and suffer less from a short last round)
    return d->splitK == 0 && d->ldsBytes > 0 && (160 * 1024) / d->ldsBytes == 1;
}
// scratch of the largest partitioning tail_split can choose for this many tiles (0: no hybrid launch)
size_t tail_split_bytes(const InstanceDesc *d, int64_t tiles) {
    if (!tail_split_member(d)) return 0;
    const int64_t slots = split_slots(d, false);
    const int64_t tail = tiles % slots;
    if (tiles < slots || tail == 0) return 0;
    int64_t s = slots / tail;
    if (s > 16) s = 16;
    return s >= 2 ? (size_t)s * (size_t)tail * (size_t)d->bm * (size_t)d->bn * sizeof(float) : 0;
}
int64_t tail_split(const InstanceDesc *d, int64_t tiles, int64_t kTiles) {
    if (!tail_split_member(d)) return 0;
    const int64_t slots = split_slots(d, false);
    const int64_t rounds = tiles / slots, tail = tiles % slots;
    if (rounds == 0 || tail == 0) return 0;
    int64_t s = slots / tail;
    if (s > 16) s = 16;
    if (2 * s > kTiles) s = kTiles / 2;
    if (g_tailSplit >= 2) return s >= 2 ? (s < g_tailSplit ? s : g_tailSplit) : 0;
    if (s < 2) return 0;
    const int64_t partial = (4LL * d->bm * d->bn) / ((int64_t)(d->bm + d->bn) * d->bk);
    const int64_t plain = (rounds + 1) * (kTiles + 6);
    const int64_t hybrid = rounds * (kTiles + 6) + (kTiles + s - 1) / s + 6 + partial + 14;
    return 100 * hybrid <= 97 * plain ? s : 0;
}

// Tiles one work-group of a multi-tile fp32 member walks.  Walking T tiles takes the work-group
// launch, the pipeline fill and part of the wait behind the previous tile's stores out of T - 1 of
// T tiles, but leaves T times fewer work-groups to balance over the compute units, and the
// flattened loop itself is about 5 % slower per K-step.  Measured on outputs of 0.2 - 3.3 GB with
// T = 4 .. 8: 7 - 25 % faster when a tile has one K-step, 0 - 7 % with two, 5 % slower from four
// on; slower as soon as the launch has fewer than about ten rounds of work-groups.  Hence: only
// for tiles of at most two K-steps and at least 32 rounds of single-tile work-groups, and then so
// that 8 rounds remain (at most 8 tiles).
int multi_tiles(const InstanceDesc *d, int64_t tiles, int64_t K) {
    const int64_t waves = d->threads / 64;
    const int64_t slots = 256 * (12 / waves > 0 ? 12 / waves : 1);
    const int64_t rounds = tiles / slots;
    if (K > 2 * d->bk || rounds < 32) return 1;
    return (int)(rounds / 8 < 8 ? rounds / 8 : 8);
}

// Balanced persistent form: work-groups of the launch, and the scratch its divided tiles need (two
// raw accumulator tiles per work-group: the head and the tail of its share of the left-over tiles).
int64_t sk_groups(const InstanceDesc *d) { return 256LL * (g_skPerCU > 0 ? g_skPerCU : d->sk); }
size_t sk_workspace_bytes(const InstanceDesc *d) {
    return (size_t)sk_groups(d) * 2 * (size_t)d->bm * (size_t)d->bn * sizeof(float);
}

const InstanceDesc *desc_of(int dtype, int id) {
    if (dtype == KS_F32) return (id >= 0 && id < kNumF32) ? &kF32[id] : nullptr;
    if (dtype == KS_BF16 || dtype == KS_F16) return (id >= 0 && id < kNumBf16) ? &kBf16[id] : nullptr;
    return nullptr;
}

// C = beta * C (+ bias) for K == 0 (C is not read when beta == 0)
__global__ void scale_c_kernel(float *C, long long ldc, long long strideC, int M, int N, int batch,
                               float beta, const float *bias, int out16) {
    const long long total = (long long)batch * M * N;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        const long long b = i / ((long long)M * N), r = i - b * (long long)M * N;
        if (out16) {
            store_bf16_out(C, b * strideC + (r / N) * ldc + (r % N), 0.0f, 0.0f, beta, bias ? bias[r % N] : 0.0f);
            continue;
        }
        float *c = C + b * strideC + (r / N) * ldc + (r % N);
        const float v = beta == 0.0f ? 0.0f : beta * *c;
        *c = bias ? v + bias[r % N] : v;
    }
}

// Plain 16-byte-per-lane copy of known size: the yardstick that hardware traffic counters
// (rocprofv3 FETCH_SIZE / WRITE_SIZE) are scaled by.
__global__ void copy_kernel(const floatx4 *src, floatx4 *dst, long long n16) {
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n16;
         i += (long long)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Split-K second pass, four consecutive entries of a row per lane (N, ldc, strideC multiples of 4;
// ws and C 16-byte aligned).  Each entry is summed in the same order as in the scalar form.
__global__ void splitk_reduce4_kernel(const float *ws, float *C, long long ldc, long long strideC, int M,
                                      int N, int batch, int splitK, float alpha, float beta,
                                      const float *bias) {
    const long long per = (long long)batch * M * N, per4 = per >> 2;
    for (long long q = blockIdx.x * (long long)blockDim.x + threadIdx.x; q < per4;
         q += (long long)gridDim.x * blockDim.x) {
        const long long i = q << 2;
        floatx4 acc = *reinterpret_cast<const floatx4 *>(ws + i);
        // partial sums are fetched eight at a time (independent loads) and added in partition order
        int s = 1;
        for (; s + 8 <= splitK; s += 8) {
            floatx4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const floatx4 *>(ws + (long long)(s + u) * per + i);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; s < splitK; ++s) acc += *reinterpret_cast<const floatx4 *>(ws + (long long)s * per + i);
        const long long b = i / ((long long)M * N), r = i - b * (long long)M * N;
        floatx4 *c = reinterpret_cast<floatx4 *>(C + b * strideC + (r / N) * ldc + (r % N));
        floatx4 v = alpha * acc;
        if (beta != 0.0f) {
            const floatx4 c0 = *c;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaf(beta, c0[e], alpha * acc[e]);
        }
        if (bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += bias[r % N + e];
        }
        *c = v;
    }
}

// Split-K second pass: C = alpha * (ws[0] + ws[1] + ... in this fixed order) + beta * C (+ bias)
__global__ void splitk_reduce_kernel(const float *ws, float *C, long long ldc, long long strideC, int M,
                                     int N, int batch, int splitK, float alpha, float beta,
                                     const float *bias, int out16) {
    const long long per = (long long)batch * M * N;
    for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < per;
         i += (long long)gridDim.x * blockDim.x) {
        float acc = ws[i];
        int s = 1;
        for (; s + 8 <= splitK; s += 8) {                 // eight independent loads, added in partition order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = ws[(long long)(s + u) * per + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; s < splitK; ++s) acc += ws[(long long)s * per + i];
        const long long b = i / ((long long)M * N), r = i - b * (long long)M * N;
        if (out16) {
            store_bf16_out(C, b * strideC + (r / N) * ldc + (r % N), acc, alpha, beta, bias ? bias[r % N] : 0.0f);
            continue;
        }
        float *c = C + b * strideC + (r / N) * ldc + (r % N);
        float v = alpha * acc;
        if (beta != 0.0f) v = fmaf(beta, *c, v);
        if (bias) v += bias[r % N];
        *c = v;
    }
}

// Second pass of a launch whose last round was partitioned along K (tail_split): work-group
// (b, y) adds up rows 8 y .. 8 y + 7 of the compact partial tiles [partition][b] of tile
// tileBase + b in partition order and writes them to C.  Few tiles are partitioned (fewer than one
// round of work-groups), so the rows of a tile are spread over many work-groups; partial sums are
// read 16 bytes per lane (the workspace is 16-byte aligned, tiles are multiples of 16 floats wide).
#define KS_TAIL_REDUCE_ROWS 8
__global__ void tail_reduce_kernel(const GemmParams p) {
    const TileCoord tc = tile_of_logical(p, blockIdx.x);       // partition 0 of tile tileBase + blockIdx.x
    const int bm = p.bm, bn = p.bn, S = p.splitK;
    const long long tileElems = (long long)bm * bn;
    const float *w0 = p.ws + (long long)blockIdx.x * tileElems;
    const long long per = (long long)p.tileSpan * tileElems;
    const int r0 = tc.tm * bm, c0 = tc.tn * bn;
    const int rows = p.M - r0 < bm ? p.M - r0 : bm, cols = p.N - c0 < bn ? p.N - c0 : bn;
    const int rFirst = (int)blockIdx.y * KS_TAIL_REDUCE_ROWS;
    const int q = bn / 4;                                      // float4 units per tile row
    for (int u = threadIdx.x; u < KS_TAIL_REDUCE_ROWS * q; u += blockDim.x) {
        const int r = rFirst + u / q, c = (u % q) * 4;
        if (r >= rows || c >= cols) continue;
        const float *w = w0 + (long long)r * bn + c;
        floatx4 acc = *reinterpret_cast<const floatx4 *>(w);
        int s = 1;
        for (; s + 8 <= S; s += 8) {                 // eight independent loads, added in partition order
            floatx4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = *reinterpret_cast<const floatx4 *>(w + (long long)(s + k) * per);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc += v[k];
        }
        for (; s < S; ++s) acc += *reinterpret_cast<const floatx4 *>(w + (long long)s * per);
        const long long at = (long long)(r0 + r) * p.ldc + (c0 + c);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c + e >= cols) break;
            if (p.out16) {
                store_bf16_out(p.C, at + e, acc[e], p.alpha, p.beta, p.bias ? p.bias[c0 + c + e] : 0.0f);
                continue;
            }
            float *cp = p.C + at + e;
            float v = p.alpha * acc[e];
            if (p.beta != 0.0f) v = fmaf(p.beta, *cp, v);
            if (p.bias) v += p.bias[c0 + c + e];
            *cp = v;
        }
    }
}

int validate(int transA, int transB, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
             const void *B, int64_t ldb, const float *C, int64_t ldc, int64_t batch,
             int64_t strideC) {
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return KS_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || batch < 0) return KS_ERR_INVALID_ARG;
    const int64_t lim = 2147483647LL - 512;
    if (M >= lim || N >= lim || K >= lim || batch >= lim) return KS_ERR_UNSUPPORTED;
    // leading dimensions take part in 64-bit element offsets (row * ld, row < 2^31): with ld < 2^31
    // every such product stays below 2^62
    const int64_t ldLim = 1LL << 31;
    if (lda >= ldLim || ldb >= ldLim || ldc >= ldLim) return KS_ERR_UNSUPPORTED;
    if (M == 0 || N == 0 || batch == 0) return KS_OK;
    if (!C || ldc < N) return KS_ERR_INVALID_ARG;
    if (K > 0) {
        if (!A || !B) return KS_ERR_INVALID_ARG;
        if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return KS_ERR_INVALID_ARG;
    }
    if (batch > 1) {
        int64_t span = 0;                             // elements one item of C covers
        if (__builtin_mul_overflow(M - 1, ldc, &span) || __builtin_add_overflow(span, N, &span))
            return KS_ERR_UNSUPPORTED;
        const int64_t s = strideC < 0 ? -strideC : strideC;
        if (s < span) return KS_ERR_INVALID_ARG;
    }
    return KS_OK;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Scratch for split-K partial sums: the registered workspace, or the library's static array.
struct Workspace {
    void *ptr;
    size_t bytes;
};
Workspace registered_ws() { return Workspace{g_ws, g_wsBytes}; }

int remainder_member(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch, int tA, int tB, Workspace w);

int run_ws(Workspace wsp, int dtype, int id, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
           const void *A, int64_t lda, const void *B, int64_t ldb, float beta, float *C, int64_t ldc,
           int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, hipStream_t stream,
           const float *bias = nullptr, int out16 = 0, ks_launch_plan_t *planOnly = nullptr) {
    const InstanceDesc *d = desc_of(dtype, id);
    if (!d) return KS_ERR_INVALID_ARG;
    const int rc = validate(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, batch, strideC);
    if (rc != KS_OK) return rc;
    if (planOnly) {
        *planOnly = ks_launch_plan_t{};
        planOnly->kernel_id = id;
        planOnly->split_k = 1;
        planOnly->tiles_per_workgroup = 1;
    }
    if (M == 0 || N == 0 || batch == 0) return KS_OK;
    if (planOnly && K == 0) return KS_OK;
    std::call_once(g_once, init_tables);

    // An error left behind by an earlier, unrelated runtime call must not be blamed on this launch.
    (void)hipGetLastError();

    if (K == 0) {
        const long long total = (long long)batch * M * N;
        const int grid = (int)((total + 255) / 256 < 65535 ? (total + 255) / 256 : 65535);
        hipLaunchKernelGGL(scale_c_kernel, dim3(grid), dim3(256), 0, stream, C, (long long)ldc,
                           (long long)strideC, (int)M, (int)N, (int)batch, beta, bias, out16);
        return hipGetLastError() == hipSuccess ? KS_OK : KS_ERR_LAUNCH;
    }

    // a pruned build holds only the kept members
    if ((dtype == KS_F32 ? g_f32[id] : g_bf16[id]) == nullptr) return KS_ERR_UNSUPPORTED;

    // 16-bit operands whose K is not a whole number of K-steps would take the member's general
    // kernel for all of K (measured 1.5 - 2.2 times slower than the direct-to-LDS path on large
    // problems).  Where everything else qualifies for that path, the K range is cut instead: the
    // remainder (fewer than one K-step, general kernel) goes first and applies alpha, beta and the
    // bias, then the whole K-steps run on the fast path with beta = 1.  The partial result passes
    // through C in fp32 (one more rounding per entry, far inside the bound), so an output kept in
    // bf16 is not served this way.  The two extra passes over C cost 15 - 40 us on 2048^2 .. 4096^2
    // outputs; measured against the general kernel over all of K the cut gains 24 - 100 % when an
    // operand is not K-contiguous (NN, TN, TT; level at 2048^2 NN), while with both operands
    // K-contiguous (NT), where the general kernel is at its best, it loses 40 % at 2048^2, is level
    // at 1024^2 and gains 4 - 12 % from 4096^2 on: NT is cut only for outputs of at least 2^24 entries.
    if (dtype != KS_F32 && !out16 && g_forceGeneric == 0 && K % d->bk != 0 && K % 8 == 0 && K >= 4LL * d->bk) {
        const int64_t Kr = K % d->bk, Kh = K - Kr;
        const bool akc = transA == 0, bkc = transB == 1;
        const bool pays = !(akc && bkc) || M * N >= (1LL << 24);
        const bool vecOk = pays && aligned(A, 16) && aligned(B, 16) && lda % 8 == 0 && ldb % 8 == 0 && (akc || M % 8 == 0) &&
                           (bkc || N % 8 == 0) && (batch == 1 || (strideA % 8 == 0 && strideB % 8 == 0)) &&
                           lda <= (1LL << 22) && ldb <= (1LL << 22);
        if (vecOk) {
            const uint16_t *Ar = static_cast<const uint16_t *>(A) + (akc ? Kh : Kh * lda);
            const uint16_t *Br = static_cast<const uint16_t *>(B) + (bkc ? Kh : Kh * ldb);
            if (planOnly) {
                const int prc = run_ws(wsp, dtype, id, transA, transB, M, N, Kh, alpha, A, lda, B, ldb, 1.0f, C, ldc, batch,
                                       strideA, strideB, strideC, stream, nullptr, 0, planOnly);
                if (prc == KS_OK) planOnly->k_remainder = (int32_t)Kr;
                return prc;
            }
            // the remainder is a GEMM with a very short K of its own, bound by the pass over C: it
            // runs with the member the deployed tree names for that problem
            int idr = remainder_member(dtype, M, N, Kr, batch, transA, transB, wsp);
            if (idr < 0) idr = id;
            const int r1 = run_ws(wsp, dtype, idr, transA, transB, M, N, Kr, alpha, Ar, lda, Br, ldb, beta, C, ldc, batch,
                                  strideA, strideB, strideC, stream, bias, 0, nullptr);
            if (r1 != KS_OK) return r1;
            return run_ws(wsp, dtype, id, transA, transB, M, N, Kh, alpha, A, lda, B, ldb, 1.0f, C, ldc, batch, strideA,
                          strideB, strideC, stream, nullptr, 0, nullptr);
        }
    }

    GemmParams p;
    p.A = A; p.B = B; p.C = C; p.ws = nullptr; p.bias = bias; p.out16 = out16;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.strideA = strideA; p.strideB = strideB;
    p.strideC = out16 ? 0 : strideC; p.strideC16 = out16 ? strideC : 0;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.batch = (int)batch;
    p.tilesM = (int)((M + d->bm - 1) / d->bm);
    p.tilesN = (int)((N + d->bn - 1) / d->bn);
    const int64_t kTiles = (K + d->bk - 1) / d->bk;
    p.splitK = d->splitK;
    if (d->splitK == 0) {
        // automatic split: as many K partitions as fill the device, at least two K-steps each,
        // and no more than the registered workspace can hold (1 = the plain single-kernel form)
        const int64_t steps = (kTiles + d->kw - 1) / d->kw;
        int64_t s = auto_split(d, (int64_t)p.tilesM * p.tilesN * batch, steps, dtype == KS_F32);
        if (g_splitForced > 0) s = g_splitForced > 1 && 2 * (int64_t)g_splitForced > steps ? (steps / 2 > 1 ? steps / 2 : 1) : g_splitForced;
        const size_t per = (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
        if (!wsp.ptr) s = 1;
        else if ((size_t)s * per > wsp.bytes) s = (int64_t)(wsp.bytes / per);
        p.splitK = s < 1 ? 1 : (int)s;
    }
    p.kChunk = (int)(((kTiles + p.splitK - 1) / p.splitK) * d->bk);
    p.alpha = alpha; p.beta = beta;

    int64_t grid64 = (int64_t)p.tilesM * p.tilesN * batch * p.splitK;
    if (grid64 > 2147483647LL) return KS_ERR_UNSUPPORTED;
    // three-dimensional launch only where the tile order cannot matter for L2: few work-groups
    // and operands that fit one XCD's L2 several times over
    const double operandBytes = (double)(M + N) * (double)K * (double)batch * (dtype == KS_F32 ? 4 : 2);
    p.grid3d = grid64 <= KS_GRID3D_MAX && operandBytes <= (double)KS_GRID3D_BYTES && p.tilesM <= 65535 &&
                       batch * p.splitK <= 65535
                   ? 1
                   : 0;
    p.tilesPerWG = 1;
    p.bandRows = d->band;
    p.skGroups = 0; p.skRounds = 0; p.skTailTiles = 0;
    p.tileBase = 0; p.tileSpan = 0; p.bm = d->bm; p.bn = d->bn;
    if (d->sk > 0) {
        // Balanced persistent form where it pays (measured against the plain member of the same
        // tiles on the tuning tables): tiles that do not divide evenly over the work-groups, fewer
        // than four rounds of them (with more, the uneven last round matters less than what the
        // hardware's own dispatch gains by handing a tile to whichever unit is free), and at
        // least 1024 of K per tile and one K-step per share (below that the raw accumulator tiles
        // of the divided tiles and the second kernel cost more than the balance gains).  A forced work-group count
        // (ks_set_balanced_groups) takes the form whenever it can run.  Its scratch must be there
        // unless no tile is divided; otherwise the plain member runs.
        // With few tiles every tile is divided among many work-groups; a 512-thread member then
        // runs faster with one work-group per compute unit than with two (fewer raw accumulator
        // tiles per output tile, and the whole unit for each share): measured 2-10 % up to 80
        // tiles of 128x128, even from 110 to 224, 3-5 % the other way from 270 on.
        const int64_t groups = g_skPerCU == 0 && d->sk == 2 && d->threads >= 512 && grid64 <= 96 ? 256 : sk_groups(d);
        const int64_t tail = grid64 % groups;
        const bool fits = tail == 0 || (wsp.ptr && wsp.bytes >= sk_workspace_bytes(d) && aligned(wsp.ptr, 16));
        const bool pays = g_skPerCU > 0 || (tail != 0 && grid64 < 4 * groups && K >= 1024 && tail * kTiles >= groups);
        if (fits && pays && tail * kTiles < (1LL << 50)) {
            p.skGroups = (int)groups;
            p.skRounds = (int)(grid64 / groups);
            p.skTailTiles = (int)tail;
            p.ws = static_cast<float *>(wsp.ptr);
            p.grid3d = 0;
            grid64 = groups;
        }
    }
    if (dtype == KS_F32 && !p.grid3d && p.splitK == 1 && p.skGroups == 0 && f32_multi_tile(d->core, d->bm, d->bn, d->p1, d->p2, d->kw)) {
        p.tilesPerWG = g_tilesPerWG > 0 ? g_tilesPerWG : multi_tiles(d, grid64, K);
        grid64 = (grid64 + p.tilesPerWG - 1) / p.tilesPerWG;
    }

    if (p.splitK > 1) {
        const size_t need = (size_t)p.splitK * (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
        if (!wsp.ptr || wsp.bytes < need) return KS_ERR_WORKSPACE;
        p.ws = static_cast<float *>(wsp.ptr);
    }

    // contiguous direction: A is K-contiguous when not transposed, B when transposed
    const bool akc = transA == 0, bkc = transB == 1;
    const int w = dtype == KS_F32 ? 4 : 8;            // elements per 16-byte access
    const int64_t extA = akc ? K : M, extB = bkc ? K : N;
    const bool vec = aligned(A, 16) && aligned(B, 16) && lda % w == 0 && ldb % w == 0 &&
                     extA % w == 0 && extB % w == 0 &&
                     (batch == 1 || (strideA % w == 0 && strideB % w == 0));
    const int splitBit = p.splitK > 1 ? 8 : 0;       // read by instances whose split is chosen per call
    const int variant = (akc ? 4 : 0) + (bkc ? 2 : 0) + (vec ? 1 : 0) + splitBit;

    // bf16 fast path: operand tiles go global -> LDS directly.  Needs 16-byte accesses, whole
    // K-steps, and tile-relative byte offsets that fit 32 bits.
    const int f16Bit = dtype == KS_F16 ? 16 : 0;     // same 16-bit members, binary16 MFMA
    const bool dma = dtype != KS_F32 && vec && g_forceGeneric == 0 && K % d->bk == 0 &&
                     lda <= (1LL << 22) && ldb <= (1LL << 22);
    // Hybrid launch of a 16-bit member whose split is chosen per call: whole rounds of work-groups
    // compute their tiles over all of K, the tiles of the last, partly filled round are cut along
    // K (tail_split), and a third kernel adds their partial tiles up.
    int64_t tailS = 0, tailTiles = 0, mainGrid = grid64;
    if (dma && d->splitK == 0 && p.splitK == 1 && batch == 1 && g_tailSplit != 0 && wsp.ptr &&
        aligned(wsp.ptr, 16)) {
        const int64_t slots = split_slots(d, false);
        const int64_t s = tail_split(d, grid64, kTiles);
        const int64_t tail = grid64 % slots;
        if (s >= 2 && (size_t)s * (size_t)tail * (size_t)d->bm * (size_t)d->bn * sizeof(float) <= wsp.bytes) {
            tailS = s; tailTiles = tail; mainGrid = grid64 - tail;
            p.grid3d = 0;                            // both launches walk the one-dimensional tile order
        }
    }
    if (planOnly) {
        planOnly->tail_split = (int32_t)tailS;
        planOnly->split_k = p.splitK;
        planOnly->vector_loads = vec ? 1 : 0;
        planOnly->grid_3d = p.grid3d;
        planOnly->tiles_per_workgroup = p.tilesPerWG;
        planOnly->workgroups = tailS ? mainGrid + tailTiles * tailS : grid64;
        planOnly->balanced_groups = p.skGroups;
        planOnly->divided_tiles = p.skTailTiles;
        planOnly->path = !dma ? 0
                         : bf16_two_groups(d->core == KS_CORE_MFMA32 ? 32 : 16, d->bm, d->bn, d->bk, d->p1, d->p2,
                                           d->ldsBytes / (d->bk * (d->bm + d->bn) * 2))
                             ? 2
                             : 1;
        return KS_OK;
    }
    if (tailS) {
        const int layoutBits = (akc ? 2 : 0) + (bkc ? 1 : 0) + f16Bit;
        g_bf16_dma[id](p, (int)mainGrid, layoutBits, stream);
        if (hipGetLastError() != hipSuccess) return KS_ERR_LAUNCH;
        GemmParams q = p;
        q.splitK = (int)tailS;
        q.kChunk = (int)(((kTiles + tailS - 1) / tailS) * d->bk);
        q.tileBase = (int)mainGrid;
        q.tileSpan = (int)tailTiles;
        q.ws = static_cast<float *>(wsp.ptr);
        g_bf16_dma[id](q, (int)(tailTiles * tailS), layoutBits + 8, stream);
        if (hipGetLastError() != hipSuccess) return KS_ERR_LAUNCH;
        hipLaunchKernelGGL(tail_reduce_kernel,
                           dim3((unsigned)tailTiles, (unsigned)((d->bm + KS_TAIL_REDUCE_ROWS - 1) / KS_TAIL_REDUCE_ROWS)),
                           dim3(256), 0, stream, q);
        return hipGetLastError() == hipSuccess ? KS_OK : KS_ERR_LAUNCH;
    }
    if (dma)
        g_bf16_dma[id](p, (int)grid64, (akc ? 2 : 0) + (bkc ? 1 : 0) + splitBit + f16Bit, stream);
    else
        (dtype == KS_F32 ? g_f32[id] : g_bf16[id])(p, (int)grid64, variant + f16Bit, stream);
    if (hipGetLastError() != hipSuccess) return KS_ERR_LAUNCH;

    if (p.splitK > 1) {
        const long long total = (long long)batch * M * N;
        // four entries per lane once there are enough entries to fill the device that way; small
        // outputs with many partitions run one entry per lane (same sums either way)
        const bool vec4 = !out16 && N % 4 == 0 && ldc % 4 == 0 && aligned(C, 16) && aligned(p.ws, 16) &&
                          (batch == 1 || strideC % 4 == 0) && total >= 4LL * 256 * 256;
        const long long units = vec4 ? total / 4 : total;
        const int grid = (int)((units + 255) / 256 < 1048576 ? (units + 255) / 256 : 1048576);
        if (vec4)
            hipLaunchKernelGGL(splitk_reduce4_kernel, dim3(grid), dim3(256), 0, stream, p.ws, C, (long long)ldc,
                               (long long)strideC, (int)M, (int)N, (int)batch, p.splitK, alpha, beta, bias);
        else
            hipLaunchKernelGGL(splitk_reduce_kernel, dim3(grid), dim3(256), 0, stream, p.ws, C, (long long)ldc,
                               (long long)strideC, (int)M, (int)N, (int)batch, p.splitK, alpha, beta, bias,
                               out16);
        if (hipGetLastError() != hipSuccess) return KS_ERR_LAUNCH;
    }
    return KS_OK;
}

int run(int dtype, int id, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
        const void *A, int64_t lda, const void *B, int64_t ldb, float beta, float *C, int64_t ldc,
        int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, hipStream_t stream,
        const float *bias = nullptr, int out16 = 0) {
    return run_ws(registered_ws(), dtype, id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch,
                  strideA, strideB, strideC, stream, bias, out16);
}

}  // namespace
}  // namespace ks

using namespace ks;

extern "C" int ks_num_kernels(int dtype) {
    if (dtype == KS_F32) return kNumF32;
    if (dtype == KS_BF16 || dtype == KS_F16) return kNumBf16;
    return KS_ERR_INVALID_ARG;
}

extern "C" int ks_kernel_info(int dtype, int kernel_id, ks_kernel_info_t *out) {
    const InstanceDesc *d = desc_of(dtype, kernel_id);
    if (!d || !out) return KS_ERR_INVALID_ARG;
    out->id = d->id;
    out->dtype = dtype;
    out->core = d->core;
    out->bm = d->bm; out->bn = d->bn; out->bk = d->bk;
    const int frag = d->core == KS_CORE_MFMA32 ? 32 : 16;
    if (d->core == KS_CORE_FMA) {
        out->wm = d->p1; out->wn = d->p2; out->tm = d->p1; out->tn = d->p2;
    } else if (d->core == KS_CORE_KSLICE) {
        out->wm = d->p2; out->wn = d->p2; out->tm = d->p2 / 16; out->tn = d->p2 / 16;
    } else {
        out->wm = d->p1; out->wn = d->p2; out->tm = d->p1 / frag; out->tn = d->p2 / frag;
    }
    out->k_waves = d->kw;
    out->threads = d->threads;
    out->split_k = d->splitK;
    out->lds_bytes = d->ldsBytes;
    out->band_rows = d->band;
    out->balanced_per_cu = d->sk;
    std::call_once(g_once, init_tables);
    out->available = (dtype == KS_F32 ? g_f32[kernel_id] : g_bf16[kernel_id]) != nullptr ? 1 : 0;
    return KS_OK;
}

extern "C" int ks_calibration_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) return KS_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16)
        return KS_ERR_INVALID_ARG;
    (void)hipGetLastError();
    const long long n16 = (long long)(bytes / 16);
    const int grid = (int)((n16 + 255) / 256 < 16384 ? (n16 + 255) / 256 : 16384);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const floatx4 *>(src), static_cast<floatx4 *>(dst), n16);
    return hipGetLastError() == hipSuccess ? KS_OK : KS_ERR_LAUNCH;
}

extern "C" int ks_set_fast_path(int enabled) {
    g_forceGeneric = enabled ? 0 : 1;
    return KS_OK;
}

extern "C" int ks_set_tiles_per_workgroup(int n) {
    if (n < 0 || n > 64) return KS_ERR_INVALID_ARG;
    g_tilesPerWG = n;
    return KS_OK;
}

extern "C" int ks_set_balanced_groups(int per_cu) {
    if (per_cu < 0 || per_cu > 8) return KS_ERR_INVALID_ARG;
    g_skPerCU = per_cu;
    return KS_OK;
}

extern "C" int ks_set_tail_split(int partitions) {
    if (partitions != -1 && partitions != 0 && (partitions < 2 || partitions > 16)) return KS_ERR_INVALID_ARG;
    g_tailSplit = partitions;
    return KS_OK;
}

extern "C" int ks_set_split_partitions(int partitions) {
    if (partitions < 0 || partitions > 256) return KS_ERR_INVALID_ARG;
    g_splitForced = partitions;
    return KS_OK;
}

extern "C" int ks_set_workspace(void *device_ptr, size_t bytes) {
    if (device_ptr == nullptr || bytes == 0) {
        g_ws = nullptr;
        g_wsBytes = 0;
        return KS_OK;
    }
    if (reinterpret_cast<uintptr_t>(device_ptr) % sizeof(float)) return KS_ERR_INVALID_ARG;
    g_ws = device_ptr;
    g_wsBytes = bytes;
    return KS_OK;
}

extern "C" size_t ks_workspace_bytes_needed(int dtype, int kernel_id, int64_t M, int64_t N,
                                            int64_t batch) {
    const InstanceDesc *d = desc_of(dtype, kernel_id);
    if (!d || M <= 0 || N <= 0 || batch <= 0) return 0;
    if (d->sk > 0) return sk_workspace_bytes(d);
    if (d->splitK == 1) return 0;
    int64_t s = d->splitK;
    if (s == 0) {
        const int64_t tiles = ((M + d->bm - 1) / d->bm) * ((N + d->bn - 1) / d->bn) * batch;
        s = auto_split_max(d, tiles, dtype == KS_F32);
        if (s <= 1) return dtype != KS_F32 && batch == 1 ? tail_split_bytes(d, tiles) : 0;
    }
    return (size_t)s * (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
}

#define KS_GEMM_PASS                                                                            \
    transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch, strideA, strideB, strideC, \
        static_cast<hipStream_t>(stream)

// Kernel for the selecting entry points: the tree's choice, unless that is a split-K instance and
// the registered workspace cannot hold its partial sums; then the instance with the same tiles
// and no split is used instead, so that a caller who never registers a workspace is still served.
static int select_checked(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch, int tA, int tB,
                          Workspace w = registered_ws()) {
    const int id = ks_select(dtype, M, N, K, batch, tA, tB);
    if (id < 0) return id;
    const InstanceDesc *d = desc_of(dtype, id);
    if (!d || d->splitK <= 1 || M <= 0 || N <= 0 || batch <= 0) return id;
    const size_t need = (size_t)d->splitK * (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
    if (w.ptr && w.bytes >= need) return id;
    const int n = dtype == KS_F32 ? kNumF32 : kNumBf16;
    std::call_once(g_once, init_tables);
    for (int pass = 0; pass < 2; ++pass)          // same K-step first, then any K-step
        for (int i = 0; i < n; ++i) {
            const InstanceDesc *e = desc_of(dtype, i);
            if ((dtype == KS_F32 ? g_f32[i] : g_bf16[i]) != nullptr &&      // present in a pruned build
                e->splitK == 1 && e->core == d->core && e->bm == d->bm && e->bn == d->bn &&
                e->p1 == d->p1 && e->p2 == d->p2 && (pass == 1 || e->bk == d->bk))
                return i;
        }
    return id;
}

namespace ks {
namespace {
// member that runs the remainder of a K range that is not a whole number of K-steps (run_ws)
int remainder_member(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch, int tA, int tB, Workspace w) {
    const int id = select_checked(dtype, M, N, K, batch, tA, tB, w);
    if (id < 0) return id;
    std::call_once(g_once, init_tables);
    return g_bf16[id] != nullptr ? id : -1;
}
}  // namespace
}  // namespace ks

extern "C" int ks_gemm_f32_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                       int64_t K, float alpha, const float *A, int64_t lda,
                                       const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                                       int64_t batch, int64_t strideA, int64_t strideB,
                                       int64_t strideC, void *stream) {
    return run(KS_F32, kernel_id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_bf16_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                        int64_t K, float alpha, const uint16_t *A, int64_t lda,
                                        const uint16_t *B, int64_t ldb, float beta, float *C,
                                        int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                                        int64_t strideC, void *stream) {
    return run(KS_BF16, kernel_id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                           const float *A, int64_t lda, const float *B, int64_t ldb, float beta,
                           float *C, int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                           int64_t strideC, void *stream) {
    const int id = select_checked(KS_F32, M, N, K, batch, transA, transB);
    if (id < 0) return id;
    return run(KS_F32, id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                            const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, float beta,
                            float *C, int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                            int64_t strideC, void *stream) {
    const int id = select_checked(KS_BF16, M, N, K, batch, transA, transB);
    if (id < 0) return id;
    return run(KS_BF16, id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_f16(int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                           const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, float beta,
                           float *C, int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                           int64_t strideC, void *stream) {
    const int id = select_checked(KS_F16, M, N, K, batch, transA, transB);
    if (id < 0) return id;
    return run(KS_F16, id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_f16_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                       int64_t K, float alpha, const uint16_t *A, int64_t lda,
                                       const uint16_t *B, int64_t ldb, float beta, float *C,
                                       int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                                       int64_t strideC, void *stream) {
    return run(KS_F16, kernel_id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_bias(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N,
                            int64_t K, float alpha, const void *A, int64_t lda, const void *B,
                            int64_t ldb, float beta, float *C, int64_t ldc, const float *bias,
                            int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                            void *stream) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB);
        if (kernel_id < 0) return kernel_id;
    }
    return run(dtype, kernel_id, KS_GEMM_PASS, bias);
}

extern "C" int ks_gemm_out_bf16(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                int64_t K, float alpha, const void *A, int64_t lda, const void *B,
                                int64_t ldb, float beta, uint16_t *C16, int64_t ldc, const float *bias,
                                int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                                void *stream) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB);
        if (kernel_id < 0) return kernel_id;
    }
    float *C = reinterpret_cast<float *>(C16);        // element size is carried by the out16 flag
    return run(dtype, kernel_id, KS_GEMM_PASS, bias, 1);
}

// Entry point for callers that cannot allocate device memory (HIP graph capture, serving loops):
// split-K partial sums go to a static device array instead of a registered workspace.
#define KS_STATIC_SCRATCH_BYTES (16u << 20)
namespace ks {
namespace {
__device__ __align__(256) float scratch[KS_STATIC_SCRATCH_BYTES / sizeof(float)];
constexpr int kMaxDevices = 64;
float *g_scratchPtr[kMaxDevices];      // device address of `scratch` on each device, once known
std::mutex g_scratchMutex;

// Device address of this device's copy of the static array (every device holds its own).  The
// array's name is only a host-side handle: the address kernels can use comes from the runtime.
int static_scratch(Workspace *out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KS_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratchMutex);
    if (!g_scratchPtr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return KS_ERR_LAUNCH;
        }
        g_scratchPtr[dev] = static_cast<float *>(ptr);
    }
    out->ptr = g_scratchPtr[dev];
    out->bytes = KS_STATIC_SCRATCH_BYTES;
    return KS_OK;
}
}  // namespace
}  // namespace ks

extern "C" int ks_gemm_static_scratch(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                      int64_t K, float alpha, const void *A, int64_t lda, const void *B,
                                      int64_t ldb, float beta, float *C, int64_t ldc, int64_t batch,
                                      int64_t strideA, int64_t strideB, int64_t strideC, void *stream) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    Workspace w{nullptr, 0};
    const int rc = static_scratch(&w);
    if (rc != KS_OK) return rc;
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB, w);
        if (kernel_id < 0) return kernel_id;
    }
    return run_ws(w, dtype, kernel_id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_with_workspace(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N,
                                      int64_t K, float alpha, const void *A, int64_t lda, const void *B,
                                      int64_t ldb, float beta, float *C, int64_t ldc, int64_t batch,
                                      int64_t strideA, int64_t strideB, int64_t strideC, void *workspace_device,
                                      size_t workspace_bytes, void *stream) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if ((workspace_device == nullptr) != (workspace_bytes == 0)) return KS_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace_device) % sizeof(float)) return KS_ERR_INVALID_ARG;
    const Workspace w{workspace_device, workspace_bytes};
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB, w);
        if (kernel_id < 0) return kernel_id;
    }
    return run_ws(w, dtype, kernel_id, KS_GEMM_PASS);
}

extern "C" int ks_gemm_plan(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                            float alpha, const void *A, int64_t lda, const void *B, int64_t ldb, float beta,
                            float *C, int64_t ldc, int64_t batch, int64_t strideA, int64_t strideB,
                            int64_t strideC, ks_launch_plan_t *out) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if (!out) return KS_ERR_INVALID_ARG;
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB);
        if (kernel_id < 0) return kernel_id;
    }
    void *stream = nullptr;
    return run_ws(registered_ws(), dtype, kernel_id, KS_GEMM_PASS, nullptr, 0, out);
}

extern "C" int ks_time_gemm(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N,
                            int64_t K, float alpha, const void *A, int64_t lda, const void *B,
                            int64_t ldb, float beta, float *C, int64_t ldc, int64_t batch,
                            int64_t strideA, int64_t strideB, int64_t strideC, void *stream,
                            int warmup, int iters, int reps, float *ms_out) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if (iters < 1 || iters > 1024 || reps < 1 || warmup < 0 || !ms_out) return KS_ERR_INVALID_ARG;
    if (kernel_id < 0) {
        kernel_id = select_checked(dtype, M, N, K, batch, transA, transB);
        if (kernel_id < 0) return kernel_id;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // one pool of events per host thread (events are created once and reused by later calls)
    static thread_local hipEvent_t ev[2 * 1024];
    static thread_local int evCount = 0;
    while (evCount < 2 * iters) {
        if (hipEventCreate(&ev[evCount]) != hipSuccess) return KS_ERR_LAUNCH;
        ++evCount;
    }
    // the first launch also proves the arguments: if it is refused nothing else is enqueued
    int rc = KS_OK;
    for (int i = 0; i < warmup; ++i) {
        rc = run(dtype, kernel_id, KS_GEMM_PASS);
        if (rc != KS_OK) return rc;
    }
    for (int i = 0; i < iters; ++i) {
        if (hipEventRecord(ev[2 * i], s) != hipSuccess) return KS_ERR_LAUNCH;
        for (int r = 0; r < reps; ++r) {
            rc = run(dtype, kernel_id, KS_GEMM_PASS);
            if (rc != KS_OK) return rc;
        }
        if (hipEventRecord(ev[2 * i + 1], s) != hipSuccess) return KS_ERR_LAUNCH;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return KS_ERR_LAUNCH;
    for (int i = 0; i < iters; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) return KS_ERR_LAUNCH;
        ms_out[i] = ms / (float)reps;
    }
    return KS_OK;
}
