/*
 * ks_gemm.h - C ABI of the tiled-GEMM kernel family with learned kernel selection.
 *
 * The library is the matrix-multiply case study of "Towards automated kernel
 * selection in machine learning systems" (Lawson, 2020) rebuilt for one AMD
 * MI355X (gfx950): a family of tiled GEMM kernels parameterised by work-group
 * tile, wave/register tile and K-step (Section II), an offline tuner that turns
 * brute-force timings into a pruned kept set with a decision-tree regression
 * (Sections II-A, III, III-A) and a decision-tree runtime selector over the
 * kept set (Section IV).
 *
 * Conventions shared by every entry point
 *   - All matrices are ROW-MAJOR.  op(A) is M x K: transA == 0 means A is stored
 *     M x K with row stride lda >= K; transA == 1 means A is stored K x M with
 *     lda >= M.  op(B) is K x N: transB == 0 -> stored K x N, ldb >= N;
 *     transB == 1 -> stored N x K, ldb >= K.  C is M x N with ldc >= N.
 *     (A column-major caller uses C^T = op(B)^T op(A)^T: swap A<->B and M<->N.)
 *   - Batch item b uses A + b*strideA, B + b*strideB, C + b*strideC (strides in
 *     elements).  strideA / strideB may be 0 (the operand is shared).
 *   - A, B, C, the workspace and every other pointer named "device" are DEVICE
 *     pointers owned by the caller; the library never allocates, frees or keeps
 *     them (except the registered workspace pointer).  Everything else is host
 *     memory.  Calls are asynchronous on `stream` (a hipStream_t; NULL = the
 *     default stream): buffers must stay alive until the stream has drained.
 *   - beta == 0 means C is not read.  alpha == 0 has no special case.
 *   - Every function returns a ks_status (0 = success, negative = error) unless
 *     stated otherwise; on error nothing is launched and C is untouched.
 *   - No entry point is a CPU fallback: without a HIP device the compute calls
 *     fail with KS_ERR_LAUNCH.
 *   - Threads: the compute entry points keep no per-call host state and may be
 *     called from several host threads (each on its own stream) at once, with
 *     one exception: the registered workspace is a single buffer, so two GEMMs
 *     that both run a split-K member must not be in flight together (same
 *     stream, or ordered by the caller); ks_gemm_with_workspace takes the
 *     scratch per call and has no such limit.  ks_set_workspace,
 *     ks_set_fast_path, ks_set_tiles_per_workgroup, ks_set_balanced_groups,
 *     ks_set_tail_split, ks_set_split_partitions and ks_set_selector are not thread-safe: they change process-wide settings
 *     that the compute entry points read.  ks_time_gemm keeps its events per
 *     host thread.  The library acts on the calling thread's current HIP device
 *     and never changes it.
 */
#ifndef KS_GEMM_H
#define KS_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KS_OK = 0,
    KS_ERR_INVALID_ARG = -1,   /* bad flag, negative size, short leading dimension, NULL operand,
                                  overlapping batch items of C, id out of range */
    KS_ERR_UNSUPPORTED = -2,   /* size beyond the 32-bit tile arithmetic of the kernels; a member that a
                                  pruned build does not contain */
    KS_ERR_LAUNCH = -3,        /* the HIP runtime refused the launch / no device */
    KS_ERR_WORKSPACE = -4      /* a split-K kernel needs a larger registered workspace */
} ks_status;

/* type of A and B; C is fp32.  KS_F16 (IEEE binary16) runs the instantiations of the 16-bit family
 * (the ids, registry entries and deployed tree of KS_BF16) with the binary16 MFMA instructions. */
typedef enum { KS_F32 = 0, KS_BF16 = 1, KS_F16 = 2 } ks_dtype;
typedef enum {
    KS_CORE_FMA = 0, KS_CORE_MFMA16 = 1, KS_CORE_MFMA32 = 2, KS_CORE_DIRECT = 3, KS_CORE_KSLICE = 4
} ks_core;

/* One member of the kernel family (Section II: work-group tile, per-work-item tile and
 * accumulator step are the compile-time parameters of the paper's kernel). */
typedef struct {
    int32_t id;          /* dense, 0 .. ks_num_kernels(dtype)-1; frozen */
    int32_t dtype;       /* ks_dtype */
    int32_t core;        /* ks_core: per-lane FMA outer product, MFMA with 16x16 / 32x32 fragments staged
                            through LDS, 16x16 MFMA fed from global memory directly (no LDS), or the
                            same with the K range of a work-group cut into one slice per wave */
    int32_t bm, bn, bk;  /* work-group tile rows, cols; K-step staged through LDS */
    int32_t wm, wn;      /* wave tile (MFMA cores); equals tm x tn layout unit for the FMA core */
    int32_t tm, tn;      /* per-lane register tile (FMA core) or fragments per wave (MFMA cores) */
    int32_t threads;     /* work-group size */
    int32_t split_k;     /* number of K partitions reduced through the workspace (1 = none; 0 = chosen
                            per call: enough partitions to fill the device, fewer if the registered
                            workspace is smaller, none without a workspace) */
    int32_t lds_bytes;   /* static LDS of the instantiation (both stages) */
    int32_t k_waves;     /* K slices inside one work-group, summed through LDS at the end: one wave per
                            slice and wave tile for core KS_CORE_KSLICE, one complete group of waves
                            (threads / k_waves lanes, its own LDS stages) per slice for the LDS-staged
                            MFMA cores; 1 = none */
    int32_t band_rows;   /* tile order of a one-dimensional launch: tiles are walked in bands of this many
                            tile rows, column-major inside a band (which tiles share an XCD's L2) */
    int32_t available;   /* 1: compiled into this library; 0: pruned away (a library built with only the
                            kept set of the deployed trees, Section III, holds the kept members and the
                            four bring-up tiles; forcing an absent member returns KS_ERR_UNSUPPORTED) */
    int32_t balanced_per_cu; /* > 0: the member has a balanced persistent form (the launch shape, the
                            run-time axis of the Section II kernel, is then a fixed 256 * balanced_per_cu
                            work-groups that each compute the same number of K-steps: whole tiles
                            first, then an equal share of the tiles left over, whose parts a second
                            kernel adds in K order).  Taken per call where it pays: tiles that do
                            not divide evenly over those work-groups, fewer than four rounds of them,
                            K >= 1024, and a registered workspace of ks_workspace_bytes_needed()
                            bytes; the plain member of the same tiles runs otherwise.  0: no such form */
} ks_kernel_info_t;

/* Node of a deployed decision tree (Section IV: nested integer comparisons).
 * feature < 0 marks a leaf whose kernel id is `value`; otherwise go to `left` when
 * features[feature] <= threshold, else to `right`. */
typedef struct {
    int32_t feature;
    int32_t left, right;
    int32_t value;
    int64_t threshold;
} ks_tree_node_t;

/* Feature vector the trees see, computed from the call's sizes with integer arithmetic only:
 * 0:M 1:N 2:K 3:batch 4:transA 5:transB  (the first KS_NUM_RAW_FEATURES)
 * 6:M*N 7:M*N*K 8:min(M,N) 9:max(M,N)   (derived; saturating at INT64_MAX) */
#define KS_NUM_RAW_FEATURES 6
#define KS_NUM_FEATURES 10
#define KS_MAX_TREE_NODES 4096

/* ---------------------------------------------------------------- GEMM (Section II)
 * C_b = alpha * op(A_b) * op(B_b) + beta * C_b for b in [0, batch).
 * ks_gemm_* picks the kernel with ks_select (Section IV) and is bit-identical to
 * ks_gemm_*_with_kernel(ks_select(...), ...) whenever the registered workspace can hold the
 * chosen kernel's split-K partial sums; if it cannot (or none is registered) the instance with
 * the same tiles and split_k == 1 runs instead.  A, B, C: device pointers.
 * bf16 operands are raw bfloat16 bit patterns; accumulation and C are fp32.
 * Degenerate sizes: M, N or batch == 0 -> success, nothing launched; K == 0 -> C = beta*C.
 * Errors: KS_ERR_INVALID_ARG (see ks_status), KS_ERR_UNSUPPORTED when M, N or K >= 2^31 - 512 or a leading dimension >= 2^31,
 * KS_ERR_WORKSPACE, KS_ERR_LAUNCH. */
int ks_gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                float beta, float *C, int64_t ldc,
                int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);
int ks_gemm_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                 float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                 float beta, float *C, int64_t ldc,
                 int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);

/* fp16 inputs (one of the data types the paper's Section II kernel can be instantiated for is
 * left open; this is the IEEE binary16 form): A and B are binary16 bit patterns, products are
 * exact in fp32 and accumulate in fp32 like the bf16 form.  Arguments, statuses and ownership as
 * for ks_gemm_bf16; kernel ids are those of KS_BF16. */
int ks_gemm_f16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                float beta, float *C, int64_t ldc,
                int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);
int ks_gemm_f16_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                            float alpha, const uint16_t *A, int64_t lda, const uint16_t *B,
                            int64_t ldb, float beta, float *C, int64_t ldc,
                            int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                            void *stream);

/* Tuner path (Section II-A brute force): the same call with the instantiation forced. */
int ks_gemm_f32_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                            float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                            float beta, float *C, int64_t ldc,
                            int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                            void *stream);
int ks_gemm_bf16_with_kernel(int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                             float alpha, const uint16_t *A, int64_t lda, const uint16_t *B,
                             int64_t ldb, float beta, float *C, int64_t ldc,
                             int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                             void *stream);

/* Fully-connected layer form (Section II-A names fully-connected layers among the sources of the
 * GEMMs): C_b = alpha * op(A_b) * op(B_b) + beta * C_b + 1 * bias^T, i.e. bias[j] is added to column
 * j of every row of every batch item after the alpha / beta step, inside the kernel's epilogue
 * (inside the reduction pass for split-K members).  bias: device, N floats, read-only, may be
 * NULL (then exactly ks_gemm_*).  dtype: ks_dtype of A and B.  kernel_id < 0: the deployed tree
 * selects; otherwise that instantiation runs.  Other arguments, statuses and ownership as for
 * ks_gemm_f32 / ks_gemm_bf16. */
int ks_gemm_bias(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                 float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                 float beta, float *C, int64_t ldc, const float *bias,
                 int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);

/* Output kept in bf16 (mixed precision for inference-style layers; the accumulator stays fp32):
 * C16 holds bf16 bit patterns, M x N with row stride ldc and batch stride strideC counted in
 * 2-byte elements; when beta != 0 the old value is widened exactly, and
 * alpha * acc + beta * C + bias[j] (fp32) is rounded to bf16, to nearest with ties to even, in the
 * kernel's epilogue (split-K members: in the reduction pass; their partial sums stay fp32).
 * bias may be NULL.  dtype: type of A and B (any ks_dtype); kernel_id < 0 selects.  Other
 * arguments, statuses and ownership as for ks_gemm_bias. */
int ks_gemm_out_bf16(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                     float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                     float beta, uint16_t *C16, int64_t ldc, const float *bias,
                     int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): ks_gemm_*_with_kernel (kernel_id >= 0) or ks_gemm_*
 * (kernel_id < 0: the deployed tree selects) with the split-K partial sums kept in a static device
 * array of the library, KS_STATIC_SCRATCH_BYTES = 16 MiB per device (held by every device the
 * library runs on until the process ends), instead of the registered workspace, which this call
 * neither reads nor needs.  The call allocates and frees nothing.  dtype: type of A and B; A, B, C:
 * device pointers as for ks_gemm_f32 / ks_gemm_bf16; the array's device address is looked up once
 * per device on the first call there (the calling thread's current device).
 *   - A forced member with a fixed split_k > 1 needs split_k * batch * M * N * 4 bytes: beyond
 *     16 MiB the call returns KS_ERR_WORKSPACE and launches nothing.  Members with split_k == 0
 *     take as many partitions as fit; with kernel_id < 0 a selected fixed-split member that does
 *     not fit is replaced by its split_k == 1 twin, as in ks_gemm_*.
 *   - Nothing has to start at zero: every partition writes its whole slice before the reduction
 *     pass reads it, so the array may hold the previous call's contents.
 *   - All calls on one device share that device's array: two such GEMMs that both split must not
 *     be in flight together on one device (same stream, or ordered by the caller); overlapping
 *     calls race. */
#define KS_STATIC_SCRATCH_BYTES (16u << 20)
int ks_gemm_static_scratch(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                           float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                           float beta, float *C, int64_t ldc,
                           int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, void *stream);

/* The same GEMM with the scratch passed per call instead of registered: ks_gemm_*_with_kernel
 * (kernel_id >= 0) or ks_gemm_* (kernel_id < 0, with the same fallback to the split_k == 1 twin when
 * the scratch is too small) using `workspace_device` (device pointer, at least 4-byte aligned; may
 * be NULL with workspace_bytes == 0) for split-K partial sums and for the divided tiles of the
 * balanced persistent form.  The registered workspace is neither read nor needed, so GEMMs on
 * different streams or host threads that each bring their own scratch may be in flight together
 * (Section II-A's tuner times one cell at a time; a serving process does not).  Needs what
 * ks_workspace_bytes_needed reports for the member; errors as for ks_gemm_*. */
int ks_gemm_with_workspace(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                           float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                           float beta, float *C, int64_t ldc,
                           int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                           void *workspace_device, size_t workspace_bytes, void *stream);

/* What a GEMM call would launch, without launching it: the same checks and decisions as
 * ks_gemm_*_with_kernel (kernel_id >= 0) or ks_gemm_* (kernel_id < 0) with the workspace that is
 * registered now.  For measurement tools that have to name the device function a call resolves to
 * (a member whose split is chosen per call runs another kernel, plus the reduction pass, when it
 * splits).  Arguments and statuses as for the GEMM calls; out: host. */
typedef struct {
    int32_t kernel_id;            /* the member that runs (after selection and the no-workspace fallback) */
    int32_t split_k;              /* K partitions taken; > 1 means partial-sum kernel + reduction pass */
    int32_t path;                 /* 0: the member's general kernel; 1: direct-to-LDS 16-bit kernel;
                                     2: direct-to-LDS kernel in its two-groups-of-waves form */
    int32_t vector_loads;         /* 16-byte global accesses are legal for these operands */
    int32_t grid_3d;              /* launched (tilesN, tilesM, batch * split_k) instead of one-dimensional */
    int32_t tiles_per_workgroup;  /* > 1: the multi-tile form of the large fp32 members */
    int64_t workgroups;
    int32_t balanced_groups;      /* > 0: the balanced persistent form runs, with this many work-groups */
    int32_t divided_tiles;        /* left-over tiles of that form, handed to its second kernel (0: none launched) */
    int32_t tail_split;           /* > 0: hybrid launch of a 16-bit member (ks_set_tail_split): the tiles of the
                                     last, partly filled round of work-groups run in this many K partitions
                                     (three kernels: whole tiles, partitioned tiles, their reduction) */
    int32_t k_remainder;          /* > 0 (16-bit operands only): K is not a whole number of the member's K-steps;
                                     the last k_remainder of K run first through the member's general kernel
                                     (applying alpha, beta and the bias), then the whole K-steps run on the
                                     direct-to-LDS path with beta = 1, which the other fields describe */
} ks_launch_plan_t;
int ks_gemm_plan(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                 float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                 float beta, float *C, int64_t ldc,
                 int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                 ks_launch_plan_t *out);

/* Brute-force timing of one (workload, instantiation) cell (Section II-A: runtime recorded over a
 * number of iterations).  Runs `warmup` untimed launches, then `iters` samples; a sample is
 * `reps` back-to-back launches bracketed by one pair of HIP events on `stream`.  Synchronises and
 * writes the per-launch time of each sample (elapsed / reps) in milliseconds to
 * ms_out[0 .. iters-1] (host).  dtype selects the f32 / bf16 entry point; A and B are device
 * pointers of that type.  kernel_id < 0 times the selected kernel (ks_select).
 * 1 <= iters <= 1024, reps >= 1, warmup >= 0. */
int ks_time_gemm(int dtype, int kernel_id, int transA, int transB, int64_t M, int64_t N, int64_t K,
                 float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                 float beta, float *C, int64_t ldc,
                 int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                 void *stream, int warmup, int iters, int reps, float *ms_out);

/* ---------------------------------------------------------------- registry (Section II)
 * The enumerated family: 64 fp32 instantiations (the size of the paper's compiled set) and
 * the bf16 set. */
int ks_num_kernels(int dtype);                                   /* count, or negative status */
int ks_kernel_info(int dtype, int kernel_id, ks_kernel_info_t *out);   /* out: host */

/* ---------------------------------------------------------------- selection (Section IV)
 * Walks the deployed decision tree for `dtype` with integer comparisons only and returns the
 * chosen kernel id (>= 0), or a negative status for a bad flag / negative size.  Pure, total
 * over non-negative sizes, thread-safe, allocation-free, no device access. */
int ks_select(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch, int transA, int transB);
/* The integer features ks_select compares (out: host array of KS_NUM_FEATURES). */
int ks_features(int64_t M, int64_t N, int64_t K, int64_t batch, int transA, int transB,
                int64_t *out);
/* Replace the deployed tree of `dtype` by a copy of nodes[0 .. n-1] (host; node 0 is the root).
 * The tree is validated (child indices in range and acyclic by construction: children must have
 * larger indices than their parent; leaf values must be kernel ids).  n == 0 restores the tree
 * compiled into the library.  Not thread-safe against concurrent ks_select / ks_gemm calls. */
int ks_set_selector(int dtype, const ks_tree_node_t *nodes, int n);
/* Copy the deployed tree out (host).  Returns the node count, or a negative status if cap is
 * too small. */
int ks_get_selector(int dtype, ks_tree_node_t *nodes, int cap);

/* The bf16 instantiations have two code paths with the same tiles: a generic one (any alignment,
 * any K) and a direct-to-LDS one used when operands are 16-byte aligned, leading dimensions and
 * contiguous extents are multiples of 8 and K is a multiple of the K-step.  When only the last
 * condition fails (K a multiple of 8 and at least four K-steps, output in fp32; with both operands
 * K-contiguous, where the generic path is at its best, only for outputs of 2^24 entries or more), the call runs as
 * two launches: the remainder of K beyond the whole K-steps through the generic path first, with
 * alpha, beta and the bias, then the whole K-steps through the direct-to-LDS path with beta = 1
 * (ks_launch_plan_t::k_remainder).  enabled == 0 forces the generic path for all of K (for testing
 * it at aligned shapes); nonzero restores the default. */
int ks_set_fast_path(int enabled);

/* The large-tile fp32 32x32-MFMA members (LDS-staged, tile of at least 8192 entries and 128
 * columns, wave tile of at most 2048, one K group) have a second form in which a work-group walks
 * several consecutive tiles, requesting the next tile's operands before the finished tile's C is
 * stored; a one-dimensional launch without split-K uses it with a count chosen per call from the
 * tile count and K (only for very large outputs with at most two K-steps per tile).  n == 0
 * restores that default; 1 <= n <= 64 forces the count (1 = every work-group one tile) for testing
 * and tuning.  Results do not depend on it (every tile is computed the same way whoever walks it).
 * Not thread-safe. */
int ks_set_tiles_per_workgroup(int n);

/* The members with a balanced persistent form (ks_kernel_info_t::balanced_per_cu > 0) launch
 * 256 * balanced_per_cu work-groups (the launch shape is the run-time axis of the Section II
 * kernel); a 512-thread member with two per compute unit launches 256 when the problem has at
 * most 96 tiles.  1 <= per_cu <= 8 forces another count per compute unit for testing and tuning, and
 * makes those members take the form on every call whose scratch is there (or that divides no
 * tile); 0 restores the members' own count and the per-call choice.  ks_workspace_bytes_needed
 * follows the forced count.  Results stay within the stated bound but the summation order of
 * divided tiles changes with the count.  Not thread-safe. */
int ks_set_balanced_groups(int per_cu);

/* Hybrid launches of the 16-bit members whose K split is chosen per call (split_k == 0), on their
 * direct-to-LDS path with batch 1 (the launch shape is the run-time axis of the Section II kernel).
 * Members whose LDS stages admit one work-group per compute unit take part (a round is then 256
 * work-groups).  When the tiles fill at least one whole round and leave a partly filled last round, the tiles of that round are cut along K into as many partitions as fill it (2 to
 * 16, at least two K-steps each): whole tiles, the partitioned tiles (partial sums as compact
 * tiles in the workspace, at most work-groups-per-round tiles of bm x bn floats) and a reduction
 * that adds the partitions in order run as three kernels on the stream.  partitions == -1 (the
 * default) takes the form where a cost estimate in K-steps says it saves 3 % of the call and the
 * workspace holds the tiles; 0 never; 2 .. 16 forces it wherever it can run, with at most that
 * many partitions (testing and tuning).  Results stay within the stated bound (the summation order
 * of the partitioned tiles changes).  Not thread-safe. */
int ks_set_tail_split(int partitions);

/* Members whose K split is chosen per call (split_k == 0) take the partition count of a cost
 * estimate in K-steps (work-groups per round, K-steps per partition, the reduction pass).
 * 1 <= partitions <= 256 forces that many instead (1 = no split), lowered to K-steps / 2 where a
 * partition would hold fewer than two K-steps and to what the workspace holds, for testing and
 * tuning (the partition count is part of the launch shape, the run-time axis of the Section II
 * kernel); 0 restores the estimate.  ks_workspace_bytes_needed does not follow a forced count.
 * Results stay within the stated bound (the summation order changes with the count).  Not
 * thread-safe. */
int ks_set_split_partitions(int partitions);

/* Measurement aid: copies `bytes` (a multiple of 16; both device pointers 16-byte aligned) with a
 * plain one-read-one-write kernel (ks::copy_kernel).  Hardware traffic counters collected over a
 * profile that contains this launch are scaled by what they report for it. */
int ks_calibration_copy(void *dst_device, const void *src_device, size_t bytes, void *stream);

/* Measurement aid: what the matrix pipe alone sustains on given operand VALUES (the clock this
 * device holds under matrix load depends on the bit patterns the instructions chew on).  2048
 * work-groups of eight waves load twelve 16-byte fragments per lane once from `operands_device`
 * (at least KS_MFMA_PROBE_BYTES, 16-byte aligned; pass the A operand of the GEMM in question) and
 * issue `rounds` x 32 dependent-free MFMAs of `dtype` each (fragment = 32: 32x32x16 for the 16-bit
 * types, 32x32x2 for fp32; fragment = 16, 16-bit types only: 16x16x32), with no LDS or memory traffic.
 * Runs the kernel twice on `stream`, synchronises, and reports the second run: TFLOP/s from HIP
 * events and, if mhz_out != NULL, the shader clock of work-group 0 (cycle counter over the
 * 100 MHz reference counter).  1 <= rounds <= 2^24.  Not thread-safe against itself. */
#define KS_MFMA_PROBE_BYTES (64u * 8u * 12u * 1024u)
int ks_mfma_sustained(int dtype, int fragment, const void *operands_device, size_t bytes, int rounds, void *stream,
                      double *tflops_out, double *mhz_out);

/* Measurement aid: the two-group 256 x 256 x 64 bf16 kernel on an NT problem (A: M x K, B: N x K,
 * both K-contiguous bf16 device buffers; C: M x N fp32 device buffer that is overwritten) with one of
 * its data paths left out, to read off what each path costs on given operand values:
 *   mode 0  the kernel as ks_gemm_bf16 runs it (C is the product)
 *   mode 1  no direct-to-LDS global loads after the first two K-steps
 *   mode 2  no LDS fragment reads after the first two K-steps
 *   mode 3  neither (MFMAs, barriers and the C write only)
 *   mode 4  the kernel of mode 0, whose work-group 0 also reads the shader cycle counter and the
 *           100 MHz reference counter at both ends of its K loop: *mhz_out (host, required in
 *           modes 4 to 6, ignored otherwise) receives the clock the device held during the last launch
 *   mode 5  as mode 4 with 16x16x32 fragments instead of 32x32x16
 *   mode 6  as mode 5, but every work-group fetches the operand panels of tile (0, 0): all loads
 *           hit in L2 and nothing crosses the fabric (what the traffic beyond L2 costs)
 * For modes 1-3 the MFMAs run on the first K-steps' operands over and over, and in mode 6 every
 * tile is the product of the first panels: C is then NOT a GEMM result.  M, N multiples of 256, K a multiple of 64 and at least 128.  Two untimed launches, then
 * `iters` launches timed with HIP events one by one; ms_out[0 .. iters-1] (host) receives the
 * milliseconds.  Synchronises.  Not thread-safe against itself. */
int ks_bf16_ablation(int mode, const uint16_t *A_device, const uint16_t *B_device, float *C_device,
                     int64_t M, int64_t N, int64_t K, void *stream, int iters, float *ms_out,
                     double *mhz_out);

/* ---------------------------------------------------------------- workspace
 * Split-K kernels (K partitioned over work-groups, partial sums reduced in a fixed order, no
 * atomics) need split_k * batch * M * N floats of scratch.  The caller registers one device
 * buffer per process (at least 4-byte aligned; 16-byte alignment lets the reduction pass use
 * 16-byte accesses); NULL / 0 unregisters.  Kernels with split_k == 1 never touch it. */
int ks_set_workspace(void *device_ptr, size_t bytes);
/* Bytes the kernel would like for this output size (for split_k == 0 the most it can use: the
 * partial sums of the largest partition count it may choose, or, for a 16-bit member that launches
 * in the hybrid form on this many tiles, the compact partial tiles of at most 16 partitions of its
 * last round; for a member with a balanced persistent form, the raw tiles of its work-groups). */
size_t ks_workspace_bytes_needed(int dtype, int kernel_id, int64_t M, int64_t N, int64_t batch);

/* ---------------------------------------------------------------- offline tuner (host only)
 * Sections II-A, III, III-A, IV on a timing table.  All arrays are host memory, row-major.
 *   perf       rows x cols, performance of configuration c on workload s (any positive unit)
 *   features   rows x n_features int64 feature vectors (ks_features layout, any prefix length)
 * Trees are CART with integer thresholds floor(midpoint); "x <= t" goes left.  Ties: argmax ->
 * lowest index; a split replaces the current best only if its gain is larger by a relative
 * 1e-9; best-first priority ties -> earliest node.  Fully deterministic. */

/* Section II-A: the performance of configuration c on workload s from its measured time,
 * out[s][c] = 2 * M * N * K * batch / seconds[s][c] (flop/s).  sizes: rows x 4 int64 (M, N, K, batch);
 * seconds: rows x cols, every entry positive. */
int ks_tune_performance(const int64_t *sizes, const double *seconds, int rows, int cols, double *out);

/* Section II-A: out[s][c] = perf[s][c] / max_c perf[s][c]. */
int ks_tune_normalise(const double *perf, int rows, int cols, double *out);

/* Section III (decision-tree pruning): fit a multi-output regression tree on `normalised`
 * with at most max_leaves leaves (best-first), take each leaf's mean vector as a cluster
 * representative and keep its best configuration.  kept_out (capacity max_leaves) receives the
 * sorted distinct kept ids; returns how many, or a negative status.  If tree_out != NULL
 * (capacity 2*max_leaves - 1 nodes) it receives the regression tree, leaf `value` = the
 * representative's best configuration. */
int ks_tune_prune_tree(const int64_t *features, int n_features, const double *normalised,
                       int rows, int cols, int max_leaves, int min_samples_leaf,
                       int32_t *kept_out, ks_tree_node_t *tree_out, int *tree_nodes_out);

/* Section III, the methods the decision tree is compared with.  Each writes the sorted distinct
 * kept ids to kept_out (capacity n) and returns how many, or a negative status.
 *   top_n:   the n configurations that are optimal for the most rows (equal counts -> lowest id;
 *            configurations that never win are not kept).
 *   kmeans:  Lloyd's k-means with n clusters on the rows of `normalised`, deterministic maximin
 *            seeding (first centre: row nearest to the mean; next: row farthest from its nearest
 *            centre; lowest row on ties), stop when no row changes cluster or after max_iter.
 *            pca_dims == 0: cluster in configuration space and keep each centroid's best
 *            configuration.  pca_dims > 0: cluster in the coordinates of that many leading
 *            principal components (covariance of the centred rows), map each centroid back
 *            (mean + coordinates . components) and keep its best configuration. */
int ks_tune_prune_top_n(const double *normalised, int rows, int cols, int n, int32_t *kept_out);
int ks_tune_prune_kmeans(const double *normalised, int rows, int cols, int n, int pca_dims,
                         int max_iter, int32_t *kept_out);

/*   hdbscan: density-based clustering of the rows of `normalised` (core distance to the
 *            min_samples-th nearest row, itself included; mutual reachability; minimum spanning tree;
 *            condensed single-linkage tree with min_cluster_size; excess-of-mass selection, the root
 *            never selected), in which the number of clusters is a result; each cluster's centroid
 *            contributes its best configuration, rows labelled noise take no part, and with no
 *            cluster at all the centroid of all rows is used.  labels_out (rows entries, may be NULL)
 *            receives the cluster of every row, numbered by first member, or -1 for noise.
 *            kept_cap: capacity of kept_out.  KS_ERR_UNSUPPORTED above about 22000 rows (the
 *            distance matrix is dense). */
int ks_tune_prune_hdbscan(const double *normalised, int rows, int cols, int min_cluster_size,
                          int min_samples, int32_t *kept_out, int kept_cap, int32_t *labels_out);

/* Section II-B: fraction of the total variance of the rows of `normalised` carried by each
 * principal component, descending (ratio_out: cols doubles). */
int ks_tune_pca_variance(const double *normalised, int rows, int cols, double *ratio_out);

/* Section III-A score: geometric mean over rows of max_{c in kept} normalised[s][c]. */
int ks_tune_achievable(const double *normalised, int rows, int cols, const int32_t *kept,
                       int n_kept, double *score_out);

/* Section IV: label each row with its fastest kept configuration and fit a Gini
 * classification tree (depth-first, max_depth, min_samples_leaf).  row_weight may be NULL
 * (every row counts 1, the paper's setting) or give one non-negative weight per row.
 * Writes at most cap nodes to tree_out and returns the node count, or a negative status. */
int ks_tune_fit_selector(const int64_t *features, int n_features, const double *perf, int rows,
                         int cols, const int32_t *kept, int n_kept, int max_depth,
                         int min_samples_leaf, const double *row_weight,
                         ks_tree_node_t *tree_out, int cap);

/* Walk `tree` for every row; chosen_out[s] = leaf value. */
int ks_tune_predict(const ks_tree_node_t *tree, int n_nodes, const int64_t *features,
                    int n_features, int rows, int32_t *chosen_out);

/* Table I score: geometric mean over rows of normalised[s][chosen[s]]. */
int ks_tune_selector_score(const double *normalised, int rows, int cols, const int32_t *chosen,
                           double *score_out);

const char *ks_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* KS_GEMM_H */
