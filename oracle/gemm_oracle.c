/*
 * CPU oracle for the general matrix multiply of the paper's case study
 * (Section II, "A matrix multiply case study"): the result every tiled kernel
 * of the family must reproduce,
 *
 *     C_b = alpha * op(A_b) * op(B_b) + beta * C_b        for b in [0, batch)
 *
 * written out as the plain definition: one fp64 dot product per output entry,
 * summed in increasing k, no blocking, no reordering.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it shares no code with the HIP kernels or their host dispatch.
 *
 * Conventions (the paper only says "general matrix multiply"; these are the
 * readings the whole repository uses):
 *   - row-major storage.  op(A) is M x K: transA == 0 -> A stored M x K with
 *     row stride lda >= K; transA == 1 -> A stored K x M with lda >= M.
 *     op(B) is K x N: transB == 0 -> stored K x N, ldb >= N; transB == 1 ->
 *     stored N x K, ldb >= K.  C is M x N with ldc >= N.
 *   - batch item b starts at A + b*strideA, B + b*strideB, C + b*strideC
 *     (strides in elements; strideA/strideB may be 0 = broadcast).
 *   - beta == 0 means C is not read (NaN/Inf already in C do not propagate).
 *   - alpha == 0 gets no special case: 0 * acc is computed.
 *   - bf16 operands are widened exactly (bf16 is the top 16 bits of an fp32).
 *   - fp16 operands (IEEE 754 binary16: 1 sign, 5 exponent, 10 fraction bits,
 *     bias 15, subnormals, infinities and NaNs) are widened exactly as well.
 *   - the fp64 value alpha*acc + beta*c0 is rounded once to fp32 on store.
 *   - the *_out_bf16 entry points keep C in bf16: the old value (read only when
 *     beta != 0) is widened exactly, and the fp64 value alpha*acc + beta*c0 + bias[j]
 *     is rounded ONCE to bf16, to nearest with ties to even (8 significant bits,
 *     fp32's exponent range, subnormals; overflow goes to infinity).  Mixed
 *     precision of this kind is what Section II's remark that the kernel is
 *     templated over its data type leaves open; the reading is ours.
 *   - the *_bias entry points add a length-N fp32 vector to every row of every
 *     batch item, out[b][i][j] = alpha*acc + beta*c0 + bias[j]: the bias of a
 *     fully-connected layer whose weights are op(B) (Section II-A lists
 *     fully-connected layers among the sources of the GEMM shapes).  The sum is
 *     formed in fp64 and still rounded once.  bias == NULL adds nothing.
 *
 * Returns 0, or -1 on an argument that makes the definition meaningless.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#include <math.h>

static inline double widen_f32(const void *p, int64_t idx) {
    return (double)((const float *)p)[idx];
}

static inline double widen_bf16(const void *p, int64_t idx) {
    uint32_t bits = (uint32_t)((const uint16_t *)p)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* binary16 -> double from the bit fields: (-1)^s * 2^(e-15) * (1 + f/1024) for 0 < e < 31,
 * (-1)^s * 2^-14 * (f/1024) for e == 0, infinity / NaN for e == 31 */
static inline double widen_f16(const void *p, int64_t idx) {
    uint16_t h = ((const uint16_t *)p)[idx];
    int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 31) {
        v = f ? (double)NAN : (double)INFINITY;
    } else if (e == 0) {
        v = ldexp((double)f, -24);
    } else {
        v = ldexp((double)(1024 + f), e - 25);
    }
    return sign ? -v : v;
}

/* double -> bf16 bit pattern, round to nearest even, by the format's definition */
static uint16_t round_to_bf16(double x) {
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x)) return 0x7FC0u;
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = m * 2^e, 0.5 <= m < 1  ->  floor(log2 a) = e - 1 */
    int ex = e - 1;
    if (ex < -126) ex = -126;           /* subnormal spacing */
    double q = ldexp(1.0, ex - 7);      /* spacing of bf16 values in this binade */
    double n = nearbyint(a / q);        /* default rounding mode: to nearest, ties to even */
    double v = n * q;
    if (v >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    float f = (float)v;                 /* exact: v has at most 8 significant bits */
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (uint16_t)(sign | (bits >> 16));
}

uint16_t oracle_round_to_bf16(double x) { return round_to_bf16(x); }

typedef double (*widen_fn)(const void *, int64_t);

static int check_args(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc, int64_t batch) {
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return -1;
    if (M < 0 || N < 0 || K < 0 || batch < 0) return -1;
    if (M > 0 && K > 0 && lda < (transA ? M : K)) return -1;
    if (N > 0 && K > 0 && ldb < (transB ? K : N)) return -1;
    if (M > 0 && N > 0 && ldc < N) return -1;
    return 0;
}

/* one entry of op(A)*op(B) for one batch item, fp64, increasing k */
static double dot_entry(widen_fn w, int transA, int transB, int64_t K,
                        const void *A, int64_t offA, int64_t lda,
                        const void *B, int64_t offB, int64_t ldb,
                        int64_t i, int64_t j) {
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        int64_t ia = transA ? (k * lda + i) : (i * lda + k);
        int64_t ib = transB ? (j * ldb + k) : (k * ldb + j);
        acc += w(A, offA + ia) * w(B, offB + ib);
    }
    return acc;
}

static int gemm_any(widen_fn w, int transA, int transB, int64_t M, int64_t N, int64_t K,
                    float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                    float beta, float *C, int64_t ldc, int64_t batch,
                    int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    if (check_args(transA, transB, M, N, K, lda, ldb, ldc, batch)) return -1;
    if (M == 0 || N == 0 || batch == 0) return 0;
    int64_t rows = batch * M;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / M, i = r % M;
        for (int64_t j = 0; j < N; ++j) {
            double acc = dot_entry(w, transA, transB, K, A, b * strideA, lda,
                                   B, b * strideB, ldb, i, j);
            float *c = C + b * strideC + i * ldc + j;
            double out = (double)alpha * acc;
            if (beta != 0.0f) out += (double)beta * (double)*c;
            if (bias) out += (double)bias[j];
            *c = (float)out;
        }
    }
    return 0;
}

int oracle_gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                    float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                    float beta, float *C, int64_t ldc, int64_t batch,
                    int64_t strideA, int64_t strideB, int64_t strideC) {
    return gemm_any(widen_f32, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                    batch, strideA, strideB, strideC, NULL);
}

int oracle_gemm_bias_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                         float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                         float beta, float *C, int64_t ldc, int64_t batch,
                         int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    return gemm_any(widen_f32, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                    batch, strideA, strideB, strideC, bias);
}

int oracle_gemm_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                     float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                     float beta, float *C, int64_t ldc, int64_t batch,
                     int64_t strideA, int64_t strideB, int64_t strideC) {
    return gemm_any(widen_bf16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                    batch, strideA, strideB, strideC, NULL);
}

int oracle_gemm_bias_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                          float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                          float beta, float *C, int64_t ldc, int64_t batch,
                          int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    return gemm_any(widen_bf16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                    batch, strideA, strideB, strideC, bias);
}

int oracle_gemm_bias_f16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                         float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                         float beta, float *C, int64_t ldc, int64_t batch,
                         int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    return gemm_any(widen_f16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                    batch, strideA, strideB, strideC, bias);
}

/* C kept in bf16 (see the header): in place on C16 */
static int gemm_out16_any(widen_fn w, int transA, int transB, int64_t M, int64_t N, int64_t K,
                          float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                          float beta, uint16_t *C16, int64_t ldc, int64_t batch,
                          int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    if (check_args(transA, transB, M, N, K, lda, ldb, ldc, batch)) return -1;
    if (M == 0 || N == 0 || batch == 0) return 0;
    int64_t rows = batch * M;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / M, i = r % M;
        for (int64_t j = 0; j < N; ++j) {
            double acc = dot_entry(w, transA, transB, K, A, b * strideA, lda,
                                   B, b * strideB, ldb, i, j);
            uint16_t *c = C16 + b * strideC + i * ldc + j;
            double out = (double)alpha * acc;
            if (beta != 0.0f) out += (double)beta * widen_bf16(c, 0);
            if (bias) out += (double)bias[j];
            *c = round_to_bf16(out);
        }
    }
    return 0;
}

int oracle_gemm_out_bf16(int in_dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                         float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                         float beta, uint16_t *C16, int64_t ldc, int64_t batch,
                         int64_t strideA, int64_t strideB, int64_t strideC, const float *bias) {
    widen_fn w = in_dtype == 0 ? widen_f32 : in_dtype == 1 ? widen_bf16 : in_dtype == 2 ? widen_f16 : NULL;
    if (!w) return -1;
    return gemm_out16_any(w, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C16, ldc,
                          batch, strideA, strideB, strideC, bias);
}

/* one fp16 bit pattern widened, for the pins of the conversion itself */
double oracle_widen_f16(uint16_t bits) { return widen_f16(&bits, 0); }

/*
 * The same definition for a list of n output entries (b[t], i[t], j[t]) only:
 * out[t] = (float)(alpha * dot + beta * C0[b,i,j]).  C0 is the output buffer
 * as it was before the GEMM (only read when beta != 0; may be NULL otherwise).
 * Used to check full-size problems entry by entry without the full triple loop.
 */
static int entries_any(widen_fn w, int transA, int transB, int64_t M, int64_t N, int64_t K,
                       float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                       float beta, const float *C0, int64_t ldc, int64_t batch,
                       int64_t strideA, int64_t strideB, int64_t strideC,
                       int64_t n, const int64_t *bb, const int64_t *ii, const int64_t *jj,
                       float *out) {
    if (check_args(transA, transB, M, N, K, lda, ldb, ldc, batch)) return -1;
    if (n < 0) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (bb[t] < 0 || bb[t] >= batch || ii[t] < 0 || ii[t] >= M || jj[t] < 0 || jj[t] >= N)
            return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double acc = dot_entry(w, transA, transB, K, A, bb[t] * strideA, lda,
                               B, bb[t] * strideB, ldb, ii[t], jj[t]);
        double o = (double)alpha * acc;
        if (beta != 0.0f) o += (double)beta * (double)C0[bb[t] * strideC + ii[t] * ldc + jj[t]];
        out[t] = (float)o;
    }
    return 0;
}

int oracle_gemm_f32_entries(int transA, int transB, int64_t M, int64_t N, int64_t K,
                            float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                            float beta, const float *C0, int64_t ldc, int64_t batch,
                            int64_t strideA, int64_t strideB, int64_t strideC,
                            int64_t n, const int64_t *bb, const int64_t *ii, const int64_t *jj,
                            float *out) {
    return entries_any(widen_f32, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc,
                       batch, strideA, strideB, strideC, n, bb, ii, jj, out);
}

int oracle_gemm_bf16_entries(int transA, int transB, int64_t M, int64_t N, int64_t K,
                             float alpha, const uint16_t *A, int64_t lda, const uint16_t *B,
                             int64_t ldb, float beta, const float *C0, int64_t ldc, int64_t batch,
                             int64_t strideA, int64_t strideB, int64_t strideC,
                             int64_t n, const int64_t *bb, const int64_t *ii, const int64_t *jj,
                             float *out) {
    return entries_any(widen_bf16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc,
                       batch, strideA, strideB, strideC, n, bb, ii, jj, out);
}

int oracle_gemm_f16_entries(int transA, int transB, int64_t M, int64_t N, int64_t K,
                            float alpha, const uint16_t *A, int64_t lda, const uint16_t *B,
                            int64_t ldb, float beta, const float *C0, int64_t ldc, int64_t batch,
                            int64_t strideA, int64_t strideB, int64_t strideC,
                            int64_t n, const int64_t *bb, const int64_t *ii, const int64_t *jj,
                            float *out) {
    return entries_any(widen_f16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc,
                       batch, strideA, strideB, strideC, n, bb, ii, jj, out);
}

/* threads the parallel loops above will use (1 when built without OpenMP) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
