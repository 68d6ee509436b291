// Measurement aids behind the C ABI: what the matrix pipe alone sustains on given operand values.
// Nothing here is on the GEMM path.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/ks_gemm.h"
#include "gemm_bf16_pp.hpp"

namespace ks {
namespace {

__device__ unsigned long long g_probeClocks[2];      // shader clocks, 100 MHz reference ticks (work-group 0)

// Every wave loads twelve 16-byte operand fragments per lane once (what one K-step of a 128 x 64
// wave tile holds), then issues `rounds` x 32 MFMAs on them into eight accumulator fragments:
// no LDS, no memory traffic, two waves per SIMD.  KIND 0: 32x32x16 bf16, 1: 32x32x16 f16,
// 2: 32x32x2 f32, 3: 16x16x32 bf16, 4: 16x16x32 f16 (thirty-two 16 x 16 accumulator fragments, the
// same number of matrix-pipe passes per round, half the flops per instruction).
template <int KIND>
__global__ __launch_bounds__(512) void mfma_sustained_kernel(const uintx4 *src, int rounds, float *sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uintx4 *mine = src + ((size_t)((blockIdx.x & 63) * 8 + wave) * 12) * 64 + lane;
    uintx4 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = mine[i * 64];
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = mine[(8 + i) * 64];
    floatx16 acc[KIND >= 3 ? 1 : 8];
    floatx4 acc4[KIND >= 3 ? 32 : 1];
#pragma unroll
    for (int i = 0; i < (KIND >= 3 ? 1 : 8); ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
#pragma unroll
    for (int i = 0; i < (KIND >= 3 ? 32 : 1); ++i) acc4[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    unsigned long long c0 = 0, r0 = 0;
    const bool stamp = blockIdx.x == 0 && threadIdx.x == 0;
    if (stamp) { c0 = __builtin_amdgcn_s_memtime(); r0 = __builtin_amdgcn_s_memrealtime(); }
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    if constexpr (KIND >= 3) {
                        floatx4 &c4 = acc4[(q * 4 + ks) * 2 + m];
                        c4 = mfma_16x16x32<KIND == 4>(__builtin_bit_cast(bf16x8, a[m * 4 + ks]),
                                                      __builtin_bit_cast(bf16x8, b[ks]), c4);
                        continue;
                    }
                    floatx16 &c = acc[KIND >= 3 ? 0 : q * 2 + m];
                    if constexpr (KIND == 2)
                        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a[m * 4 + ks][q]),
                                                                 __builtin_bit_cast(float, b[ks][q]), c, 0, 0, 0);
                    else
                        c = mfma_32x32x16<KIND == 1>(__builtin_bit_cast(bf16x8, a[m * 4 + ks]),
                                                     __builtin_bit_cast(bf16x8, b[ks]), c);
                }
    }
    if (stamp) {
        g_probeClocks[0] = __builtin_amdgcn_s_memtime() - c0;
        g_probeClocks[1] = __builtin_amdgcn_s_memrealtime() - r0;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < (KIND >= 3 ? 1 : 8); ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
#pragma unroll
    for (int i = 0; i < (KIND >= 3 ? 32 : 1); ++i) s += acc4[i][0] + acc4[i][1] + acc4[i][2] + acc4[i][3];
    if (sink != nullptr && s == 123.4567f) sink[threadIdx.x] = s;     // keeps the accumulators alive
}

std::mutex g_probeMutex;

}  // namespace
}  // namespace ks

using namespace ks;

extern "C" int ks_mfma_sustained(int dtype, int fragment, const void *operands_device, size_t bytes, int rounds,
                                 void *stream, double *tflops_out, double *mhz_out) {
    if (dtype != KS_F32 && dtype != KS_BF16 && dtype != KS_F16) return KS_ERR_INVALID_ARG;
    if (fragment != 32 && !(fragment == 16 && dtype != KS_F32)) return KS_ERR_INVALID_ARG;
    if (!operands_device || bytes < KS_MFMA_PROBE_BYTES || rounds < 1 || rounds > (1 << 24) || !tflops_out)
        return KS_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(operands_device) % 16) return KS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_probeMutex);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    (void)hipGetLastError();
    if (hipEventCreate(&e0) != hipSuccess) return KS_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return KS_ERR_LAUNCH; }
    const int groups = 256 * 8;
    const uintx4 *src = static_cast<const uintx4 *>(operands_device);
    int rc = KS_OK;
    float ms = 0.f;
    for (int pass = 0; pass < 2 && rc == KS_OK; ++pass) {            // the first pass settles the clock
        if (hipEventRecord(e0, s) != hipSuccess) rc = KS_ERR_LAUNCH;
        if (dtype == KS_BF16 && fragment == 16) hipLaunchKernelGGL(mfma_sustained_kernel<3>, dim3(groups), dim3(512), 0, s, src, rounds, (float *)nullptr);
        else if (dtype == KS_F16 && fragment == 16) hipLaunchKernelGGL(mfma_sustained_kernel<4>, dim3(groups), dim3(512), 0, s, src, rounds, (float *)nullptr);
        else if (dtype == KS_BF16) hipLaunchKernelGGL(mfma_sustained_kernel<0>, dim3(groups), dim3(512), 0, s, src, rounds, (float *)nullptr);
        else if (dtype == KS_F16) hipLaunchKernelGGL(mfma_sustained_kernel<1>, dim3(groups), dim3(512), 0, s, src, rounds, (float *)nullptr);
        else hipLaunchKernelGGL(mfma_sustained_kernel<2>, dim3(groups), dim3(512), 0, s, src, rounds, (float *)nullptr);
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
            rc = KS_ERR_LAUNCH;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != KS_OK) return rc;
    const double flopPerMfma = dtype == KS_F32 ? 2.0 * 32 * 32 * 2 : fragment == 16 ? 2.0 * 16 * 16 * 32 : 2.0 * 32 * 32 * 16;
    *tflops_out = (double)groups * 8 * (double)rounds * 32 * flopPerMfma / ((double)ms * 1e-3) / 1e12;
    if (mhz_out) {
        unsigned long long h[2] = {0, 0};
        if (hipMemcpyFromSymbol(h, HIP_SYMBOL(g_probeClocks), sizeof(h)) != hipSuccess) return KS_ERR_LAUNCH;
        *mhz_out = h[1] ? (double)h[0] / ((double)h[1] * 0.01) : 0.0;
    }
    return KS_OK;
}

extern "C" int ks_bf16_ablation(int mode, const uint16_t *A, const uint16_t *B, float *C, int64_t M, int64_t N,
                                int64_t K, void *stream, int iters, float *ms_out, double *mhz_out) {
    if (mode < 0 || mode > 6 || !A || !B || !C || !ms_out || iters < 1 || iters > 1024) return KS_ERR_INVALID_ARG;
    if (mode >= 4 && !mhz_out) return KS_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K < 128 || M % 256 || N % 256 || K % 64 || M > 65536 || N > 65536 || K > (1 << 22))
        return KS_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(A) % 16 || reinterpret_cast<uintptr_t>(B) % 16) return KS_ERR_INVALID_ARG;
    GemmParams p{};
    p.A = A; p.B = B; p.C = C;
    p.lda = K; p.ldb = K; p.ldc = N;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.batch = 1;
    p.tilesM = (int)(M / 256); p.tilesN = (int)(N / 256);
    p.splitK = 1; p.kChunk = (int)K; p.grid3d = 0; p.tilesPerWG = 1; p.bandRows = 8;
    p.alpha = 1.0f; p.beta = 0.0f;
    const dim3 grid((unsigned)(p.tilesM * p.tilesN)), block(512);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    (void)hipGetLastError();
    if (hipEventCreate(&e0) != hipSuccess) return KS_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return KS_ERR_LAUNCH; }
    int rc = KS_OK;
    for (int it = -2; it < iters && rc == KS_OK; ++it) {             // two untimed launches first
        if (hipEventRecord(e0, s) != hipSuccess) rc = KS_ERR_LAUNCH;
        switch (mode) {
            case 0: hipLaunchKernelGGL((gemm_bf16_pp_kernel<32, false, true, true, false, 0>), grid, block, 0, s, p); break;
            case 1: hipLaunchKernelGGL((gemm_bf16_pp_kernel<32, false, true, true, false, 1>), grid, block, 0, s, p); break;
            case 2: hipLaunchKernelGGL((gemm_bf16_pp_kernel<32, false, true, true, false, 2>), grid, block, 0, s, p); break;
            case 3: hipLaunchKernelGGL((gemm_bf16_pp_kernel<32, false, true, true, false, 3>), grid, block, 0, s, p); break;
            case 4: hipLaunchKernelGGL((gemm_bf16_pp_kernel<32, false, true, true, false, 4>), grid, block, 0, s, p); break;
            case 5: hipLaunchKernelGGL((gemm_bf16_pp_kernel<16, false, true, true, false, 4>), grid, block, 0, s, p); break;
            default: hipLaunchKernelGGL((gemm_bf16_pp_kernel<16, false, true, true, false, 12>), grid, block, 0, s, p); break;
        }
        float ms = 0.f;
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
            rc = KS_ERR_LAUNCH;
        if (it >= 0) ms_out[it] = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == KS_OK && mode >= 4) {
        // clock of work-group 0 during the K loop of the last launch
        unsigned long long h[2] = {0, 0};
        if (hipMemcpyFromSymbol(h, HIP_SYMBOL(pp_probe_clocks), sizeof(h)) != hipSuccess) return KS_ERR_LAUNCH;
        *mhz_out = h[1] ? (double)h[0] / ((double)h[1] * 0.01) : 0.0;
    }
    return rc;
}
