"""GPU parity of ks_gemm_out_bf16 (C read and written as bf16) against the fp64 CPU oracle's
bf16-output form: every instantiation for fp32, bf16 and fp16 operands, ragged batched shapes with
alpha, beta and a bias, split-K members (rounding happens in the reduction pass), K = 0, and
integer cases in which the rounding decision must agree bit for bit."""
import numpy as np
import pytest

import workloads as wl
from helpers import c_padding_mask, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def run_out16(gpu, dp, kid, C16_host, bias):
    import torch
    import paper_2003_06795_amd.binding as ks
    p = dp.p
    C = torch.from_numpy(C16_host.view(np.int16).copy()).cuda()
    b = None if bias is None else torch.from_numpy(bias).cuda()
    ks.gemm_out_bf16(gpu.DT[p.dtype], -1 if kid is None else kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha,
                     dp.A, p.lda, dp.B, p.ldb, p.beta, C, p.ldc, b, p.batch, p.strideA, p.strideB, p.strideC)
    torch.cuda.synchronize()
    return C.cpu().numpy().view(np.uint16)


def oracle_out16(p, C16_host, bias):
    from oracle import gemm as og
    C = C16_host.copy()
    og.gemm_out_bf16(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C,
                     p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    return C


def prep(gpu, p, kid):
    import paper_2003_06795_amd.binding as ks
    need = ks.workspace_bytes_needed(gpu.DT[p.dtype], kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_every_kernel_within_one_bf16_step(gpu, dtype):
    import paper_2003_06795_amd.binding as ks
    for (tA, tB) in ((0, 0), (1, 1), (0, 1)):
        p = wl.make_problem(dtype, tA, tB, 150, 201, 203 if dtype == "f32" else 264, batch=2, alpha=0.5,
                            beta=-1.25, seed=61, key=2 * tA + tB, pad=(0, 0, 3),
                            dist="uniform" if dtype == "f32" else "normal")
        bias = (3.0 * wl.uniform_pm1(p.N, 62, tA)).astype(np.float32)
        C16 = wl.f32_to_bf16_rne(p.C0)
        ref = oracle_out16(p, C16, bias)
        dp = gpu.DeviceProblem(p)
        live = ~c_padding_mask(p)
        reff = wl.bf16_to_f32(ref).astype(np.float64)
        for kid in list(range(ks.num_kernels(gpu.DT[dtype]))) + [None]:
            if kid is not None:
                prep(gpu, p, kid)
            print("out16", dtype, tA, tB, "kernel", kid, flush=True)
            got = run_out16(gpu, dp, kid, C16, bias)
            assert np.array_equal(got[~live], C16[~live]), "kernel %s wrote outside C" % kid
            gotf = wl.bf16_to_f32(got).astype(np.float64)
            # the fp32 result may sit on the other side of a rounding boundary: one bf16 step
            # (2^-7 relative) on top of the fp32 path's own bound
            err = np.abs(gotf[live] - reff[live])
            bound = tolerance(p) + 2.0 ** -22 * 4.0 + 2.0 ** -7 * np.abs(reff[live])
            assert np.all(np.isfinite(gotf[live])) and np.all(err <= bound), "%s kernel %s" % (dtype, kid)
            # and most entries agree exactly
            assert np.mean(got[live] == ref[live]) > 0.97, "%s kernel %s" % (dtype, kid)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_integer_sums_round_identically(gpu, dtype):
    import paper_2003_06795_amd.binding as ks
    # exact integer sums up to a few thousand: not representable in bf16's 8 bits, so every entry
    # is a rounding decision taken from the same exact value on both sides
    p = wl.make_problem(dtype, 1, 0, 96, 80, 64, alpha=1.0, beta=0.0, seed=63, dist="ints", c_fill="nan")
    bias = np.arange(-40, 40, dtype=np.float32)
    C16 = np.full(p.C0.size, 0x7FC0, dtype=np.uint16)
    ref = oracle_out16(p, C16, bias)
    dp = gpu.DeviceProblem(p)
    for kid in range(ks.num_kernels(gpu.DT[dtype])):
        prep(gpu, p, kid)
        assert np.array_equal(run_out16(gpu, dp, kid, C16, bias), ref), "%s kernel %d" % (dtype, kid)


def test_k_zero_and_null_bias(gpu):
    p = wl.make_problem("bf16", 0, 0, 9, 17, 0, batch=2, alpha=2.0, beta=0.5, seed=64)
    C16 = wl.f32_to_bf16_rne(p.C0)
    dp = gpu.DeviceProblem(p)
    assert np.array_equal(run_out16(gpu, dp, 0, C16, None), oracle_out16(p, C16, None))
    bias = wl.uniform_pm1(p.N, 65, 0)
    assert np.array_equal(run_out16(gpu, dp, 3, C16, bias), oracle_out16(p, C16, bias))
