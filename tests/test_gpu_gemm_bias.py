"""GPU parity of ks_gemm_bias (fused fully-connected bias, Section II-A) against the fp64 CPU oracle:
every instantiation of both dtypes on ragged shapes spanning several tiles, both transposes, batch,
alpha / beta, K = 0, split-K members (bias applied by the reduction pass), and the selector path."""
import itertools

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


def bias_of(p, seed):
    return (3.0 * wl.uniform_pm1(p.N, 4000 + seed, 5)).astype(np.float32)


def oracle_bias(p, bias):
    from oracle import gemm as og
    C = p.C0.copy()
    og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C,
                 p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    return C


def run_bias(gpu, dp, kid, bias_dev):
    import torch
    import paper_2003_06795_amd.binding as ks
    p = dp.p
    C = dp.C0.clone()
    ks.gemm_bias(gpu.DT[p.dtype], -1 if kid is None else kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha,
                 dp.A, p.lda, dp.B, p.ldb, p.beta, C, p.ldc, bias_dev, p.batch, p.strideA, p.strideB,
                 p.strideC)
    torch.cuda.synchronize()
    return C.cpu().numpy()[:p.C0.size]


def check(p, bias, got, ref, what):
    live = ~c_padding_mask(p)
    # the stated GEMM bound plus the roundings of the final fp32 add
    tol = tolerance(p) + 2.0 ** -22 * (float(np.max(np.abs(bias))) + float(np.max(np.abs(ref[live]))))
    err = float(np.max(np.abs(got[live].astype(np.float64) - ref[live].astype(np.float64))))
    assert np.all(np.isfinite(got[live])), what
    assert err <= tol, "%s: max|diff| %.3e > tol %.3e" % (what, err, tol)
    mask = c_padding_mask(p)
    assert np.array_equal(got[mask], p.C0[mask], equal_nan=True), what + ": wrote outside C's logical entries"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_every_kernel_with_bias(gpu, dtype, tA, tB):
    import torch
    import paper_2003_06795_amd.binding as ks
    # ragged in M and N (several 16 / 32 / 64 tiles plus a tail), K not a multiple of any K-step
    p = wl.make_problem(dtype, tA, tB, 150, 201, 203 if dtype == "f32" else 264, batch=2, alpha=0.5,
                        beta=-1.25, seed=31, key=2 * tA + tB, pad=(0, 0, 3),
                        dist="normal" if dtype == "bf16" else "uniform")
    bias = bias_of(p, 2 * tA + tB)
    bias_dev = torch.from_numpy(bias).cuda()
    dp, ref = gpu.DeviceProblem(p), oracle_bias(p, bias)
    for kid in range(ks.num_kernels(gpu.DT[dtype])):
        need = ks.workspace_bytes_needed(gpu.DT[dtype], kid, p.M, p.N, p.batch)
        if need:
            gpu.ensure_workspace(need)
        print("bias", dtype, tA, tB, "kernel", kid, flush=True)
        check(p, bias, run_bias(gpu, dp, kid, bias_dev), ref, "%s kernel %d" % (dtype, kid))
    check(p, bias, run_bias(gpu, dp, None, bias_dev), ref, "%s selector" % dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bias_aligned_fast_paths_beta_zero_and_k_zero(gpu, dtype):
    import torch
    import paper_2003_06795_amd.binding as ks
    # aligned shape (vector loads, direct-to-LDS bf16 path), beta = 0 over NaN-filled C
    p = wl.make_problem(dtype, 0, 1, 256, 192, 256, alpha=1.0, beta=0.0, seed=5, c_fill="nan",
                        dist="normal" if dtype == "bf16" else "uniform")
    bias = bias_of(p, 9)
    bias_dev = torch.from_numpy(bias).cuda()
    dp, ref = gpu.DeviceProblem(p), oracle_bias(p, bias)
    for kid in range(ks.num_kernels(gpu.DT[dtype])):
        need = ks.workspace_bytes_needed(gpu.DT[dtype], kid, p.M, p.N, p.batch)
        if need:
            gpu.ensure_workspace(need)
        check(p, bias, run_bias(gpu, dp, kid, bias_dev), ref, "%s kernel %d aligned" % (dtype, kid))
    # K = 0: C = beta * C + bias
    q = wl.make_problem(dtype, 0, 0, 19, 33, 0, batch=2, alpha=2.0, beta=0.5, seed=6)
    bq = bias_of(q, 10)
    dq = gpu.DeviceProblem(q)
    check(q, bq, run_bias(gpu, dq, 0, torch.from_numpy(bq).cuda()), oracle_bias(q, bq), "K = 0")
    # a null bias is the plain GEMM, bit for bit
    assert np.array_equal(run_bias(gpu, dp, 3, None), dp.run(3), equal_nan=True)


def test_bias_small_integers_are_exact(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f32", 1, 0, 70, 90, 40, alpha=2.0, beta=0.0, seed=7, dist="ints")
    bias = np.arange(-45, 45, dtype=np.float32)
    dp, ref = gpu.DeviceProblem(p), oracle_bias(p, bias)
    live = ~c_padding_mask(p)
    for kid in range(ks.num_kernels(ks.F32)):
        need = ks.workspace_bytes_needed(ks.F32, kid, p.M, p.N, p.batch)
        if need:
            gpu.ensure_workspace(need)
        got = run_bias(gpu, dp, kid, torch.from_numpy(bias).cuda())
        assert np.array_equal(got[live], ref[live]), "kernel %d" % kid
