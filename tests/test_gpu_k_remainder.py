"""16-bit GEMMs whose K is not a whole number of the member's K-steps: the remainder of K runs
first through the general kernel (alpha, beta, bias), the whole K-steps then on the direct-to-LDS
path with beta = 1.  Every 16-bit member against the oracle and against the general kernel over
all of K, and the cases that must not be cut."""
import numpy as np
import pytest

import workloads as wl
from helpers import tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    import paper_2003_06795_amd.binding as ks
    gpu_util.ensure_workspace(256 << 20)
    yield gpu_util
    ks.set_fast_path(True)


def plan_of(ks, gpu, p, dp, kid):
    return ks.gemm_plan(gpu.DT[p.dtype], kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                        p.beta, dp.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)


@pytest.mark.parametrize("layout", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_every_member_with_a_remainder_of_k(gpu, layout):
    import paper_2003_06795_amd.binding as ks
    for kid in range(ks.num_kernels(ks.BF16)):
        ki = ks.kernel_info(ks.BF16, kid)
        M, N = 2 * ki["bm"] + 8, ki["bn"] + 24
        K = 5 * ki["bk"] + 8 * (1 + kid % 7)                      # remainder 8 .. 56
        p = wl.make_problem("bf16", layout[0], layout[1], M, N, K, batch=1 + kid % 2, alpha=1.5, beta=-0.25,
                            seed=81, key=kid, dist="normal")
        dp = gpu.DeviceProblem(p)
        ks.set_fast_path(False)
        assert plan_of(ks, gpu, p, dp, kid)["k_remainder"] == 0
        general = dp.run(kid)
        ks.set_fast_path(True)
        plan = plan_of(ks, gpu, p, dp, kid)
        if layout == (0, 1):          # both operands K-contiguous: small outputs stay on the general kernel
            assert plan["k_remainder"] == 0 and plan["path"] == 0, (kid, plan)
        else:
            assert plan["k_remainder"] == K % ki["bk"] and plan["path"] >= 1, (kid, plan)
        got = dp.run(kid)
        tol = tolerance(p)
        ref = gpu.oracle_full(p).astype(np.float64)
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        assert err <= tol, "kernel %d %s: %.3e > %.3e" % (kid, (M, N, K), err, tol)
        assert float(np.max(np.abs(got.astype(np.float64) - general))) <= 2 * tol


def test_bias_fp16_and_the_cases_that_are_not_cut(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    from oracle import gemm as og
    ks.set_fast_path(True)
    kid = ks.select(ks.BF16, 1024, 1024, 1032, 1, 0, 0)
    ki = ks.kernel_info(ks.BF16, kid)
    bk = ki["bk"]
    # bias is applied once, by the first launch
    p = wl.make_problem("bf16", 0, 0, 328, 264, 6 * bk + 24, alpha=0.5, beta=0.75, seed=82, key=0, dist="normal")
    dp = gpu.DeviceProblem(p)
    assert plan_of(ks, gpu, p, dp, kid)["k_remainder"] == 24
    bias = wl.uniform_pm1(p.N, 82, 9, 0)
    C = dp.C0.clone()
    ks.gemm_bias(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, C, p.ldc,
                 torch.from_numpy(bias).cuda(), p.batch, p.strideA, p.strideB, p.strideC)
    torch.cuda.synchronize()
    ref = p.C0.copy()
    og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref, p.ldc, bias,
                 p.batch, p.strideA, p.strideB, p.strideC)
    assert float(np.max(np.abs(C.cpu().numpy().astype(np.float64) - ref))) <= tolerance(p) + 2.0 ** -22 * 4.0
    # fp16 inputs, the selecting entry point
    p = wl.make_problem("f16", 1, 0, 328, 264, 6 * bk + 40, alpha=1.0, beta=0.0, seed=82, key=1, dist="normal",
                        c_fill="nan")
    dp = gpu.DeviceProblem(p)
    got = dp.run()
    assert float(np.max(np.abs(got.astype(np.float64) - gpu.oracle_full(p)))) <= tolerance(p)
    # not cut: an output kept in bf16, fewer than four K-steps, K not a multiple of 8, fp32
    one = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(8, device="cuda")
    K = 6 * bk + 24
    assert ks.gemm_plan(ks.BF16, kid, 0, 0, 256, 256, K, 1.0, one, K, one, 256, 0.0, c, 256)["k_remainder"] == 24
    assert ks.gemm_plan(ks.BF16, kid, 0, 0, 256, 256, 3 * bk + 8, 1.0, one, 3 * bk + 8, one, 256, 0.0, c,
                        256)["k_remainder"] == 0
    assert ks.gemm_plan(ks.BF16, kid, 0, 0, 256, 256, K + 4, 1.0, one, K + 4, one, 256, 0.0, c, 256)["k_remainder"] == 0
    assert ks.gemm_plan(ks.BF16, kid, 0, 0, 256, 256, 6 * bk, 1.0, one, 6 * bk, one, 256, 0.0, c, 256)["k_remainder"] == 0
    # both operands K-contiguous: only large outputs are cut
    assert ks.gemm_plan(ks.BF16, kid, 0, 1, 2048, 2048, K, 1.0, one, K, one, K, 0.0, c, 2048)["k_remainder"] == 0
    assert ks.gemm_plan(ks.BF16, kid, 0, 1, 4096, 4096, K, 1.0, one, K, one, K, 0.0, c, 4096)["k_remainder"] == 24
    f = torch.zeros(8, device="cuda")
    assert ks.gemm_plan(ks.F32, 47, 0, 1, 256, 256, 1000, 1.0, f, 1000, f, 1000, 0.0, c, 256)["k_remainder"] == 0
    p = wl.make_problem("bf16", 0, 0, 136, 264, K, alpha=1.0, beta=0.5, seed=82, key=2, dist="normal")
    dp = gpu.DeviceProblem(p)
    C16 = wl.f32_to_bf16_rne(p.C0)
    ref16 = C16.copy()
    og.gemm_out_bf16(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref16, p.ldc,
                     None, p.batch, p.strideA, p.strideB, p.strideC)
    D = torch.from_numpy(C16.view(np.int16).copy()).cuda()
    ks.gemm_out_bf16(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, D,
                     p.ldc, None, p.batch, p.strideA, p.strideB, p.strideC)
    torch.cuda.synchronize()
    gotf = wl.bf16_to_f32(D.cpu().numpy().view(np.uint16)).astype(np.float64)
    reff = wl.bf16_to_f32(ref16).astype(np.float64)
    assert np.all(np.abs(gotf - reff) <= tolerance(p) + 2.0 ** -7 * np.abs(reff))


def test_cut_k_together_with_a_hybrid_launch(gpu):
    """The whole K-steps of a cut call may themselves launch in the hybrid form (partly filled last
    round partitioned along K): four kernels in a row on one output."""
    import paper_2003_06795_amd.binding as ks
    ks.set_fast_path(True)
    ks.set_tail_split(-1)
    big = [i for i in range(ks.num_kernels(ks.BF16)) if ks.kernel_info(ks.BF16, i)["split_k"] == 0 and
           ks.kernel_info(ks.BF16, i)["bm"] == 256 and ks.kernel_info(ks.BF16, i)["bn"] == 256 and
           ks.kernel_info(ks.BF16, i)["threads"] == 512][-1]
    M, N, K = 17 * 256 - 8, 17 * 256 - 24, 2048 + 24
    p = wl.make_problem("bf16", 0, 0, M, N, K, alpha=1.0, beta=0.5, seed=83, key=0, dist="normal")
    dp = gpu.DeviceProblem(p)
    plan = plan_of(ks, gpu, p, dp, big)
    assert plan["k_remainder"] == 24 and plan["tail_split"] >= 2, plan
    got = dp.run(big)
    bb, ii, jj = gpu.sample_entries(p, 4000, 9)
    err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
    assert err <= tolerance(p)


def test_seeded_random_shapes_through_every_launch_form(gpu):
    """Forty seeded 16-bit problems (ragged M and N, K any multiple of 8, four layouts, alpha and
    beta drawn) through the selecting entry point with the hybrid form forced where it can run:
    whatever mix of K cut, hybrid launch, split-K and plain launch a call resolves to, sampled
    entries meet the bound."""
    import paper_2003_06795_amd.binding as ks
    r = np.random.default_rng(84)
    ks.set_fast_path(True)
    forms = set()
    try:
        for n in range(40):
            M = int(r.integers(1, 700)) * 8
            N = int(r.integers(1, 700)) * 8
            K = int(r.integers(8, 400)) * 8
            tA, tB = int(r.integers(0, 2)), int(r.integers(0, 2))
            dtype = "bf16" if n % 4 else "f16"
            p = wl.make_problem(dtype, tA, tB, M, N, K, alpha=float(r.uniform(-2, 2)),
                                beta=float(r.choice([0.0, 1.0, -0.5])), seed=84, key=n, dist="normal")
            dp = gpu.DeviceProblem(p)
            ks.set_tail_split(8 if n % 2 else -1)
            plan = plan_of(ks, gpu, p, dp, -1)
            forms.add((plan["k_remainder"] > 0, plan["tail_split"] > 0, plan["split_k"] > 1, plan["path"]))
            got = dp.run()
            bb, ii, jj = gpu.sample_entries(p, 1500, n, tile=64)
            err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
            assert err <= tolerance(p), (n, (tA, tB, M, N, K), plan, err)
    finally:
        ks.set_tail_split(-1)
    assert len(forms) >= 4, forms
