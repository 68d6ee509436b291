"""Hybrid launches of the 16-bit members whose K split is chosen per call: whole rounds of tiles
run over all of K, the tiles of the last, partly filled round are cut along K and added up by a
third kernel.  Every such member against the oracle (sampled entries, every edge tile) and
against its own plain launch, ragged shapes, alpha / beta, bias, bf16 output, fp16 inputs, the
per-call rule, and the fall-back when the workspace cannot hold the partial tiles."""
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
    ks.set_tail_split(-1)


def per_call_members(ks):
    """Members that take part: split chosen per call, LDS stages that admit one work-group per unit."""
    out = []
    for i in range(ks.num_kernels(ks.BF16)):
        ki = ks.kernel_info(ks.BF16, i)
        if ki["split_k"] == 0 and (160 * 1024) // ki["lds_bytes"] == 1:
            out.append(i)
    return out


def slots_of(ki):
    """Work-groups of the member resident at once (the library's own count)."""
    waves = ki["threads"] // 64
    per_cu = max(12 // waves, 1)
    per_cu = min(per_cu, max((160 * 1024) // ki["lds_bytes"], 1))
    return 256 * per_cu


def shape_with_a_tail(ki, extra=21, K=512):
    """Ragged M, N whose tiles fill one round of work-groups and leave `extra`-odd tiles over."""
    tn = 17
    tm = -(-(slots_of(ki) + extra) // tn)
    return tm * ki["bm"] - 8, tn * ki["bn"] - 8, K


def plan_of(ks, gpu, p, dp, kid):
    return ks.gemm_plan(gpu.DT[p.dtype], kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                        p.beta, dp.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)


@pytest.mark.parametrize("layout", [(0, 0), (0, 1)])
def test_every_member_in_the_hybrid_form(gpu, layout):
    import paper_2003_06795_amd.binding as ks
    members = per_call_members(ks)
    assert len(members) >= 8
    for n, kid in enumerate(members):
        ki = ks.kernel_info(ks.BF16, kid)
        M, N, K = shape_with_a_tail(ki)
        p = wl.make_problem("bf16", layout[0], layout[1], M, N, K, alpha=1.25, beta=-0.5, seed=71, key=kid,
                            dist="normal")
        dp = gpu.DeviceProblem(p)
        ks.set_tail_split(0)
        assert plan_of(ks, gpu, p, dp, kid)["tail_split"] == 0
        plain = dp.run(kid)
        ks.set_tail_split(8)
        plan = plan_of(ks, gpu, p, dp, kid)
        assert plan["path"] >= 1 and plan["split_k"] == 1, (kid, plan)
        tiles = -(-M // ki["bm"]) * -(-N // ki["bn"])
        tail = tiles % slots_of(ki)
        assert 2 <= plan["tail_split"] <= 8, (kid, plan)
        assert plan["workgroups"] == tiles - tail + tail * plan["tail_split"], (kid, plan, tiles, tail)
        got = dp.run(kid)
        ks.set_tail_split(-1)
        tol = tolerance(p)
        bb, ii, jj = gpu.sample_entries(p, 3000, 11 + n, tile=64)
        ref = gpu.oracle_entries(p, bb, ii, jj)
        err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - ref)))
        assert err <= tol, "kernel %d %s: %.3e > %.3e" % (kid, (M, N, K), err, tol)
        # whole rounds are the same kernel on the same tiles: most of C is bit-identical to the plain
        # launch, the partitioned tiles agree to rounding
        same = float(np.mean(got == plain))
        assert same >= (tiles - tail - 1) / tiles * 0.9, (kid, same)
        assert float(np.max(np.abs(got.astype(np.float64) - plain))) <= 2 * tol


def test_bias_bf16_output_and_fp16_inputs(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    from oracle import gemm as og
    kid = per_call_members(ks)[0]
    ki = ks.kernel_info(ks.BF16, kid)
    M, N, K = shape_with_a_tail(ki, extra=9, K=384)
    try:
        ks.set_tail_split(4)
        # fp16 inputs through the same members
        p = wl.make_problem("f16", 0, 1, M, N, K, alpha=0.75, beta=0.0, seed=72, key=1, dist="normal")
        dp = gpu.DeviceProblem(p)
        assert plan_of(ks, gpu, p, dp, kid)["tail_split"] >= 2
        got = dp.run(kid)
        bb, ii, jj = gpu.sample_entries(p, 2000, 5, tile=64)
        err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
        assert err <= tolerance(p)
        # bias and an output kept in bf16 (the third kernel applies both)
        p = wl.make_problem("bf16", 0, 0, M, N, K, alpha=0.5, beta=0.25, seed=72, key=2, dist="normal")
        dp = gpu.DeviceProblem(p)
        bias = wl.uniform_pm1(p.N, 72, 9, 0)
        dbias = torch.from_numpy(bias).cuda()
        C = dp.C0.clone()
        ks.gemm_bias(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, C,
                     p.ldc, dbias, p.batch, p.strideA, p.strideB, p.strideC)
        torch.cuda.synchronize()
        ref = p.C0.copy()
        og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref, p.ldc,
                     bias, p.batch, p.strideA, p.strideB, p.strideC)
        assert float(np.max(np.abs(C.cpu().numpy().astype(np.float64) - ref))) <= tolerance(p) + 2.0 ** -22 * 4.0
        C16 = wl.f32_to_bf16_rne(p.C0)
        ref16 = C16.copy()
        og.gemm_out_bf16(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref16,
                         p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
        reff = wl.bf16_to_f32(ref16).astype(np.float64)
        D = torch.from_numpy(C16.view(np.int16).copy()).cuda()
        ks.gemm_out_bf16(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, D,
                         p.ldc, dbias, p.batch, p.strideA, p.strideB, p.strideC)
        torch.cuda.synchronize()
        gotf = wl.bf16_to_f32(D.cpu().numpy().view(np.uint16)).astype(np.float64)
        bound = tolerance(p) + 2.0 ** -22 * 4.0 + 2.0 ** -7 * np.abs(reff)
        assert np.all(np.isfinite(gotf)) and np.all(np.abs(gotf - reff) <= bound)
    finally:
        ks.set_tail_split(-1)


def test_rule_switch_and_workspace_fall_back(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    ks.set_tail_split(-1)
    # the 256 x 256 two-group member with a per-call split: 17 x 17 tiles = one round of 256 and 33 over
    big = [i for i in per_call_members(ks) if ks.kernel_info(ks.BF16, i)["bm"] == 256 and
           ks.kernel_info(ks.BF16, i)["bn"] == 256 and ks.kernel_info(ks.BF16, i)["threads"] == 512][-1]
    one = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(4, device="cuda")
    M = N = 17 * 256
    long_k = ks.gemm_plan(ks.BF16, big, 0, 1, M, N, 4096, 1.0, one, 4096, one, 4096, 0.0, c, N)
    assert long_k["tail_split"] >= 2 and long_k["split_k"] == 1, long_k         # 64 K-steps: it pays
    short_k = ks.gemm_plan(ks.BF16, big, 0, 1, M, N, 256, 1.0, one, 256, one, 256, 0.0, c, N)
    assert short_k["tail_split"] == 0, short_k                                 # four K-steps: it does not
    full = ks.gemm_plan(ks.BF16, big, 0, 1, 4096, 4096, 4096, 1.0, one, 4096, one, 4096, 0.0, c, 4096)
    assert full["tail_split"] == 0                                             # exactly one round
    batched = ks.gemm_plan(ks.BF16, big, 0, 1, M, N, 4096, 1.0, one, 4096, one, 4096, 0.0, c, N, 2, 0, 0, M * N)
    assert batched["tail_split"] == 0
    ks.set_tail_split(0)
    assert ks.gemm_plan(ks.BF16, big, 0, 1, M, N, 4096, 1.0, one, 4096, one, 4096, 0.0, c, N)["tail_split"] == 0
    ks.set_tail_split(-1)
    # a registered workspace too small for the partial tiles: the plain launch runs
    small = torch.empty(1 << 18, dtype=torch.float32, device="cuda")
    try:
        ks.set_workspace(small)
        assert ks.gemm_plan(ks.BF16, big, 0, 1, M, N, 4096, 1.0, one, 4096, one, 4096, 0.0, c, N)["tail_split"] == 0
    finally:
        gpu.ensure_workspace(1)
        ks.set_workspace(gpu.ensure_workspace.__defaults__[0]["buf"])
    # members that share a compute unit keep the plain launch
    shared = [i for i in range(ks.num_kernels(ks.BF16)) if ks.kernel_info(ks.BF16, i)["split_k"] == 0 and
              (160 * 1024) // ks.kernel_info(ks.BF16, i)["lds_bytes"] >= 2][0]
    ks.set_tail_split(8)
    assert ks.gemm_plan(ks.BF16, shared, 0, 1, M, N, 4096, 1.0, one, 4096, one, 4096, 0.0, c, N)["tail_split"] == 0
    ks.set_tail_split(-1)
    assert ks.workspace_bytes_needed(ks.BF16, big, M, N, 1) == 7 * 33 * 256 * 256 * 4
    assert ks.workspace_bytes_needed(ks.BF16, big, 4096, 4096, 1) == 0
    for bad in (1, 17, -2):
        assert ks.lib().ks_set_tail_split(bad) == ks.ERR_INVALID_ARG
    # the default rule on a real problem, against the oracle
    p = wl.make_problem("bf16", 0, 1, M - 8, N - 24, 2048, seed=73, key=0, dist="normal")
    dp = gpu.DeviceProblem(p)
    plan = plan_of(ks, gpu, p, dp, big)
    assert plan["tail_split"] >= 2, plan
    got = dp.run(big)
    bb, ii, jj = gpu.sample_entries(p, 4000, 3)
    err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
    assert err <= tolerance(p)


def test_scratch_passed_per_call_and_static_scratch(gpu):
    """The partial tiles may also live in a workspace handed over per call or in the library's static
    array (when it is large enough); the registered workspace is then not touched."""
    import torch
    import paper_2003_06795_amd.binding as ks
    kid = [i for i in per_call_members(ks) if ks.kernel_info(ks.BF16, i)["bm"] == 128][-1]
    ki = ks.kernel_info(ks.BF16, kid)
    M, N, K = shape_with_a_tail(ki, extra=5, K=1024)
    p = wl.make_problem("bf16", 0, 1, M, N, K, alpha=1.0, beta=0.5, seed=74, key=0, dist="normal")
    dp = gpu.DeviceProblem(p)
    try:
        ks.set_tail_split(4)
        assert plan_of(ks, gpu, p, dp, kid)["tail_split"] >= 2
        ref = dp.run(kid)                                   # registered workspace
        need = ks.workspace_bytes_needed(ks.BF16, kid, M, N, 1)
        assert need > 0
        canary = torch.full((gpu.ensure_workspace(1).numel(),), 3.5, dtype=torch.float32, device="cuda")
        ks.set_workspace(canary)
        own = torch.empty(need // 4, dtype=torch.float32, device="cuda")
        C = dp.C0.clone()
        ks.gemm_with_workspace(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                               p.beta, C, p.ldc, own, batch=1)
        D = dp.C0.clone()
        ks.gemm_static_scratch(ks.BF16, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                               p.beta, D, p.ldc)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), ref)
        assert np.array_equal(D.cpu().numpy(), ref)
        assert bool((canary == 3.5).all())
    finally:
        ks.set_tail_split(-1)
        ks.set_workspace(gpu.ensure_workspace(1))
