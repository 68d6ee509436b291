"""GPU parity of the balanced persistent form (fp32 members with balanced_per_cu > 0): a fixed
number of work-groups, whole tiles first, then equal shares of the K-steps of the left-over tiles,
whose parts a second kernel adds.  Compared with the CPU oracle through the C ABI."""
import itertools

import numpy as np
import pytest

import workloads as wl
from helpers import tolerance, c_padding_mask

pytestmark = pytest.mark.gpu

LAYOUTS = list(itertools.product((0, 1), (0, 1)))


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    return gpu_util


@pytest.fixture()
def ks():
    import paper_2003_06795_amd.binding as ks
    yield ks
    ks.set_balanced_groups(0)


def balanced_ids(ks):
    return [i for i in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, i)["balanced_per_cu"] > 0]


def plain_twin(ks, kid):
    """The member with the same tiles, K-step and no split: what a balanced member runs as when it
    has no scratch."""
    a = ks.kernel_info(ks.F32, kid)
    for i in range(ks.num_kernels(ks.F32)):
        b = ks.kernel_info(ks.F32, i)
        if i != kid and b["balanced_per_cu"] == 0 and b["split_k"] == 1 and b["k_waves"] == 1 and \
                all(a[f] == b[f] for f in ("core", "bm", "bn", "bk", "wm", "wn")):
            return i
    return None


def check(p, got, ref, what):
    live = ~c_padding_mask(p)
    err = float(np.max(np.abs(got[live].astype(np.float64) - ref[live].astype(np.float64))))
    assert np.all(np.isfinite(got[live])), what
    assert err <= tolerance(p), "%s: max|diff| %.3e > tol %.3e" % (what, err, tolerance(p))
    mask = c_padding_mask(p)
    assert np.array_equal(got[mask], p.C0[mask], equal_nan=True), what + ": wrote outside C's logical entries"


def plan_of(ks, gpu, dp, kid):
    p = dp.p
    return ks.gemm_plan(ks.F32, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta,
                        dp.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)


def test_family_has_balanced_members(ks):
    ids = balanced_ids(ks)
    assert ids, "no member with a balanced persistent form"
    for kid in ids:
        ki = ks.kernel_info(ks.F32, kid)
        assert ki["core_name"] == "mfma32" and ki["split_k"] == 1 and ki["k_waves"] == 1
        assert plain_twin(ks, kid) is not None
        need = ks.workspace_bytes_needed(ks.F32, kid, 1000, 1000, 1)
        assert need == 256 * ki["balanced_per_cu"] * 2 * ki["bm"] * ki["bn"] * 4


# (tiles of 64 / 128 rows and columns: the counts below give, with 256 work-groups, one whole round
# plus divided left-over tiles; with 512 or 768 work-groups only divided tiles)
SHAPES = [
    # M, N, K, batch, pad, batch_pad, per_cu
    (1283, 964, 300, 1, (0, 0, 0), (0, 0, 0), 1),      # ragged edges, scalar loads (K = 300 is a multiple of 4 but M is odd)
    (1288, 968, 296, 1, (4, 8, 4), (0, 0, 0), 1),      # float4 loads, padded leading dimensions
    (520, 392, 1064, 3, (0, 0, 0), (8, 16, 24), 0),    # batched, member's own work-group count
    (392, 264, 4104, 1, (0, 0, 0), (0, 0, 0), 0),      # a dozen tiles, long K: every tile cut into many shares
    (2184, 2056, 72, 1, (0, 0, 0), (0, 0, 0), 1),      # several whole rounds, short K (shares of one or two steps)
]


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES)
def test_balanced_form_within_tolerance(gpu, ks, shape, tA, tB):
    M, N, K, batch, pad, bpad, per_cu = shape
    p = wl.make_problem("f32", tA, tB, M, N, K, batch=batch, alpha=1.25, beta=-0.5, seed=31,
                        key=M + 2 * tA + tB, pad=pad, batch_pad=bpad)
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    ks.set_balanced_groups(per_cu)
    for kid in balanced_ids(ks):
        gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, kid, M, N, batch))
        plan = plan_of(ks, gpu, dp, kid)
        ki = ks.kernel_info(ks.F32, kid)
        tiles = -(-M // ki["bm"]) * -(-N // ki["bn"]) * batch
        groups = 256 * (per_cu or ki["balanced_per_cu"])
        if per_cu == 0 and ki["balanced_per_cu"] == 2 and ki["threads"] >= 512 and tiles <= 96:
            groups = 256               # few tiles: a 512-thread member takes one work-group per compute unit
        assert plan["balanced_groups"] == groups and plan["divided_tiles"] == tiles % groups
        assert plan["workgroups"] == groups and plan["split_k"] == 1
        got = dp.run(kid)
        check(p, got, ref, "balanced kernel %d %s tA=%d tB=%d" % (kid, shape[:4], tA, tB))
        assert np.array_equal(got, dp.run(kid), equal_nan=True), "kernel %d: two runs differ" % kid


@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_balanced_form_small_integers_bit_exact(gpu, ks, tA, tB):
    """Entries in [-8, 8] with K * 64 < 2^24: every partial sum is an integer fp32 holds exactly, so
    the parts of a divided tile add up to the oracle's bits whatever the cut."""
    p = wl.make_problem("f32", tA, tB, 1100, 1300, 520, batch=1, alpha=1.0, beta=0.0, seed=6,
                        key=tA * 2 + tB, dist="ints", c_fill="nan", pad=(1, 0, 3))
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    live = ~c_padding_mask(p)
    for per_cu in (1, 0):
        ks.set_balanced_groups(per_cu)
        for kid in balanced_ids(ks):
            gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, kid, p.M, p.N, p.batch))
            assert np.array_equal(dp.run(kid)[live], ref[live]), "kernel %d per_cu %d" % (kid, per_cu)


def test_without_scratch_the_plain_member_runs(gpu, ks):
    p = wl.make_problem("f32", 0, 1, 1283, 964, 300, alpha=1.0, beta=0.25, seed=32)
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    try:
        ks.set_workspace(None)
        for kid in balanced_ids(ks):
            plan = plan_of(ks, gpu, dp, kid)
            assert plan["balanced_groups"] == 0 and plan["divided_tiles"] == 0
            got = dp.run(kid)
            check(p, got, ref, "kernel %d without scratch" % kid)
            assert np.array_equal(got, dp.run(plain_twin(ks, kid)), equal_nan=True)
    finally:
        gpu.ensure_workspace.__defaults__[0].clear()      # the next test registers a fresh buffer


def test_evenly_dividing_tile_count_needs_no_scratch(gpu, ks):
    """256 tiles per round and nothing left over: the persistent form runs without a workspace and
    every entry comes from one work-group, so it equals the plain member bit for bit."""
    try:
        ks.set_workspace(None)
        ks.set_balanced_groups(1)
        for kid in balanced_ids(ks):
            ki = ks.kernel_info(ks.F32, kid)
            M, N = 16 * ki["bm"], 32 * ki["bn"]           # 512 tiles: two rounds of 256 work-groups
            p = wl.make_problem("f32", 0, 0, M, N, 136, alpha=-1.0, beta=0.0, seed=33, c_fill="nan")
            dp = gpu.DeviceProblem(p)
            plan = plan_of(ks, gpu, dp, kid)
            assert plan["balanced_groups"] == 256 and plan["divided_tiles"] == 0
            got = dp.run(kid)
            bb, ii, jj = gpu.sample_entries(p, 300, 5, tile=ki["bm"])
            ref = gpu.oracle_entries(p, bb, ii, jj)
            vals = got.reshape(M, N)[ii, jj]
            assert np.max(np.abs(vals - ref)) <= tolerance(p)
            assert np.array_equal(got, dp.run(plain_twin(ks, kid)))
    finally:
        gpu.ensure_workspace.__defaults__[0].clear()


def test_balanced_form_with_bias_and_bf16_output(gpu, ks):
    import torch
    from oracle import gemm as og
    p = wl.make_problem("f32", 0, 0, 1283, 964, 300, batch=1, alpha=0.75, beta=0.5, seed=34)
    dp = gpu.DeviceProblem(p)
    bias = wl.uniform_pm1(p.N, 34, 9, 3)
    dbias = torch.from_numpy(bias).cuda()
    ref = p.C0.copy()
    og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref, p.ldc,
                 bias, p.batch, p.strideA, p.strideB, p.strideC)
    ks.set_balanced_groups(1)
    for kid in balanced_ids(ks):
        gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, kid, p.M, p.N, p.batch))
        C = dp.C0.clone()
        ks.gemm_bias(ks.F32, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, C,
                     p.ldc, dbias, p.batch, p.strideA, p.strideB, p.strideC)
        torch.cuda.synchronize()
        err = float(np.max(np.abs(C.cpu().numpy().astype(np.float64) - ref)))
        tol = tolerance(p) + 2.0 ** -22 * (float(np.max(np.abs(bias))) + float(np.max(np.abs(ref))))
        assert err <= tol, "kernel %d with bias: %.3e > %.3e" % (kid, err, tol)
    # C kept in bf16: the second kernel rounds the summed value once, as the single-kernel epilogue does
    C16 = wl.f32_to_bf16_rne(p.C0)
    ref16 = C16.copy()
    og.gemm_out_bf16(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref16,
                     p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    reff = wl.bf16_to_f32(ref16).astype(np.float64)
    for kid in balanced_ids(ks):
        C = torch.from_numpy(C16.view(np.int16).copy()).cuda()
        ks.gemm_out_bf16(ks.F32, kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, C,
                         p.ldc, dbias, p.batch, p.strideA, p.strideB, p.strideC)
        torch.cuda.synchronize()
        got = C.cpu().numpy().view(np.uint16)
        gotf = wl.bf16_to_f32(got).astype(np.float64)
        bound = tolerance(p) + 2.0 ** -22 * 4.0 + 2.0 ** -7 * np.abs(reff)
        assert np.all(np.isfinite(gotf)) and np.all(np.abs(gotf - reff) <= bound), "kernel %d, bf16 output" % kid
        assert np.mean(got == ref16) > 0.97, "kernel %d, bf16 output: too few entries agree exactly" % kid


@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_balanced_form_at_full_size(gpu, ks, tA, tB):
    """The largest shape of the fp32 tuning set (3016 x 1448 x 3656: 288 tiles of 128 x 128 on 512
    work-groups, 1104 tiles of 64 x 64 on 768) in the launch bench.py times: the members take the
    balanced form by themselves; sampled entries against the oracle."""
    import torch
    M, N, K = 3016, 1448, 3656
    p = wl.make_problem("f32", tA, tB, M, N, K, seed=35, key=tA * 2 + tB, c_fill="zeros")
    A, B = torch.from_numpy(p.A).cuda(), torch.from_numpy(p.B).cuda()
    bb, ii, jj = gpu.sample_entries(p, 1024, 35, tile=128)
    ref = gpu.oracle_entries(p, bb, ii, jj)
    flat = torch.from_numpy(ii * p.ldc + jj).cuda()
    for kid in balanced_ids(ks):
        gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, kid, M, N, 1))
        C = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
        args = (tA, tB, M, N, K, 1.0, A, p.lda, B, p.ldb, 0.0, C, p.ldc)
        plan = ks.gemm_plan(ks.F32, kid, *args)
        assert plan["balanced_groups"] > 0 and plan["divided_tiles"] > 0, (kid, plan)
        ks.gemm_f32_with_kernel(kid, *args)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(C).any()), "kernel %d left entries unwritten" % kid
        err = float(np.max(np.abs(C[flat].cpu().numpy().astype(np.float64) - ref)))
        assert err <= tolerance(p), "kernel %d: %.3e > %.3e" % (kid, err, tolerance(p))


def test_few_tiles_take_one_work_group_per_compute_unit(gpu, ks):
    """A 512-thread member with two work-groups per compute unit launches 256 of them for problems
    of at most 96 tiles (12 x 8 tiles here) and its own 512 from 97 tiles on (13 x 8, where one
    more row of A adds a tile row); both sides of the limit against the oracle on sampled entries."""
    import torch
    for kid in balanced_ids(ks):
        ki = ks.kernel_info(ks.F32, kid)
        if ki["balanced_per_cu"] != 2 or ki["threads"] < 512:
            continue
        gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, kid, 13 * ki["bm"], 8 * ki["bn"], 1))
        for M, groups in ((12 * ki["bm"], 256), (12 * ki["bm"] + 1, 512)):
            N, K = 8 * ki["bn"] - 24, 1096
            p = wl.make_problem("f32", 0, 1, M, N, K, alpha=1.0, beta=0.5, seed=36, key=M)
            dp = gpu.DeviceProblem(p)
            plan = plan_of(ks, gpu, dp, kid)
            assert plan["balanced_groups"] == groups and plan["workgroups"] == groups, (kid, M, plan)
            assert plan["divided_tiles"] == (-(-M // ki["bm"]) * 8) % groups
            got = dp.run(kid)
            bb, ii, jj = gpu.sample_entries(p, 2000, 36, tile=ki["bm"])
            err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
            assert err <= tolerance(p), (kid, M, err)
