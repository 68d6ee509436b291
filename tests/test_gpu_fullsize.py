"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (the
deployed selector picks the kernel), on sampled output entries the CPU oracle computes one by one."""
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
    return gpu_util


def run_selected_and_check(gpu, p, n_samples, seed, what):
    """C starts as NaN when beta == 0 (so unwritten entries show) and as p.C0 otherwise."""
    import torch
    import paper_2003_06795_amd.binding as ks
    dt = gpu.DT[p.dtype]
    kid = ks.select(dt, p.M, p.N, p.K, p.batch, p.transA, p.transB)
    need = ks.workspace_bytes_needed(dt, kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)
    a = p.A if p.dtype == "f32" else p.A.view(np.int16)
    b = p.B if p.dtype == "f32" else p.B.view(np.int16)
    A, B = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    if p.beta == 0.0:
        C = torch.full((p.C0.size,), float("nan"), dtype=torch.float32, device="cuda")
    else:
        C = torch.from_numpy(p.C0).cuda()
    fn = ks.gemm_f32 if p.dtype == "f32" else ks.gemm_bf16
    fn(p.transA, p.transB, p.M, p.N, p.K, p.alpha, A, p.lda, B, p.ldb, p.beta, C, p.ldc, p.batch,
       p.strideA, p.strideB, p.strideC)
    torch.cuda.synchronize()
    bb, ii, jj = gpu.sample_entries(p, n_samples, seed)
    flat = torch.from_numpy(bb * p.strideC + ii * p.ldc + jj).cuda()
    got = C[flat].cpu().numpy()
    ref = gpu.oracle_entries(p, bb, ii, jj)
    err = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))))
    assert np.all(np.isfinite(got)), what
    assert err <= tolerance(p), "%s (kernel %d): max|diff| %.3e > tol %.3e" % (what, kid, err, tolerance(p))
    if p.beta == 0.0:
        # every logical entry was written: no NaN left anywhere in the dense output
        assert not bool(torch.isnan(C).any()), what + ": entries of C left unwritten"
    return kid


def test_config2_largest_and_random_rows(gpu):
    rows = wl.config2_rows()
    order = np.argsort([-(r[3] * r[4] * r[5]) for r in rows])
    pick = list(order[:8]) + list(np.random.default_rng(2).choice(len(rows), 24, replace=False))
    used = set()
    for i in pick:
        s, tA, tB, M, N, K, b = rows[int(i)]
        p = wl.make_problem("f32", tA, tB, M, N, K, seed=1, key=int(i), c_fill="zeros")
        used.add(run_selected_and_check(gpu, p, 512, int(i), "config 2 row %d (%d x %d x %d)" % (i, M, N, K)))
    assert len(used) >= 3          # the sample exercises several members of the kept set


@pytest.mark.parametrize("shape", [
    (49, 32, 3), (196, 64, 27), (49, 2048, 4608), (3136, 128, 288), (25088, 512, 1152),
    (100352, 256, 576), (401408, 64, 27), (401408, 2048, 3),
    (401408, 512, 27), (100352, 2048, 64),          # large outputs, short K: the multi-tile form
])
def test_config3_im2col_shapes(gpu, shape):
    M, N, K = shape
    p = wl.make_problem("f32", 0, 0, M, N, K, seed=2, key=M % 1000 + K, c_fill="zeros")
    run_selected_and_check(gpu, p, 1024, K, "config 3 %s" % (shape,))


def test_config3_operand_beyond_4_gib(gpu):
    """A is 401408 x 4608 fp32 = 7.4 GB: row offsets need 64 bits."""
    M, N, K = 401408, 32, 4608
    p = wl.make_problem("f32", 0, 0, M, N, K, seed=2, key=9, c_fill="zeros")
    assert p.A.nbytes > 2 ** 32
    bb, ii, jj = np.zeros(3, np.int64), np.array([0, M // 2 + 7, M - 1]), np.array([0, 5, N - 1])
    run_selected_and_check(gpu, p, 1024, 3, "config 3 401408 x 32 x 4608")


def test_config4_batched_small_all_64_shapes_full_oracle(gpu):
    for n, (M, N, K) in enumerate(wl.config4_shapes()):
        p = wl.make_problem("f32", 0, 0, M, N, K, batch=wl.CONFIG4_BATCH, alpha=wl.CONFIG4_ALPHA,
                            beta=wl.CONFIG4_BETA, seed=3, key=n)
        dp = gpu.DeviceProblem(p)
        got, ref = dp.run(None), gpu.oracle_full(p)
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        assert err <= tolerance(p), "config 4 %s: %.3e > %.3e" % ((M, N, K), err, tolerance(p))


@pytest.mark.parametrize("layout", wl.CONFIG5_LAYOUTS)
@pytest.mark.parametrize("shape", wl.config5_shapes())
def test_config5_bf16_cells(gpu, shape, layout):
    M, N, K = shape
    tA, tB = layout
    p = wl.make_problem("bf16", tA, tB, M, N, K, seed=4, key=M + N + tB, dist="normal", c_fill="zeros")
    run_selected_and_check(gpu, p, 1024, K + tB, "config 5 %s layout %s" % (shape, layout))


# ----------------------------------------------------------------------------- forced kernels at full size
# Everything above goes through the selector; the cases below force members through
# ks_gemm_*_with_kernel so that every deployed kernel is checked in the launch form large problems
# use (one-dimensional grid with the XCD renumbering), with 64-bit row offsets, with a per-call
# split that really splits, on the general 16-bit path at sizes that are multiples of nothing, and
# through the other entry points.

def kept_ids(dtype):
    """Kernel ids at the leaves of the deployed tree."""
    import paper_2003_06795_amd.binding as ks
    t = ks.get_selector(ks.F32 if dtype == "f32" else ks.BF16)
    return sorted({int(n["value"]) for n in t if n["feature"] < 0})


def run_forced_and_check(gpu, p, kid, n_samples, seed, what, expect_1d=True, expect_split=None, expect_path=None):
    import torch
    import paper_2003_06795_amd.binding as ks
    dt = gpu.DT[p.dtype]
    need = ks.workspace_bytes_needed(dt, kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)
    a = p.A if p.dtype == "f32" else p.A.view(np.int16)
    b = p.B if p.dtype == "f32" else p.B.view(np.int16)
    A, B = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    if p.beta == 0.0:
        C = torch.full((p.C0.size,), float("nan"), dtype=torch.float32, device="cuda")
    else:
        C = torch.from_numpy(p.C0).cuda()
    args = (p.transA, p.transB, p.M, p.N, p.K, p.alpha, A, p.lda, B, p.ldb, p.beta, C, p.ldc, p.batch,
            p.strideA, p.strideB, p.strideC)
    plan = ks.gemm_plan(dt, kid, *args)
    assert plan["kernel_id"] == kid
    if expect_1d:
        assert plan["grid_3d"] == 0, what + ": expected the one-dimensional launch"
    if expect_split is not None:
        assert (plan["split_k"] > 1) == expect_split, what + ": split %d" % plan["split_k"]
    if expect_path is not None:
        assert plan["path"] in expect_path, what + ": path %d" % plan["path"]
    gpu.GEMM_K[p.dtype](kid, *args)
    torch.cuda.synchronize()
    bb, ii, jj = gpu.sample_entries(p, n_samples, seed)
    flat = torch.from_numpy(bb * p.strideC + ii * p.ldc + jj).cuda()
    got = C[flat].cpu().numpy()
    ref = gpu.oracle_entries(p, bb, ii, jj)
    assert np.all(np.isfinite(got)), what
    err = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))))
    assert err <= tolerance(p), "%s (kernel %d): max|diff| %.3e > tol %.3e" % (what, kid, err, tolerance(p))
    if p.beta == 0.0 and p.ldc == p.N:
        assert not bool(torch.isnan(C).any()), what + ": entries of C left unwritten"
    return plan


def test_every_kept_fp32_kernel_on_a_one_dimensional_launch(gpu):
    p = wl.make_problem("f32", 1, 0, 2864, 2376, 840, seed=5, key=1, c_fill="zeros")
    ids = kept_ids("f32")
    assert len(ids) >= 4
    for kid in ids:
        run_forced_and_check(gpu, p, kid, 768, kid, "fp32 kept id %d, 2864 x 2376 x 840 TN" % kid)


@pytest.mark.parametrize("tB", [0, 1])
def test_every_kept_bf16_kernel_on_a_one_dimensional_launch(gpu, tB):
    p = wl.make_problem("bf16", 0, tB, 4096, 4096, 1024, seed=5, key=2 + tB, dist="normal", c_fill="zeros")
    for kid in kept_ids("bf16"):
        run_forced_and_check(gpu, p, kid, 768, kid, "bf16 kept id %d, 4096 x 4096 x 1024 N%s" % (kid, "NT"[tB]),
                             expect_path=(1, 2))


def test_every_kept_bf16_kernel_general_path_at_ragged_sizes(gpu):
    """4100 x 4104 x 4100: K is a multiple of no K-step, M of no tile; the direct-to-LDS path does
    not apply."""
    p = wl.make_problem("bf16", 0, 1, 4100, 4104, 4100, seed=5, key=4, dist="normal", c_fill="zeros")
    for kid in kept_ids("bf16"):
        run_forced_and_check(gpu, p, kid, 512, kid, "bf16 kept id %d, 4100 x 4104 x 4100 NT" % kid, expect_path=(0,))


@pytest.mark.parametrize("N", [512, 2048])
def test_config3_workhorse_kernels_beyond_4_gib(gpu, N):
    """A = 401408 x 4608 fp32 (7.4 GB): ids 59 and 47 (128 x 128 x 32, plain and with a balanced form
    that such tile counts do not take) and 29 (64 x 64 x 32), the members the deployed trees have
    given the im2col rows of this size."""
    M, K = 401408, 4608
    p = wl.make_problem("f32", 0, 0, M, N, K, seed=2, key=N, c_fill="zeros")
    assert p.A.nbytes > 2 ** 32
    for kid in ((59, 47, 29) if N == 512 else (59, 47)):
        run_forced_and_check(gpu, p, kid, 1024, N + kid, "fp32 id %d, 401408 x %d x 4608" % (kid, N))


def test_per_call_split_members_split_at_full_size(gpu):
    """96 x 3016 x 3392: few output tiles, long K; every member whose split is chosen per call takes
    more than one partition here (workspace registered) and must still match."""
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f32", 0, 0, 96, 3016, 3392, seed=5, key=6, alpha=1.5, beta=0.5)
    gpu.ensure_workspace(64 << 20)
    split = [k for k in range(ks.num_kernels(ks.F32)) if ks.kernel_info(ks.F32, k)["split_k"] == 0]
    assert len(split) >= 8
    took = 0
    for kid in split:
        plan = run_forced_and_check(gpu, p, kid, 512, kid, "fp32 per-call split id %d" % kid, expect_1d=False)
        took += plan["split_k"] > 1
    assert took >= len(split) - 2
    p = wl.make_problem("bf16", 0, 1, 256, 256, 65536, seed=5, key=7, dist="normal", c_fill="zeros")
    for kid in [k for k in range(ks.num_kernels(ks.BF16)) if ks.kernel_info(ks.BF16, k)["split_k"] == 0]:
        run_forced_and_check(gpu, p, kid, 512, kid, "bf16 per-call split id %d" % kid, expect_1d=False,
                             expect_split=True)


def test_direct_to_lds_path_with_a_leading_dimension_near_its_limit(gpu):
    """lda = 2^22 - 8 elements: tile-relative byte offsets of the direct-to-LDS loads come close to
    2^31; the largest row offset inside a 256-row tile is 255 * lda * 2 bytes."""
    import paper_2003_06795_amd.binding as ks
    M, N, K = 264, 256, 512
    lda = (1 << 22) - 8
    p = wl.make_problem("bf16", 0, 1, M, N, K, seed=5, key=8, dist="normal", c_fill="zeros", pad=(lda - K, 0, 0))
    assert p.lda == lda
    for kid in (2, 5):
        run_forced_and_check(gpu, p, kid, 512, kid, "bf16 id %d, lda 2^22 - 8" % kid, expect_1d=False,
                             expect_path=(1, 2))


def test_other_entry_points_at_full_size(gpu):
    """fp16 operands, fused bias and bf16 output on one full-size row each (selected kernel)."""
    import torch
    import paper_2003_06795_amd.binding as ks
    from oracle import gemm as og
    # fp16 operands
    p = wl.make_problem("f16", 0, 1, 4096, 4096, 4096, seed=5, key=9, dist="normal", c_fill="zeros")
    A, B = torch.from_numpy(p.A.view(np.int16)).cuda(), torch.from_numpy(p.B.view(np.int16)).cuda()
    C = torch.full((p.C0.size,), float("nan"), dtype=torch.float32, device="cuda")
    ks.gemm_f16(0, 1, p.M, p.N, p.K, 1.0, A, p.lda, B, p.ldb, 0.0, C, p.ldc)
    torch.cuda.synchronize()
    bb, ii, jj = gpu.sample_entries(p, 1024, 11)
    got = C[torch.from_numpy(ii * p.ldc + jj).cuda()].cpu().numpy()
    err = float(np.max(np.abs(got.astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
    assert err <= tolerance(p) and not bool(torch.isnan(C).any())
    # fused bias, fp32, beta != 0: the oracle's bias form on a 64-row slab that holds the sampled rows
    M, N, K = 25088, 512, 1152
    p = wl.make_problem("f32", 0, 0, M, N, K, seed=5, key=10, alpha=0.75, beta=-0.5)
    bias = wl.uniform_pm1(N, 5, 10, 3)
    A, B, C = torch.from_numpy(p.A).cuda(), torch.from_numpy(p.B).cuda(), torch.from_numpy(p.C0).cuda()
    ks.gemm_bias(ks.F32, -1, 0, 0, M, N, K, p.alpha, A, p.lda, B, p.ldb, p.beta, C, p.ldc,
                 torch.from_numpy(bias).cuda())
    torch.cuda.synchronize()
    for r0 in (0, 12480, M - 64):
        ref = p.C0[r0 * N:(r0 + 64) * N].copy()
        og.gemm_bias("f32", 0, 0, 64, N, K, p.alpha, p.A[r0 * K:], p.lda, p.B, p.ldb, p.beta, ref, p.ldc, bias)
        got = C[r0 * N:(r0 + 64) * N].cpu().numpy()
        tol = tolerance(p) + 2.0 ** -22 * (1.0 + float(np.max(np.abs(ref))))
        assert float(np.max(np.abs(got.astype(np.float64) - ref))) <= tol
    # bf16 output, bf16 operands
    M, N, K = 4096, 2048, 4096
    p = wl.make_problem("bf16", 0, 0, M, N, K, seed=5, key=12, dist="normal", c_fill="zeros")
    A, B = torch.from_numpy(p.A.view(np.int16)).cuda(), torch.from_numpy(p.B.view(np.int16)).cuda()
    C16 = torch.zeros(M * N, dtype=torch.int16, device="cuda")
    ks.gemm_out_bf16(ks.BF16, -1, 0, 0, M, N, K, 1.0, A, p.lda, B, p.ldb, 0.0, C16, N)
    torch.cuda.synchronize()
    for r0 in (0, 2000, M - 64):
        want16 = np.zeros(64 * N, dtype=np.uint16)
        og.gemm_out_bf16("bf16", 0, 0, 64, N, K, 1.0, p.A[r0 * K:], p.lda, p.B, p.ldb, 0.0, want16, N)
        got16 = C16[r0 * N:(r0 + 64) * N].cpu().numpy().view(np.uint16)
        got = (got16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        want = (want16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        # one bf16 step (2^-7 relative) on top of the accumulation bound
        assert np.all(np.abs(got - want) <= tolerance(p) + 2.0 ** -7 * np.abs(want))
        assert np.mean(got16 == want16) > 0.97


def test_seeded_random_fp32_problems_through_whatever_form_the_call_resolves_to(gpu):
    """Forty seeded fp32 problems of the tuning set's size range (dimensions log-uniform in 16 ..
    4096, every fourth one in 1024 .. 4096, multiples of 8 or not, four layouts, alpha and beta drawn) through the selecting entry
    point with a workspace registered: plain launches, several rounds of K partitions, the balanced
    persistent form and three-dimensional grids all occur, and sampled entries (every edge tile
    among them) meet the bound whichever the call resolves to."""
    import paper_2003_06795_amd.binding as ks
    r = np.random.default_rng(91)
    gpu.ensure_workspace(256 << 20)
    forms = set()
    for n in range(40):
        lo = 1024 if n % 4 == 3 else 16                                   # every fourth one in the mid-size band
        M, N, K = (int(np.exp(r.uniform(np.log(lo), np.log(4096)))) for _ in range(3))
        if n % 3:
            M, N, K = (max(8, v // 8 * 8) for v in (M, N, K))
        tA, tB = int(r.integers(0, 2)), int(r.integers(0, 2))
        p = wl.make_problem("f32", tA, tB, M, N, K, alpha=float(r.uniform(-2, 2)), beta=float(r.choice([0.0, 1.0, -0.5])),
                            seed=91, key=n)
        dp = gpu.DeviceProblem(p)
        plan = ks.gemm_plan(ks.F32, -1, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta,
                            dp.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
        ki = ks.kernel_info(ks.F32, plan["kernel_id"])
        tiles = -(-M // ki["bm"]) * -(-N // ki["bn"])
        slots = 256 * max(12 // (ki["threads"] // 64), 1)
        forms.add(("balanced" if plan["balanced_groups"] else "rounds" if plan["split_k"] > 1 and
                   tiles * plan["split_k"] > slots else "split" if plan["split_k"] > 1 else "plain", plan["grid_3d"]))
        got = dp.run()
        bb, ii, jj = gpu.sample_entries(p, 1500, n, tile=64)
        err = float(np.max(np.abs(got[ii * p.ldc + jj].astype(np.float64) - gpu.oracle_entries(p, bb, ii, jj))))
        assert err <= tolerance(p), (n, (tA, tB, M, N, K), plan, err)
    assert {f for f, _ in forms} == {"plain", "split", "rounds", "balanced"} and {g for _, g in forms} == {0, 1}, forms
