"""GPU parity: every member of the kernel family against the CPU oracle, through the C ABI."""
import itertools

import numpy as np
import pytest

import workloads as wl
from helpers import tolerance, c_padding_mask, operand_matrices, c_views

pytestmark = pytest.mark.gpu

LAYOUTS = list(itertools.product((0, 1), (0, 1)))


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    return gpu_util


def check(p, got, ref, what):
    live = ~c_padding_mask(p)
    err = float(np.max(np.abs(got[live].astype(np.float64) - ref[live].astype(np.float64)))) if live.any() else 0.0
    tol = tolerance(p)
    assert np.all(np.isfinite(got[live])), what
    assert err <= tol, "%s: max|diff| %.3e > tol %.3e" % (what, err, tol)
    mask = c_padding_mask(p)
    assert np.array_equal(got[mask], p.C0[mask], equal_nan=True), what + ": wrote outside C's logical entries"


def ids_of(gpu, dtype):
    import paper_2003_06795_amd.binding as ks
    return list(range(ks.num_kernels(gpu.DT[dtype])))


def prep_workspace(gpu, p, kid):
    import paper_2003_06795_amd.binding as ks
    need = ks.workspace_bytes_needed(gpu.DT[p.dtype], kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)


# ----------------------------------------------------------------------------- config 1

def test_config1_four_tile_instantiations(gpu):
    import paper_2003_06795_amd.binding as ks
    p = wl.config1_problem()
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    wanted = set(wl.CONFIG1_TILES)
    found = []
    for kid in ids_of(gpu, "f32"):
        ki = ks.kernel_info(ks.F32, kid)
        key = (ki["bm"], ki["bn"], ki["tm"], ki["tn"], ki["bk"])
        if ki["core_name"] == "fma" and key in wanted:
            found.append(key)
            check(p, dp.run(kid), ref, "config1 kernel %d" % kid)
    assert sorted(found) == sorted(wanted)


# ----------------------------------------------------------------------------- every kernel, every layout

SHAPES_F32 = [
    # (M, N, K, batch, pads, batch_pad)  - several tiles of the small kernels plus ragged tails
    (200, 136, 72, 2, (0, 0, 0), (0, 0, 0)),        # multiples of 8: float4 path
    (197, 131, 67, 2, (3, 1, 2), (5, 3, 7)),        # nothing aligned: scalar path
    (264, 520, 40, 1, (4, 8, 4), (0, 0, 0)),        # wider than the 256 tiles, padded leading dims
]


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES_F32)
def test_f32_all_kernels_within_tolerance(gpu, shape, tA, tB):
    M, N, K, batch, pad, bpad = shape
    p = wl.make_problem("f32", tA, tB, M, N, K, batch=batch, alpha=1.5, beta=-0.75, seed=21,
                        key=M + 2 * tA + tB, pad=pad, batch_pad=bpad)
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    for kid in ids_of(gpu, "f32"):
        prep_workspace(gpu, p, kid)
        check(p, dp.run(kid), ref, "f32 kernel %d %s tA=%d tB=%d" % (kid, shape[:3], tA, tB))


@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_f32_small_integers_bit_exact(gpu, tA, tB):
    """Entries in [-8, 8] and K*64 < 2^24: every partial sum is an integer fp32 represents, so
    any summation order gives the oracle's bits.  A wrong fragment layout cannot hide here."""
    p = wl.make_problem("f32", tA, tB, 150, 170, 90, batch=2, alpha=1.0, beta=0.0, seed=5,
                        key=tA * 2 + tB, dist="ints", c_fill="nan", pad=(1, 0, 3))
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    live = ~c_padding_mask(p)
    for kid in ids_of(gpu, "f32"):
        prep_workspace(gpu, p, kid)
        got = dp.run(kid)
        assert np.array_equal(got[live], ref[live]), "kernel %d" % kid


@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_f32_permutation_operand_moves_rows_bit_exact(gpu, tA, tB):
    M = K = 96
    N = 80
    r = np.random.default_rng(3)
    perm = r.permutation(M)
    P = np.zeros((M, K), dtype=np.float32)
    P[np.arange(M), perm] = 1.0
    X = wl.uniform_pm1(K * N, 3, 1).reshape(K, N)
    p = wl.make_problem("f32", tA, tB, M, N, K, seed=3, c_fill="zeros")
    p.A = np.ascontiguousarray(P.T if tA else P).ravel()
    p.B = np.ascontiguousarray(X.T if tB else X).ravel()
    dp = gpu.DeviceProblem(p)
    for kid in ids_of(gpu, "f32"):
        prep_workspace(gpu, p, kid)
        assert np.array_equal(dp.run(kid).reshape(M, N), X[perm, :]), "kernel %d" % kid


SHAPES_BF16 = [
    (264, 136, 384, 2, (8, 16, 4), (8, 0, 0)),      # K a multiple of every K-step: direct-to-LDS path
    (520, 264, 256, 1, (0, 0, 0), (0, 0, 0)),       # several 256-wide tiles on the direct-to-LDS path
    (264, 136, 200, 2, (0, 0, 0), (0, 0, 0)),       # multiples of 8: 16-byte path
    (261, 131, 203, 2, (3, 1, 2), (5, 3, 7)),       # ragged: scalar path
    (40, 520, 72, 1, (8, 8, 4), (0, 0, 0)),
]


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("shape", SHAPES_BF16)
def test_bf16_all_kernels_within_tolerance(gpu, shape, tA, tB):
    M, N, K, batch, pad, bpad = shape
    p = wl.make_problem("bf16", tA, tB, M, N, K, batch=batch, alpha=0.5, beta=1.25, seed=22,
                        key=M + 2 * tA + tB, pad=pad, batch_pad=bpad, dist="normal")
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    # tight diagnostic besides the stated bound: fp32 accumulation error relative to sum |a||b|
    As, Bs, _ = operand_matrices(p)
    mag = [np.abs(a) @ np.abs(b) for a, b in zip(As, Bs)]
    for kid in ids_of(gpu, "bf16"):
        prep_workspace(gpu, p, kid)
        got = dp.run(kid)
        check(p, got, ref, "bf16 kernel %d %s tA=%d tB=%d" % (kid, shape[:3], tA, tB))
        for g, r_, m in zip(c_views(p, got), c_views(p, ref), mag):
            rel = np.max(np.abs(g.astype(np.float64) - r_) / (abs(p.alpha) * m + abs(p.beta) + 1e-30))
            assert rel < K * 2.0 ** -22, "kernel %d: accumulation error %.3e" % (kid, rel)


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("shape", [(150, 170, 330, (1, 0, 3)), (152, 168, 384, (0, 8, 3))])
def test_bf16_small_integers_bit_exact(gpu, shape, tA, tB):
    """The second shape takes the direct-to-LDS path (aligned, K a multiple of every K-step)."""
    M, N, K, pad = shape
    p = wl.make_problem("bf16", tA, tB, M, N, K, batch=2, alpha=1.0, beta=0.0, seed=6,
                        key=tA * 2 + tB, dist="ints", c_fill="nan", pad=pad)
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    live = ~c_padding_mask(p)
    for kid in ids_of(gpu, "bf16"):
        prep_workspace(gpu, p, kid)
        got = dp.run(kid)
        assert np.array_equal(got[live], ref[live]), "kernel %d" % kid


@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_bf16_generic_and_direct_to_lds_paths_agree_bitwise(gpu, tA, tB):
    """Same tiles, same summation order: the two code paths of an instantiation give equal bits."""
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("bf16", tA, tB, 392, 264, 512, batch=1, alpha=1.0, beta=0.5, seed=8,
                        key=tA * 2 + tB, dist="normal")
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    for kid in ids_of(gpu, "bf16"):
        prep_workspace(gpu, p, kid)
        fast = dp.run(kid)
        try:
            ks.set_fast_path(False)
            slow = dp.run(kid)
        finally:
            ks.set_fast_path(True)
        check(p, fast, ref, "bf16 kernel %d direct-to-LDS" % kid)
        assert np.array_equal(fast, slow), "kernel %d" % kid


# ----------------------------------------------------------------------------- conventions and edges

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_sizes(gpu, dtype):
    import paper_2003_06795_amd.binding as ks
    for (M, N, K, batch) in [(0, 5, 7, 1), (5, 0, 7, 1), (5, 6, 7, 0), (5, 6, 0, 2), (1, 1, 1, 1)]:
        for beta in (0.0, 0.5):
            p = wl.make_problem(dtype, 0, 0, M, N, K, batch=batch, alpha=2.0, beta=beta, seed=1,
                                c_fill="nan" if beta == 0.0 else "uniform")
            dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
            for kid in (0, ks.num_kernels(gpu.DT[dtype]) - 1, None):
                if kid is not None:
                    prep_workspace(gpu, p, kid)
                got = dp.run(kid)
                assert np.array_equal(got, ref, equal_nan=True) or np.max(np.abs(got - ref)) <= tolerance(p)


def test_beta_zero_ignores_nan_in_c_and_broadcast_strides(gpu):
    p = wl.make_problem("f32", 0, 1, 70, 50, 30, batch=3, alpha=1.0, beta=0.0, seed=2, c_fill="nan",
                        broadcast=(True, False))
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    for kid in (0, 20, 35, 53, None):
        check(p, dp.run(kid), ref, "kernel %s" % kid)
    p = wl.make_problem("f32", 1, 0, 70, 50, 30, batch=3, alpha=-1.0, beta=2.0, seed=2,
                        broadcast=(False, True))
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    for kid in (6, 26, 37, None):
        check(p, dp.run(kid), ref, "kernel %s" % kid)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_run_to_run_bitwise_determinism_and_batch_equals_loop(gpu, dtype):
    import torch
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem(dtype, 0, 0, 130, 140, 260, batch=3, alpha=1.0, beta=0.5, seed=9,
                        dist="normal" if dtype == "bf16" else "uniform")
    dp = gpu.DeviceProblem(p)
    for kid in ids_of(gpu, dtype):
        prep_workspace(gpu, p, kid)
        a, b = dp.run(kid), dp.run(kid)
        assert np.array_equal(a, b), "kernel %d is not deterministic" % kid
        # the same three items as three single calls
        C = dp.C0.clone()
        fn = ks.gemm_f32_with_kernel if dtype == "f32" else ks.gemm_bf16_with_kernel
        esz = 4 if dtype == "f32" else 2
        for t in range(p.batch):
            fn(kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha,
               dp.A.data_ptr() + t * p.strideA * esz, p.lda, dp.B.data_ptr() + t * p.strideB * esz,
               p.ldb, p.beta, C.data_ptr() + t * p.strideC * 4, p.ldc, 1, 0, 0, 0)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), a), "kernel %d: batched != looped" % kid


def test_argument_errors_launch_nothing(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    A = torch.ones(64, device="cuda:0")
    C = torch.full((64,), 7.0, device="cuda:0")
    bad = [
        dict(transA=2), dict(M=-1), dict(lda=3), dict(ldb=3), dict(ldc=3), dict(A=0), dict(C=0),
        dict(batch=2, strideC=8), dict(kernel_id=64), dict(kernel_id=-1),
    ]
    base = dict(kernel_id=0, transA=0, transB=0, M=4, N=4, K=4, alpha=1.0, A=A, lda=4, B=A, ldb=4,
                beta=0.0, C=C, ldc=4, batch=1, strideA=0, strideB=0, strideC=0)
    for change in bad:
        kw = dict(base)
        kw.update(change)
        with pytest.raises(ks.KsError) as e:
            ks.gemm_f32_with_kernel(**kw)
        assert e.value.status == ks.ERR_INVALID_ARG, change
    with pytest.raises(ks.KsError) as e:
        ks.gemm_f32_with_kernel(**dict(base, M=2 ** 31))
    assert e.value.status == ks.ERR_UNSUPPORTED
    with pytest.raises(ks.KsError) as e:
        ks.gemm_f32_with_kernel(**dict(base, ldc=2 ** 40))
    assert e.value.status == ks.ERR_UNSUPPORTED
    with pytest.raises(ks.KsError) as e:
        ks.set_workspace(C.data_ptr() + 2, 64)          # not a float address
    assert e.value.status == ks.ERR_INVALID_ARG
    ks.set_workspace(None)
    fixed_split = [k for k in range(ks.num_kernels(ks.BF16)) if ks.kernel_info(ks.BF16, k)["split_k"] > 1][0]
    with pytest.raises(ks.KsError) as e:
        ks.gemm_bf16_with_kernel(fixed_split, 0, 0, 4, 4, 4, 1.0, A, 4, A, 4, 0.0, C, 4)
    assert e.value.status == ks.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(C == 7.0)
    import gpu_util
    gpu_util.ensure_workspace.__defaults__[0].clear()


def test_selected_call_equals_forced_call_bitwise(gpu):
    import paper_2003_06795_amd.binding as ks
    for dtype, shape in (("f32", (300, 200, 100)), ("bf16", (300, 200, 128))):
        p = wl.make_problem(dtype, 0, 1, *shape, batch=2, alpha=1.0, beta=0.25, seed=4)
        dp = gpu.DeviceProblem(p)
        kid = ks.select(gpu.DT[dtype], p.M, p.N, p.K, p.batch, p.transA, p.transB)
        prep_workspace(gpu, p, kid)
        assert np.array_equal(dp.run(None), dp.run(kid))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_per_call_split_k_instances_with_and_without_workspace(gpu, dtype):
    """Instances whose K partitioning is chosen per call: long K and few tiles make them split when
    a workspace is registered; without one they run as a single kernel.  Both meet the bound."""
    import paper_2003_06795_amd.binding as ks
    dt = gpu.DT[dtype]
    auto = [k for k in ids_of(gpu, dtype) if ks.kernel_info(dt, k)["split_k"] == 0]
    assert auto, "the family has per-call split-K members"
    for tA, tB in LAYOUTS:
        p = wl.make_problem(dtype, tA, tB, 136, 264, 4096, batch=1, alpha=1.0, beta=0.5, seed=17, key=tA * 2 + tB,
                            dist="normal" if dtype == "bf16" else "uniform")
        dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
        for kid in auto:
            need = ks.workspace_bytes_needed(dt, kid, p.M, p.N, p.batch)
            assert need > 0
            gpu.ensure_workspace(need)
            split = dp.run(kid)
            check(p, split, ref, "%s kernel %d with workspace" % (dtype, kid))
            assert np.array_equal(split, dp.run(kid))
            try:
                ks.set_workspace(None)
                single = dp.run(kid)
            finally:
                gpu.ensure_workspace.__defaults__[0].clear()
            check(p, single, ref, "%s kernel %d without workspace" % (dtype, kid))


def plan_split(ks, gpu, dp, kid):
    p = dp.p
    return ks.gemm_plan(gpu.DT[p.dtype], kid, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                        p.beta, dp.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)["split_k"]


def test_forced_partition_counts_and_more_than_one_round_of_partitions(gpu):
    """ks_set_split_partitions forces the K partition count of the per-call split members (lowered
    to K-steps / 2 where a partition would hold fewer than two K-steps); every forced count meets
    the bound.  Left to itself an fp32 member may take more partitions than fill one round of
    work-groups: 152 tiles of 64 x 64 with K = 2592 are cut three ways or more."""
    import paper_2003_06795_amd.binding as ks
    auto = [k for k in ids_of(gpu, "f32") if ks.kernel_info(ks.F32, k)["split_k"] == 0]
    p = wl.make_problem("f32", 0, 1, 200, 136, 1000, alpha=-1.5, beta=0.5, seed=19)
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    gpu.ensure_workspace(64 * p.M * p.N * 4)
    try:
        for kid in auto:
            ki = ks.kernel_info(ks.F32, kid)
            steps = -(-(-(-p.K // ki["bk"])) // ki["k_waves"])
            for forced in (1, 2, 3, 7, 64):
                ks.set_split_partitions(forced)
                want = forced if forced == 1 or 2 * forced <= steps else max(steps // 2, 1)
                assert plan_split(ks, gpu, dp, kid) == want, (kid, forced, steps)
                check(p, dp.run(kid), ref, "f32 kernel %d, %d partitions forced" % (kid, forced))
        ks.set_split_partitions(0)
        with pytest.raises(Exception):
            ks.set_split_partitions(257)
        with pytest.raises(Exception):
            ks.set_split_partitions(-1)
        # bf16 members follow the forced count too
        q = wl.make_problem("bf16", 0, 0, 264, 136, 2048, alpha=1.0, beta=0.0, seed=19, key=1, dist="normal")
        dq, refq = gpu.DeviceProblem(q), gpu.oracle_full(q)
        kid16 = [k for k in ids_of(gpu, "bf16") if ks.kernel_info(ks.BF16, k)["split_k"] == 0][0]
        ks.set_split_partitions(5)
        assert plan_split(ks, gpu, dq, kid16) == 5
        check(q, dq.run(kid16), refq, "bf16 kernel %d, 5 partitions forced" % kid16)
    finally:
        ks.set_split_partitions(0)
    wide = [k for k in auto if ks.kernel_info(ks.F32, k)["bm"] == 64 and ks.kernel_info(ks.F32, k)["bn"] == 64 and
            ks.kernel_info(ks.F32, k)["threads"] == 512]
    assert wide, "the 64x64 member with two K groups chooses its split per call"
    r = wl.make_problem("f32", 0, 0, 1184, 480, 2592, seed=19, key=2)
    dr = gpu.DeviceProblem(r)
    gpu.ensure_workspace(ks.workspace_bytes_needed(ks.F32, wide[0], r.M, r.N, 1))
    s = plan_split(ks, gpu, dr, wide[0])
    assert s >= 3 and 152 * s > 256, s
    got = dr.run(wide[0])
    bb, ii, jj = gpu.sample_entries(r, 2000, 19, tile=64)
    err = float(np.max(np.abs(got[ii * r.ldc + jj].astype(np.float64) - gpu.oracle_entries(r, bb, ii, jj))))
    assert err <= tolerance(r), err


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_seeded_random_small_problems_every_kernel(gpu, dtype):
    """Brute force on tiny inputs: random sizes in [1, 70] (smaller than most tiles, so every edge
    predicate is exercised), random paddings, batch strides, broadcast operands, alpha/beta incl. 0."""
    import paper_2003_06795_amd.binding as ks
    r = np.random.default_rng(2024)
    for case in range(24):
        M, N, K = (int(v) for v in r.integers(1, 71, 3))
        if case % 6 == 0:
            K = int(r.integers(1, 4)) * 128                     # direct-to-LDS eligible K for bf16
            M, N = 8 * int(r.integers(1, 9)), 8 * int(r.integers(1, 9))
        batch = int(r.integers(1, 4))
        tA, tB = int(r.integers(0, 2)), int(r.integers(0, 2))
        pad = tuple(int(v) for v in r.integers(0, 3, 3) * (8 if case % 6 == 0 else 1))
        bpad = tuple(int(v) for v in r.integers(0, 2, 3) * 8)
        alpha = float(r.choice([1.0, -0.5, 2.0, 0.0]))
        beta = float(r.choice([0.0, 1.0, -1.5, 0.25]))
        bc = (bool(r.integers(0, 2)) and batch > 1, bool(r.integers(0, 2)) and batch > 1)
        p = wl.make_problem(dtype, tA, tB, M, N, K, batch=batch, alpha=alpha, beta=beta, seed=31, key=case,
                            pad=pad, batch_pad=bpad, broadcast=bc, dist="normal" if dtype == "bf16" else "uniform",
                            c_fill="nan" if beta == 0.0 else "uniform")
        dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
        for kid in ids_of(gpu, dtype):
            prep_workspace(gpu, p, kid)
            check(p, dp.run(kid), ref, "%s case %d (%d x %d x %d, batch %d, tA %d tB %d) kernel %d"
                  % (dtype, case, M, N, K, batch, tA, tB, kid))


# ----------------------------------------------------------------------------- K-sliced members, launch shapes

def test_k_sliced_members_with_empty_and_ragged_slices(gpu):
    """K shorter than the slices of a K-sliced member leaves trailing waves without work; K that
    is no multiple of 16 cuts the last non-empty slice."""
    import paper_2003_06795_amd.binding as ks
    sliced = [k for k in ids_of(gpu, "f32") if ks.kernel_info(ks.F32, k)["k_waves"] > 1]
    assert len(sliced) >= 8
    for K in (1, 7, 20, 33, 100, 257):
        for (tA, tB) in ((0, 0), (1, 1)):
            p = wl.make_problem("f32", tA, tB, 45, 70, K, batch=2, alpha=1.5, beta=0.5, seed=70 + K, key=tA)
            dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
            for kid in sliced:
                prep_workspace(gpu, p, kid)
                check(p, dp.run(kid), ref, "K-sliced kernel %d, K = %d, layout %d%d" % (kid, K, tA, tB))


def test_both_launch_shapes_agree_bitwise(gpu):
    """Small grids with small operands are launched three-dimensional, everything else as a
    renumbered one-dimensional grid; a batch count moves the same tiles from one form to the
    other (the operand bytes grow past the bound), and every batch item must come out the same."""
    import torch
    import paper_2003_06795_amd.binding as ks
    M, N, K = 96, 80, 136
    g = torch.Generator(device="cuda").manual_seed(5)
    A = torch.rand(M * K, device="cuda", generator=g) - 0.5
    B = torch.rand(K * N, device="cuda", generator=g) - 0.5
    for kid in (1, 5, 22, 28, 35, 36, 43, 58):
        one = torch.zeros(M * N, device="cuda")
        ks.gemm_f32_with_kernel(kid, 0, 0, M, N, K, 1.0, A, K, B, N, 0.0, one, N)            # 3-D launch
        batch = 64                                                                            # 64 x 94 KiB of operands
        need = ks.workspace_bytes_needed(ks.F32, kid, M, N, batch)
        if need:
            gpu.ensure_workspace(need)
        Ab, Bb = A.repeat(batch), B.repeat(batch)
        many = torch.zeros(batch * M * N, device="cuda")
        ks.gemm_f32_with_kernel(kid, 0, 0, M, N, K, 1.0, Ab, K, Bb, N, 0.0, many, N, batch, M * K, K * N, M * N)
        torch.cuda.synchronize()
        got = many.view(batch, M * N)
        info = ks.kernel_info(ks.F32, kid)
        if info["split_k"] == 1:
            assert torch.equal(got, one.expand(batch, M * N)), "kernel %d" % kid
        else:   # a per-call split may pick another partition count for the batched call
            assert torch.allclose(got, one.expand(batch, M * N), atol=1e-4), "kernel %d" % kid


def multi_tile_members(ks):
    """fp32 members whose work-groups can walk several tiles: large-tile MFMA, one K group, and
    (for a launch to do so) not a fixed split-K member."""
    out = []
    for k in range(ks.num_kernels(ks.F32)):
        i = ks.kernel_info(ks.F32, k)
        if i["core_name"] == "mfma32" and i["bm"] * i["bn"] >= 8192 and i["bn"] >= 128 and i["wm"] * i["wn"] <= 2048 \
                and i["k_waves"] == 1 and i["split_k"] <= 1:
            out.append(k)
    return out


def test_work_groups_walking_several_tiles(gpu):
    """Forced tile counts per work-group (ragged last work-group, tiles crossing batch items, edge
    tiles) give bit-identical results to one tile per work-group, which matches the oracle."""
    import paper_2003_06795_amd.binding as ks
    members = multi_tile_members(ks)
    assert len(members) >= 4
    ks.set_workspace(None)                      # per-call split members then run unsplit
    cases = [
        dict(transA=0, transB=0, M=300, N=280, K=1100, batch=2, alpha=1.0, beta=0.5),
        dict(transA=1, transB=1, M=515, N=260, K=1500, batch=1, alpha=-0.5, beta=0.0, pad=(4, 8, 4)),
        dict(transA=0, transB=1, M=130, N=129, K=2051, batch=3, alpha=1.0, beta=0.0),   # scalar loads
    ]
    try:
        for ci, c in enumerate(cases):
            c = dict(c)
            p = wl.make_problem("f32", c.pop("transA"), c.pop("transB"), c.pop("M"), c.pop("N"), c.pop("K"),
                                seed=21, key=ci, c_fill="uniform", **c)
            assert (p.M + p.N) * p.K * p.batch * 4 > (4 << 20)     # one-dimensional launch
            dp = gpu.DeviceProblem(p)
            ref = gpu.oracle_full(p)
            for kid in members:
                ks.set_tiles_per_workgroup(1)
                one = dp.run(kid)
                check(p, one, ref, "kernel %d case %d" % (kid, ci))
                for t in (2, 3, 7, 64):
                    ks.set_tiles_per_workgroup(t)
                    assert np.array_equal(dp.run(kid), one), "kernel %d case %d: %d tiles per work-group" % (kid, ci, t)
    finally:
        ks.set_tiles_per_workgroup(0)
        gpu.ensure_workspace.__defaults__[0].clear()


def test_several_tiles_with_a_single_short_k_step(gpu):
    """K shorter than one K-step and thousands of tiles: every step of the flattened loop ends a
    tile.  Automatic and forced counts agree bitwise; sampled entries match the oracle."""
    import torch
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f32", 0, 0, 6437, 2885, 20, seed=22, c_fill="nan")
    dp = gpu.DeviceProblem(p)
    bb, ii, jj = gpu.sample_entries(p, 2048, 5, tile=128)
    ref = gpu.oracle_entries(p, bb, ii, jj)
    flat = bb * p.strideC + ii * p.ldc + jj
    ks.set_workspace(None)
    try:
        for kid in multi_tile_members(ks):
            ks.set_tiles_per_workgroup(1)
            one = dp.run(kid)
            assert not np.isnan(one[~c_padding_mask(p)]).any()
            assert np.max(np.abs(one[flat].astype(np.float64) - ref)) <= tolerance(p), kid
            for t in (0, 5):
                ks.set_tiles_per_workgroup(t)
                assert np.array_equal(dp.run(kid), one), "kernel %d, %d tiles per work-group" % (kid, t)
    finally:
        ks.set_tiles_per_workgroup(0)
        gpu.ensure_workspace.__defaults__[0].clear()


def test_several_tiles_with_bias_and_bf16_output(gpu):
    """The multi-tile form goes through the same bias and bf16-output epilogues: forced tile counts
    agree bitwise with one tile per work-group, which matches the oracle."""
    import torch
    import paper_2003_06795_amd.binding as ks
    from oracle import gemm as og
    p = wl.make_problem("f32", 0, 1, 390, 261, 1700, batch=2, alpha=0.75, beta=0.5, seed=23, c_fill="uniform")
    assert (p.M + p.N) * p.K * p.batch * 4 > (4 << 20)
    dp = gpu.DeviceProblem(p)
    bias = (2.0 * wl.uniform_pm1(p.N, 23, 7)).astype(np.float32)
    bias_dev = torch.from_numpy(bias).cuda()
    ref = p.C0.copy()
    og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref,
                 p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    c16 = wl.f32_to_bf16_rne(p.C0)
    ref16 = c16.copy()
    og.gemm_out_bf16(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref16,
                     p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    live = ~c_padding_mask(p)
    args = (p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta)
    tail = (p.batch, p.strideA, p.strideB, p.strideC)

    def with_bias(kid):
        C = dp.C0.clone()
        ks.gemm_bias(ks.F32, kid, *args, C, p.ldc, bias_dev, *tail)
        torch.cuda.synchronize()
        return C.cpu().numpy()

    def with_out16(kid):
        C = torch.from_numpy(c16.view(np.int16).copy()).cuda()
        ks.gemm_out_bf16(ks.F32, kid, *args, C, p.ldc, bias_dev, *tail)
        torch.cuda.synchronize()
        return C.cpu().numpy().view(np.uint16)

    ks.set_workspace(None)
    try:
        for kid in multi_tile_members(ks):
            ks.set_tiles_per_workgroup(1)
            one, one16 = with_bias(kid), with_out16(kid)
            tol = tolerance(p) + 2.0 ** -22 * (float(np.max(np.abs(bias))) + float(np.max(np.abs(ref[live]))))
            assert np.max(np.abs(one[live].astype(np.float64) - ref[live])) <= tol, kid
            # bf16 output: within one bf16 step of the oracle's rounding of its fp64 value
            a, b = wl.bf16_to_f32(one16[live]).astype(np.float64), wl.bf16_to_f32(ref16[live]).astype(np.float64)
            assert np.max(np.abs(a - b) / np.maximum(np.abs(b), 1.0)) <= 2.0 ** -7, kid
            ks.set_tiles_per_workgroup(3)
            assert np.array_equal(with_bias(kid), one), kid
            assert np.array_equal(with_out16(kid), one16), kid
    finally:
        ks.set_tiles_per_workgroup(0)
        gpu.ensure_workspace.__defaults__[0].clear()
