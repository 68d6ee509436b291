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
