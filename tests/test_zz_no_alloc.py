"""The entry point that allocates nothing (ks_gemm_static_scratch): split-K partial sums go to the
library's static device array instead of the registered workspace.  Its output is compared with
the existing entry point (ks_gemm_*_with_kernel on a registered workspace of the same size, so
that per-call split counts agree) bit for bit, and with the CPU oracle within the stated bound,
on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import workloads as wl
from helpers import tolerance

pytestmark = pytest.mark.gpu

STATIC_BYTES = 16 << 20


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import gpu_util
    return gpu_util


def _pair(gpu, dtype, kid, shape, tA, tB, alpha, beta, batch, key, ws):
    """Runs the static-scratch call and the workspace call on the same inputs; returns both outputs
    and the problem."""
    import torch
    import paper_2003_06795_amd.binding as ks
    M, N, K = shape
    p = wl.make_problem(dtype, tA, tB, M, N, K, batch=batch, alpha=alpha, beta=beta, seed=21, key=key,
                        dist="normal" if dtype != "f32" else "uniform")
    dp = gpu.DeviceProblem(p)
    args = (p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta)
    tail = (p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
    # the static array keeps whatever the previous call left there: poison the registered
    # workspace only (the library's own array cannot be reached from here, which is the point)
    ws.fill_(float("nan"))
    ks.set_workspace(ws, STATIC_BYTES)
    C_ref = dp.C0.clone()
    gpu.GEMM_K[dtype](kid, *args, C_ref, *tail)
    ks.set_workspace(None)                       # the new entry point must not need it
    C_new = dp.C0.clone()
    ks.gemm_static_scratch(gpu.DT[dtype], kid, *args, C_new, *tail)
    torch.cuda.synchronize()
    return p, C_new.cpu().numpy()[:p.C0.size], C_ref.cpu().numpy()[:p.C0.size]


CASES = [
    # dtype, kernel id (fixed split 4 / per-call split / fixed 64 / per-call), big shape, small shape
    ("f32", 12, (520, 392, 1000), (200, 136, 264)),
    ("f32", 42, (96, 3016, 3392), (72, 200, 1800)),
    ("f32", 37, (48, 64, 4096), (16, 32, 520)),
    ("bf16", 18, (128, 192, 8192), (64, 64, 4096)),
    ("bf16", 25, (512, 256, 16384), (256, 256, 2048)),
    ("bf16", 27, (320, 200, 4104), (136, 72, 1000)),
]


@pytest.mark.parametrize("dtype,kid,big,small", CASES)
def test_static_scratch_matches_workspace_call(gpu, dtype, kid, big, small):
    import torch
    import paper_2003_06795_amd.binding as ks
    ws = torch.empty(STATIC_BYTES // 4, dtype=torch.float32, device="cuda")
    assert ks.kernel_info(gpu.DT[dtype], kid)["split_k"] != 1
    try:
        for n, shape in enumerate((big, small)):          # two calls in a row, the second smaller
            for (tA, tB) in ((0, 0), (0, 1)):
                p, new, ref = _pair(gpu, dtype, kid, shape, tA, tB, 1.25, -0.5, 2 if n == 0 else 1, n * 4 + tB, ws)
                assert np.array_equal(new.view(np.uint32), ref.view(np.uint32)), \
                    "%s kernel %d %s: static-scratch call differs from the workspace call" % (dtype, kid, shape)
                want = gpu.oracle_full(p)
                err = float(np.max(np.abs(new.astype(np.float64) - want)))
                assert err <= tolerance(p), "%s kernel %d %s: %.3e > %.3e" % (dtype, kid, shape, err, tolerance(p))
    finally:
        ks.set_workspace(None)


def test_static_scratch_selected_kernel_and_limit(gpu):
    """kernel_id < 0 selects like ks_gemm_*; a forced fixed-split member whose partial sums exceed the
    static array is refused with the workspace status and leaves C untouched."""
    import torch
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f32", 0, 1, 264, 200, 1544, seed=22, key=1)
    dp = gpu.DeviceProblem(p)
    C = dp.C0.clone()
    ks.set_workspace(None)
    ks.gemm_static_scratch(ks.F32, -1, p.transA, p.transB, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb,
                           p.beta, C, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
    torch.cuda.synchronize()
    err = float(np.max(np.abs(C.cpu().numpy()[:p.C0.size].astype(np.float64) - gpu.oracle_full(p))))
    assert err <= tolerance(p)
    # fp32 id 12 has split_k = 4: 4 * 2048 * 1024 * 4 bytes = 32 MiB > 16 MiB
    M, N, K = 2048, 1024, 64
    A = torch.zeros(M * K, device="cuda")
    B = torch.zeros(K * N, device="cuda")
    C = torch.full((M * N,), 7.0, device="cuda")
    with pytest.raises(ks.KsError) as e:
        ks.gemm_static_scratch(ks.F32, 12, 0, 0, M, N, K, 1.0, A, K, B, N, 0.0, C, N)
    assert e.value.status == ks.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((C == 7.0).all())
