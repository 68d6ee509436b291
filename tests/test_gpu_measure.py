"""The measurement aids behind the C ABI (pure MFMA loop, two-group kernel with data paths left out
and with its clock probe): argument checks, plausible outputs, and that the probed kernel still
computes the GEMM."""
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


def test_pure_mfma_loop_reports_a_rate_and_a_clock(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    ops16 = torch.zeros(ks.MFMA_PROBE_BYTES // 2, dtype=torch.bfloat16, device="cuda")
    ops32 = torch.zeros(ks.MFMA_PROBE_BYTES // 4, dtype=torch.float32, device="cuda")
    for dt, ops, fragment, peak in ((ks.BF16, ops16, 32, 2516.6), (ks.BF16, ops16, 16, 2516.6),
                                    (ks.F16, ops16, 32, 2516.6), (ks.F16, ops16, 16, 2516.6),
                                    (ks.F32, ops32, 32, 157.3)):
        tf, mhz = ks.mfma_sustained(dt, ops, rounds=200, fragment=fragment)
        assert 0.2 * peak < tf < 1.05 * peak, (dt, fragment, tf)
        assert 500.0 < mhz < 3000.0, (dt, fragment, mhz)
    with pytest.raises(ks.KsError):
        ks.mfma_sustained(ks.F32, ops32, rounds=10, fragment=16)       # no 16x16x32 fp32 form
    with pytest.raises(ks.KsError):
        ks.mfma_sustained(ks.BF16, ops16, rounds=10, fragment=8)
    with pytest.raises(ks.KsError):
        ks.mfma_sustained(ks.BF16, ops16, nbytes=1024, rounds=10)      # buffer too small


@pytest.mark.parametrize("mode", [0, 4, 5])
def test_probed_kernel_still_computes_the_product(gpu, mode):
    """Modes 0, 4 and 5 leave the computation alone: sampled entries against the oracle."""
    import torch
    import paper_2003_06795_amd.binding as ks
    M, N, K = 512, 768, 448
    p = wl.make_problem("bf16", 0, 1, M, N, K, seed=41, key=mode, dist="normal", c_fill="zeros")
    A = torch.from_numpy(p.A.view(np.int16)).cuda()
    B = torch.from_numpy(p.B.view(np.int16)).cuda()
    C = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    out = ks.bf16_ablation(mode, A, B, C, M, N, K, iters=2)
    if mode >= 4:
        ms, mhz = out
        assert 500.0 < mhz < 3000.0
    else:
        ms = out
    assert ms.shape == (2,) and float(ms.min()) > 0.0
    bb, ii, jj = gpu.sample_entries(p, 1024, 7)
    got = C.cpu().numpy()[ii * N + jj]
    ref = gpu.oracle_entries(p, bb, ii, jj)
    assert float(np.max(np.abs(got.astype(np.float64) - ref))) <= tolerance(p)


def test_ablation_rejects_what_the_kernel_cannot_take(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    A = torch.zeros(256 * 128, dtype=torch.bfloat16, device="cuda")
    C = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    for bad in (dict(M=200, N=256, K=128), dict(M=256, N=256, K=64), dict(M=256, N=256, K=100)):
        with pytest.raises(ks.KsError):
            ks.bf16_ablation(0, A, A, C, bad["M"], bad["N"], bad["K"], iters=1)
    with pytest.raises(ks.KsError):
        ks.bf16_ablation(9, A, A, C, 256, 256, 128, iters=1)
