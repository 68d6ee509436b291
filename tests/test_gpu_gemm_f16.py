"""GPU parity of the fp16-input form (KS_F16: the 16-bit family run with binary16 MFMAs) against
the fp64 CPU oracle: every instantiation, both code paths, four layouts, ragged and aligned
shapes, split-K, bias, the selector path, and bit-exact small-integer cases."""
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


def check(p, got, ref, what, extra=0.0):
    live = ~c_padding_mask(p)
    err = float(np.max(np.abs(got[live].astype(np.float64) - ref[live].astype(np.float64))))
    assert np.all(np.isfinite(got[live])), what
    assert err <= tolerance(p) + extra, "%s: max|diff| %.3e > tol %.3e" % (what, err, tolerance(p) + extra)
    # products of binary16 values are exact in fp32 and the sum is kept in fp32: the error is a
    # rounding per addition, far inside the stated bound
    ma, mb, _ = p.max_abs()
    assert err <= max(p.K, 1) * 2.0 ** -22 * (abs(p.alpha) * p.K * ma * mb + abs(p.beta) + 1.0) + extra, what
    mask = c_padding_mask(p)
    assert np.array_equal(got[mask], p.C0[mask], equal_nan=True), what + ": wrote outside C's logical entries"


def prep(gpu, p, kid):
    import paper_2003_06795_amd.binding as ks
    need = ks.workspace_bytes_needed(ks.F16, kid, p.M, p.N, p.batch)
    if need:
        gpu.ensure_workspace(need)


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_every_kernel_ragged_and_aligned(gpu, tA, tB):
    import paper_2003_06795_amd.binding as ks
    assert ks.num_kernels(ks.F16) == ks.num_kernels(ks.BF16)
    ragged = wl.make_problem("f16", tA, tB, 150, 201, 264, batch=2, alpha=0.5, beta=-1.25, seed=41,
                             key=2 * tA + tB, pad=(0, 0, 3), dist="normal")
    aligned = wl.make_problem("f16", tA, tB, 256, 320, 512, alpha=1.0, beta=0.0, seed=42, key=2 * tA + tB,
                              c_fill="nan", dist="normal")
    for p in (ragged, aligned):
        dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
        for kid in range(ks.num_kernels(ks.F16)):
            prep(gpu, p, kid)
            print("f16", tA, tB, p.M, "kernel", kid, flush=True)
            check(p, dp.run(kid), ref, "f16 kernel %d (%d,%d) M=%d" % (kid, tA, tB, p.M))
        got = dp.run(None)
        sel = ks.select(ks.F16, p.M, p.N, p.K, p.batch, tA, tB)
        assert sel == ks.select(ks.BF16, p.M, p.N, p.K, p.batch, tA, tB)
        check(p, got, ref, "f16 selector")


def test_both_code_paths_bitwise_and_integers_exact(gpu):
    import paper_2003_06795_amd.binding as ks
    p = wl.make_problem("f16", 0, 1, 192, 128, 256, alpha=1.0, beta=0.0, seed=43, dist="ints")
    dp, ref = gpu.DeviceProblem(p), gpu.oracle_full(p)
    live = ~c_padding_mask(p)
    for kid in range(ks.num_kernels(ks.F16)):
        prep(gpu, p, kid)
        fast = dp.run(kid)
        ks.set_fast_path(0)
        try:
            generic = dp.run(kid)
        finally:
            ks.set_fast_path(1)
        assert np.array_equal(fast, generic), "kernel %d: the two code paths differ" % kid
        assert np.array_equal(fast[live], ref[live]), "kernel %d: integer case not exact" % kid


def test_values_that_only_binary16_represents(gpu):
    # 1 + 2^-10 is exact in binary16 and not in bf16 (7 fraction bits): a kernel that treated the
    # bits as bf16, or the oracle doing so, would be far off
    import torch
    import paper_2003_06795_amd.binding as ks
    M = N = 64; K = 128
    a = np.full(M * K, 1.0 + 2.0 ** -10, dtype=np.float32)
    b = np.full(K * N, 0.5, dtype=np.float32)
    A = torch.from_numpy(wl.f32_to_f16_bits(a).view(np.int16)).cuda()
    B = torch.from_numpy(wl.f32_to_f16_bits(b).view(np.int16)).cuda()
    C = torch.zeros(M * N, dtype=torch.float32, device="cuda")
    ks.gemm_f16(0, 0, M, N, K, 1.0, A, K, B, N, 0.0, C, N)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy(), np.full(M * N, K * 0.5 * (1.0 + 2.0 ** -10), dtype=np.float32))


def test_bias_and_timing_entry_points_accept_fp16(gpu):
    import torch
    import paper_2003_06795_amd.binding as ks
    from oracle import gemm as og
    p = wl.make_problem("f16", 1, 0, 96, 80, 160, alpha=1.0, beta=0.5, seed=44, dist="normal")
    bias = (2.0 * wl.uniform_pm1(p.N, 45, 1)).astype(np.float32)
    ref = p.C0.copy()
    og.gemm_bias("f16", 1, 0, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, ref, p.ldc, bias)
    dp = gpu.DeviceProblem(p)
    C = dp.C0.clone()
    ks.gemm_bias(ks.F16, -1, 1, 0, p.M, p.N, p.K, p.alpha, dp.A, p.lda, dp.B, p.ldb, p.beta, C, p.ldc,
                 torch.from_numpy(bias).cuda())
    torch.cuda.synchronize()
    check(p, C.cpu().numpy()[:p.C0.size], ref, "f16 bias", extra=2.0 ** -22 * (2.0 + float(np.max(np.abs(ref)))))
    ms = ks.time_gemm(ks.F16, -1, 1, 0, p.M, p.N, p.K, 1.0, dp.A, p.lda, dp.B, p.ldb, 0.0, dp.C0.clone(), p.ldc,
                      warmup=1, iters=3, reps=2)
    assert ms.shape == (3,) and np.all(ms > 0)
