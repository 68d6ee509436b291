"""Pins for the bf16-output form of the C GEMM oracle: the rounding against an independent
integer-arithmetic rounding of float32 values, against the format's definition at ties, subnormals
and overflow, a single-rounding case, and the GEMM against numpy fp64 + that rounding."""
import itertools
import math

import numpy as np
import pytest

import workloads as wl
from oracle import gemm as og
from helpers import operand_matrices


def test_rounding_matches_integer_rne_on_float32_values():
    r = np.random.default_rng(3)
    x = np.concatenate([
        r.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** r.integers(-30, 30, 20000).astype(np.float32),
        (r.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32)).view(np.float32)])
    x = x[np.isfinite(x)]
    ref = wl.f32_to_bf16_rne(x)                      # adds 0x7FFF + lsb to the bit pattern
    got = np.array([og.round_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_rounding_landmarks_from_the_format_definition():
    f = og.round_to_bf16
    assert f(1.0) == 0x3F80 and f(-2.0) == 0xC000 and f(0.0) == 0x0000 and f(-0.0) == 0x8000
    assert f(1.0 + 2.0 ** -8) == 0x3F80              # tie -> even (down)
    assert f(1.0 + 3 * 2.0 ** -8) == 0x3F82          # tie -> even (up)
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81  # just above the tie
    assert f(2.0 ** -133) == 0x0001                  # smallest subnormal
    assert f(2.0 ** -134) == 0x0000                  # tie with zero -> even
    assert f(3 * 2.0 ** -134) == 0x0002               # 1.5 subnormal units: tie -> even (2)
    assert f(2.0 ** -126) == 0x0080                  # smallest normal
    big = (2.0 - 2.0 ** -7) * 2.0 ** 127             # largest finite bf16
    assert f(big) == 0x7F7F and f(big * (1 + 2.0 ** -10)) == 0x7F7F
    assert f(2.0 ** 128) == 0x7F80 and f(-1e300) == 0xFF80 and f(big + 2.0 ** 119) == 0x7F80
    assert f(math.inf) == 0x7F80 and (f(math.nan) & 0x7FFF) > 0x7F80


def test_single_rounding_not_via_float32():
    # 1 + 2^-8 + 2^-30 rounds to the tie 1 + 2^-8 in float32, and from there down to 1;
    # rounded once from fp64 it lies above the tie and goes up
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert og.round_to_bf16(x) == 0x3F81
    assert wl.f32_to_bf16_rne(np.array([x], dtype=np.float32))[0] == 0x3F80


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("tA,tB", [(0, 0), (1, 1)])
def test_gemm_matches_numpy_then_rounding(dtype, tA, tB):
    p = wl.make_problem(dtype, tA, tB, 19, 23, 31, batch=2, alpha=1.25, beta=-0.5, seed=51, key=tA,
                        pad=(2, 1, 3), batch_pad=(0, 3, 5), dist="normal" if dtype != "f32" else "uniform")
    bias = wl.uniform_pm1(p.N, 52, 1)
    C16 = wl.f32_to_bf16_rne(p.C0)
    before = C16.copy()
    og.gemm_out_bf16(dtype, tA, tB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C16, p.ldc, bias,
                     p.batch, p.strideA, p.strideB, p.strideC)
    As, Bs, _ = operand_matrices(p)
    c0 = wl.bf16_to_f32(before).astype(np.float64)
    touched = np.zeros(C16.size, dtype=bool)
    for t, (A, B) in enumerate(zip(As, Bs)):
        ref = np.float64(np.float32(p.alpha)) * (A @ B)
        for i in range(p.M):
            for j in range(p.N):
                idx = t * p.strideC + i * p.ldc + j
                v = ref[i, j] + np.float64(np.float32(p.beta)) * c0[idx] + np.float64(bias[j])
                want = og.round_to_bf16(v)
                # numpy's matmul sums in another order: allow the neighbouring bf16 value when v
                # sits within that difference of a rounding boundary
                if C16[idx] != want:
                    lo, hi = og.round_to_bf16(v - 1e-12 * abs(v) - 1e-300), og.round_to_bf16(v + 1e-12 * abs(v) + 1e-300)
                    assert C16[idx] in (lo, hi), (t, i, j)
                touched[idx] = True
    assert np.array_equal(C16[~touched], before[~touched])       # padding keeps its bits


def test_beta_zero_ignores_old_bits_and_interpreter_loop():
    p = wl.make_problem("f32", 0, 1, 4, 5, 6, alpha=0.75, beta=0.0, seed=9)
    C16 = np.full(p.C0.size, 0x7FC0, dtype=np.uint16)            # NaN bit patterns
    og.gemm_out_bf16("f32", 0, 1, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, 0.0, C16, p.ldc)
    for i in range(p.M):
        for j in range(p.N):
            acc = 0.0
            for k in range(p.K):
                acc += float(p.A[i * p.lda + k]) * float(p.B[j * p.ldb + k])
            assert C16[i * p.ldc + j] == og.round_to_bf16(0.75 * acc)
