"""Pins for the bias form of the C GEMM oracle (oracle_gemm_bias_*): numpy's fp64 matmul with a
broadcast vector, an interpreter loop, and cases that fix which axis the vector runs along."""
import itertools

import numpy as np
import pytest

import workloads as wl
from oracle import gemm as og
from helpers import operand_matrices, c_views, c_padding_mask


def bias_vector(p, seed=0):
    return wl.uniform_pm1(p.N, 900 + seed, 77)


def run_bias(p, bias):
    C = p.C0.copy()
    og.gemm_bias(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb,
                 p.beta, C, p.ldc, bias, p.batch, p.strideA, p.strideB, p.strideC)
    return C


def run_plain(p):
    C = p.C0.copy()
    og.gemm(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb,
            p.beta, C, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
    return C


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_matches_numpy_fp64_matmul_plus_row_broadcast(dtype, tA, tB):
    p = wl.make_problem(dtype, tA, tB, 23, 41, 37, batch=2, alpha=0.75, beta=1.5, seed=21,
                        key=tA * 2 + tB, pad=(2, 1, 3), batch_pad=(0, 5, 6))
    bias = bias_vector(p, tA * 2 + tB)
    As, Bs, Cs = operand_matrices(p)
    C = run_bias(p, bias)
    for g, A, B, C0 in zip(c_views(p, C), As, Bs, Cs):
        ref = np.float64(np.float32(p.alpha)) * (A @ B) + np.float64(np.float32(p.beta)) * C0.astype(np.float64)
        ref = ref + bias.astype(np.float64)[None, :]          # one value per column, every row
        assert np.max(np.abs(g - ref.astype(np.float32))) <= 2.0 ** -23 * np.max(np.abs(ref))
    mask = c_padding_mask(p)
    assert np.array_equal(C[mask], p.C0[mask])


def test_vector_runs_along_columns_not_rows():
    # M != N and a bias that differs in every entry: adding bias[i] instead of bias[j] either
    # reads out of range or lands on other entries
    p = wl.make_problem("f32", 0, 0, 5, 9, 3, alpha=0.0, beta=0.0, seed=4)
    bias = np.arange(1, 10, dtype=np.float32)
    g = c_views(p, run_bias(p, bias))[0]
    assert np.array_equal(g, np.tile(bias, (5, 1)))           # alpha = beta = 0: C is the bias rows


def test_k_zero_gives_beta_c_plus_bias_and_null_bias_is_plain_gemm():
    p = wl.make_problem("f32", 1, 0, 6, 4, 0, batch=2, alpha=3.0, beta=-2.0, seed=8)
    bias = bias_vector(p)
    for g, C0 in zip(c_views(p, run_bias(p, bias)), operand_matrices(p)[2]):
        ref = (-2.0 * C0.astype(np.float64) + bias.astype(np.float64)[None, :]).astype(np.float32)
        assert np.array_equal(g, ref)
    q = wl.make_problem("bf16", 0, 1, 12, 10, 33, batch=2, alpha=1.0, beta=0.5, seed=9, dist="normal")
    assert np.array_equal(run_bias(q, None), run_plain(q))


def test_interpreter_loop_and_single_rounding():
    p = wl.make_problem("f32", 1, 1, 4, 6, 7, alpha=1.5, beta=0.25, seed=13)
    bias = bias_vector(p, 1)
    got = c_views(p, run_bias(p, bias))[0]
    a32 = float(np.float32(p.alpha)); b32 = float(np.float32(p.beta))
    for i in range(p.M):
        for j in range(p.N):
            acc = 0.0
            for k in range(p.K):
                acc += float(p.A[k * p.lda + i]) * float(p.B[j * p.ldb + k])
            ref = a32 * acc + b32 * float(p.C0[i * p.ldc + j]) + float(bias[j])
            assert got[i, j] == np.float32(ref)
    # one rounding: a bias far below half an ulp of the fp32 result must not be lost when the
    # fp64 sum crosses a rounding boundary; check against rounding the plain result first
    p = wl.make_problem("f32", 0, 0, 3, 3, 2, alpha=1.0, beta=0.0, seed=2)
    plain = c_views(p, run_plain(p))[0].astype(np.float64)
    tiny = np.full(3, 2.0 ** -30, dtype=np.float32)
    with_bias = c_views(p, run_bias(p, tiny))[0]
    As, Bs, _ = operand_matrices(p)
    exact = (As[0] @ Bs[0]) + tiny.astype(np.float64)[None, :]
    assert np.array_equal(with_bias, exact.astype(np.float32))
    assert plain.shape == exact.shape


def test_sum_is_rounded_once_tie_case():
    # A*B = 1 + 2^-24 exactly, a tie that fp32 rounds down to 1; the bias 2^-40 lifts the fp64 sum
    # above the tie, so one rounding gives 1 + 2^-23, while rounding before adding gives 1
    A = np.array([1.0, 2.0 ** -12], dtype=np.float32)
    B = np.array([1.0, 2.0 ** -12], dtype=np.float32)
    C = np.zeros(1, dtype=np.float32)
    og.gemm_bias("f32", 0, 0, 1, 1, 2, 1.0, A, 2, B, 1, 0.0, C, 1, np.array([2.0 ** -40], dtype=np.float32))
    assert C[0] == np.float32(1.0 + 2.0 ** -23)
    og.gemm("f32", 0, 0, 1, 1, 2, 1.0, A, 2, B, 1, 0.0, C, 1)
    assert C[0] == np.float32(1.0)


def test_short_bias_is_rejected():
    p = wl.make_problem("f32", 0, 0, 3, 8, 2, seed=1)
    with pytest.raises(ValueError):
        run_bias(p, np.zeros(7, dtype=np.float32))
