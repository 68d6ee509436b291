"""Pins for the C GEMM oracle (oracle/gemm_oracle.c) against things other than itself:
numpy's fp64 matmul, a pure-Python triple loop, closed forms and invariants."""
import itertools

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import workloads as wl
from oracle import gemm as og
from helpers import operand_matrices, c_views, c_padding_mask


def run_oracle(p):
    C = p.C0.copy()
    og.gemm(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb,
            p.beta, C, p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
    return C


def numpy_reference(p):
    """Library routine: float64 matmul per batch item, epilogue in float64, one rounding."""
    As, Bs, Cs = operand_matrices(p)
    outs = []
    for A, B, C0 in zip(As, Bs, Cs):
        acc = A @ B if p.K > 0 else np.zeros((p.M, p.N))
        o = np.float64(np.float32(p.alpha)) * acc
        if p.beta != 0.0:
            o = o + np.float64(np.float32(p.beta)) * C0.astype(np.float64)
        outs.append(o)
    return outs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_matches_numpy_fp64_matmul(dtype, tA, tB):
    p = wl.make_problem(dtype, tA, tB, 37, 29, 53, batch=3, alpha=1.25, beta=-0.5, seed=11,
                        key=tA * 2 + tB, pad=(3, 5, 2), batch_pad=(7, 0, 4))
    got = c_views(p, run_oracle(p))
    for g, ref in zip(got, numpy_reference(p)):
        # both are fp64 sums of the same exact products; only the order differs
        np.testing.assert_allclose(g.astype(np.float64), ref, rtol=0, atol=5e-7 * 53)
        scale = np.max(np.abs(ref))
        assert np.max(np.abs(g - ref.astype(np.float32))) <= 2.0 ** -23 * scale


def test_broadcast_strides_and_padding_untouched():
    p = wl.make_problem("f32", 0, 1, 9, 7, 5, batch=4, alpha=2.0, beta=0.0, seed=3,
                        pad=(1, 2, 3), batch_pad=(0, 0, 5), broadcast=(True, False))
    C = run_oracle(p)
    for g, ref in zip(c_views(p, C), numpy_reference(p)):
        np.testing.assert_allclose(g, ref.astype(np.float32), rtol=1e-6, atol=1e-6)
    mask = c_padding_mask(p)
    assert np.array_equal(C[mask], p.C0[mask])          # gaps between rows / items keep their bits


def python_triple_loop(p):
    """The definition once more, in interpreter arithmetic (Python floats are fp64)."""
    a = p.A if p.dtype == "f32" else wl.bf16_to_f32(p.A)
    b = p.B if p.dtype == "f32" else wl.bf16_to_f32(p.B)
    out = p.C0.copy()
    al, be = float(np.float32(p.alpha)), float(np.float32(p.beta))
    for t in range(p.batch):
        for i in range(p.M):
            for j in range(p.N):
                acc = 0.0
                for k in range(p.K):
                    x = a[t * p.strideA + (k * p.lda + i if p.transA else i * p.lda + k)]
                    y = b[t * p.strideB + (j * p.ldb + k if p.transB else k * p.ldb + j)]
                    acc += float(x) * float(y)
                idx = t * p.strideC + i * p.ldc + j
                v = al * acc
                if be != 0.0:
                    v += be * float(p.C0[idx])
                out[idx] = np.float32(v)
    return out


@settings(max_examples=60, deadline=None)
@given(M=st.integers(0, 12), N=st.integers(0, 12), K=st.integers(0, 12), batch=st.integers(0, 3),
       tA=st.integers(0, 1), tB=st.integers(0, 1), dtype=st.sampled_from(["f32", "bf16"]),
       alpha=st.sampled_from([1.0, 0.0, -2.0, 0.375]), beta=st.sampled_from([0.0, 1.0, 0.5, -1.5]),
       pads=st.tuples(st.integers(0, 3), st.integers(0, 3), st.integers(0, 3)),
       bcast=st.tuples(st.booleans(), st.booleans()), seed=st.integers(0, 1000))
def test_bitwise_equal_to_python_loops(M, N, K, batch, tA, tB, dtype, alpha, beta, pads, bcast, seed):
    p = wl.make_problem(dtype, tA, tB, M, N, K, batch=batch, alpha=alpha, beta=beta, seed=seed,
                        pad=pads, batch_pad=(1, 2, 3), broadcast=bcast)
    # same order of operations in the same precision -> identical bits, padding included
    assert np.array_equal(run_oracle(p), python_triple_loop(p))


@pytest.mark.parametrize("alpha", [1.0, 2.0, 0.5])
def test_identity_left(alpha):
    n = 23
    p = wl.make_problem("f32", 0, 0, n, 31, n, alpha=alpha, beta=1.0, seed=5)
    p.A = np.eye(n, dtype=np.float32).ravel()
    Bm = p.B.reshape(n, 31)
    C0 = p.C0.reshape(n, 31)
    expect = (np.float32(alpha) * Bm.astype(np.float64) + C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(run_oracle(p).reshape(n, 31), expect)


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_permutation_matrices_move_rows_and_columns(tA, tB):
    """A permutation operand only relocates the other operand's entries: bit-exact, and it
    fails if op() or an index is transposed."""
    M = K = 19
    N = 13
    r = np.random.default_rng(9)
    perm = r.permutation(M)
    P = np.zeros((M, K), dtype=np.float32)
    P[np.arange(M), perm] = 1.0                      # (P X)[i, :] = X[perm[i], :]
    X = wl.uniform_pm1(K * N, 9, 1).reshape(K, N)
    p = wl.make_problem("f32", tA, tB, M, N, K, seed=9)
    p.A = np.ascontiguousarray(P.T if tA else P).ravel()
    p.B = np.ascontiguousarray(X.T if tB else X).ravel()
    p.lda, p.ldb = (M if tA else K), (K if tB else N)
    got = run_oracle(p).reshape(M, N)
    assert np.array_equal(got, X[perm, :])
    # permutation on the right: (X' Q)[:, j] = X'[:, q[j]]
    q = r.permutation(N)
    Q = np.zeros((N, N), dtype=np.float32)
    Q[q, np.arange(N)] = 1.0
    Xp = wl.uniform_pm1(M * N, 9, 2).reshape(M, N)
    p2 = wl.make_problem("f32", tA, tB, M, N, N, seed=9)
    p2.A = np.ascontiguousarray(Xp.T if tA else Xp).ravel()
    p2.B = np.ascontiguousarray(Q.T if tB else Q).ravel()
    p2.lda, p2.ldb = (M if tA else N), N
    assert np.array_equal(run_oracle(p2).reshape(M, N), Xp[:, q])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_ones_closed_form(dtype):
    M, N, K = 11, 17, 300
    alpha, beta = 0.5, -2.0
    p = wl.make_problem(dtype, 0, 0, M, N, K, alpha=alpha, beta=beta, seed=2)
    one = np.float32(1.0) if dtype == "f32" else np.uint16(0x3F80)
    p.A = np.full_like(p.A, one)
    p.B = np.full_like(p.B, one)
    expect = (K * alpha + beta * p.C0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(run_oracle(p), expect)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_integers_exact_against_int64_matmul(dtype):
    p = wl.make_problem(dtype, 1, 0, 33, 21, 77, batch=2, alpha=1.0, beta=0.0, seed=4, dist="ints")
    As, Bs, _ = operand_matrices(p)
    got = c_views(p, run_oracle(p))
    for A, B, g in zip(As, Bs, got):
        ref = A.astype(np.int64) @ B.astype(np.int64)     # integer arithmetic, no rounding at all
        assert np.array_equal(g.astype(np.int64), ref)
        assert np.array_equal(g, ref.astype(np.float32))


def test_one_hot_lands_on_one_entry():
    M, N, K = 9, 8, 7
    for (i, k, j) in [(0, 0, 0), (8, 6, 7), (3, 2, 5), (0, 6, 7), (8, 0, 0)]:
        for tA, tB in itertools.product((0, 1), (0, 1)):
            p = wl.make_problem("f32", tA, tB, M, N, K, c_fill="zeros")
            p.A[:] = 0
            p.B[:] = 0
            p.A[(k * p.lda + i) if tA else (i * p.lda + k)] = 3.0
            p.B[(j * p.ldb + k) if tB else (k * p.ldb + j)] = -2.0
            C = run_oracle(p).reshape(M, N)
            expect = np.zeros((M, N), dtype=np.float32)
            expect[i, j] = -6.0
            assert np.array_equal(C, expect)


def test_beta_zero_does_not_read_c_and_alpha_zero_still_multiplies():
    p = wl.make_problem("f32", 0, 0, 5, 6, 7, alpha=1.0, beta=0.0, seed=1, c_fill="nan")
    assert np.all(np.isfinite(run_oracle(p)))
    p = wl.make_problem("f32", 0, 0, 5, 6, 7, alpha=0.0, beta=1.0, seed=1)
    p.A[3] = np.nan                                         # row 0 of A
    C = run_oracle(p).reshape(5, 6)
    assert np.all(np.isnan(C[0])) and np.array_equal(C[1:], p.C0.reshape(5, 6)[1:])


def test_k_zero_scales_c():
    p = wl.make_problem("f32", 0, 0, 4, 5, 0, alpha=3.0, beta=0.5, seed=6)
    assert np.array_equal(run_oracle(p), (0.5 * p.C0.astype(np.float64)).astype(np.float32))
    p = wl.make_problem("f32", 0, 0, 4, 5, 0, alpha=3.0, beta=0.0, seed=6, c_fill="nan")
    assert np.array_equal(run_oracle(p), np.zeros(20, dtype=np.float32))


def test_bf16_widening_of_known_bit_patterns():
    # 0x3FC0 = 1.5, 0xC000 = -2.0, 0x3B80 = 2^-8, 0x4049 = 3.140625
    A = np.array([0x3FC0, 0xC000, 0x3B80, 0x4049], dtype=np.uint16)
    B = np.array([0x3F80, 0x3F80, 0x3F80, 0x3F80], dtype=np.uint16)
    C = np.zeros(1, dtype=np.float32)
    og.gemm("bf16", 0, 0, 1, 1, 4, 1.0, A, 4, B, 1, 0.0, C, 1)
    assert C[0] == np.float32(1.5 - 2.0 + 2.0 ** -8 + 3.140625)


def test_transpose_and_split_k_invariants():
    p = wl.make_problem("f32", 0, 0, 14, 9, 40, seed=8, c_fill="zeros")
    C = run_oracle(p).reshape(14, 9)
    # (A B)^T = B^T A^T : feed the same buffers as transposed operands, swapped
    Ct = np.zeros(9 * 14, dtype=np.float32)
    og.gemm("f32", 1, 1, 9, 14, 40, 1.0, p.B, p.ldb, p.A, p.lda, 0.0, Ct, 14)
    assert np.array_equal(Ct.reshape(9, 14).T, C)
    # K split in two calls chained through beta = 1 agrees to rounding of the intermediate
    A = p.A.reshape(14, 40)
    B = p.B.reshape(40, 9)
    C1 = np.zeros(14 * 9, dtype=np.float32)
    og.gemm("f32", 0, 0, 14, 9, 25, 1.0, np.ascontiguousarray(A[:, :25]).ravel(), 25,
            np.ascontiguousarray(B[:25]).ravel(), 9, 0.0, C1, 9)
    og.gemm("f32", 0, 0, 14, 9, 15, 1.0, np.ascontiguousarray(A[:, 25:]).ravel(), 15,
            np.ascontiguousarray(B[25:]).ravel(), 9, 1.0, C1, 9)
    np.testing.assert_allclose(C1.reshape(14, 9), C, rtol=0, atol=2e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_entries_equal_full_result(dtype):
    p = wl.make_problem(dtype, 1, 1, 21, 18, 33, batch=3, alpha=-1.5, beta=0.75, seed=12,
                        pad=(2, 1, 3), batch_pad=(3, 3, 3))
    full = run_oracle(p)
    r = np.random.default_rng(0)
    bb, ii, jj = r.integers(0, 3, 50), r.integers(0, 21, 50), r.integers(0, 18, 50)
    got = og.gemm_entries(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B,
                          p.ldb, p.beta, p.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC,
                          bb, ii, jj)
    assert np.array_equal(got, full[bb * p.strideC + ii * p.ldc + jj])


def test_rejects_bad_arguments():
    z = np.zeros(16, dtype=np.float32)
    with pytest.raises(ValueError):
        og.gemm("f32", 2, 0, 2, 2, 2, 1.0, z, 2, z, 2, 0.0, z.copy(), 2)
    with pytest.raises(ValueError):
        og.gemm("f32", 0, 0, 2, 2, 4, 1.0, z, 3, z, 2, 0.0, z.copy(), 2)   # lda < K
    with pytest.raises(ValueError):
        og.gemm("f32", 0, 0, 2, 4, 2, 1.0, z, 2, z, 4, 0.0, z.copy(), 3)   # ldc < N
