"""Pins for the fp16-operand form of the C GEMM oracle: the binary16 conversion against numpy's for
every bit pattern and against the format's definition at its landmarks, the GEMM against numpy's
fp64 matmul and an interpreter loop."""
import itertools
import math

import numpy as np
import pytest

import workloads as wl
from oracle import gemm as og
from helpers import operand_matrices, c_views


def test_binary16_conversion_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([og.widen_f16(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))      # -0.0 keeps its sign


def test_binary16_landmarks_from_the_format_definition():
    assert og.widen_f16(0x3C00) == 1.0 and og.widen_f16(0xBC00) == -1.0
    assert og.widen_f16(0x0001) == 2.0 ** -24                      # smallest subnormal
    assert og.widen_f16(0x03FF) == 1023 * 2.0 ** -24               # largest subnormal
    assert og.widen_f16(0x0400) == 2.0 ** -14                      # smallest normal
    assert og.widen_f16(0x7BFF) == 65504.0                         # largest finite
    assert og.widen_f16(0x3555) == (1 + 0x155 / 1024) * 2.0 ** -2  # 0.333251953125
    assert math.isinf(og.widen_f16(0x7C00)) and og.widen_f16(0xFC00) < 0
    assert math.isnan(og.widen_f16(0x7E00))


@pytest.mark.parametrize("tA,tB", list(itertools.product((0, 1), (0, 1))))
def test_matches_numpy_fp64_matmul(tA, tB):
    p = wl.make_problem("f16", tA, tB, 33, 27, 45, batch=2, alpha=-0.75, beta=0.5, seed=17,
                        key=tA * 2 + tB, pad=(1, 3, 2), batch_pad=(5, 0, 3))
    bias = wl.uniform_pm1(p.N, 55, 3)
    for use_bias in (False, True):
        C = p.C0.copy()
        if use_bias:
            og.gemm_bias("f16", tA, tB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C, p.ldc,
                         bias, p.batch, p.strideA, p.strideB, p.strideC)
        else:
            og.gemm("f16", tA, tB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C, p.ldc,
                    p.batch, p.strideA, p.strideB, p.strideC)
        As, Bs, Cs = operand_matrices(p)
        for g, A, B, C0 in zip(c_views(p, C), As, Bs, Cs):
            ref = np.float64(np.float32(p.alpha)) * (A @ B) + np.float64(np.float32(p.beta)) * C0.astype(np.float64)
            if use_bias:
                ref = ref + bias.astype(np.float64)[None, :]
            assert np.max(np.abs(g - ref.astype(np.float32))) <= 2.0 ** -23 * np.max(np.abs(ref))


def test_interpreter_loop_bit_equal_and_entries_agree():
    p = wl.make_problem("f16", 1, 0, 5, 6, 9, alpha=1.5, beta=0.0, seed=4)
    C = p.C0.copy()
    og.gemm("f16", 1, 0, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C, p.ldc)
    a = p.A.view(np.float16).astype(np.float64); b = p.B.view(np.float16).astype(np.float64)
    for i in range(p.M):
        for j in range(p.N):
            acc = 0.0
            for k in range(p.K):
                acc += float(a[k * p.lda + i]) * float(b[k * p.ldb + j])
            assert C[i * p.ldc + j] == np.float32(1.5 * acc)
    bb = np.zeros(4, np.int64); ii = np.array([0, 4, 2, 3]); jj = np.array([0, 5, 1, 3])
    e = og.gemm_entries("f16", 1, 0, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, None, p.ldc,
                        1, 0, 0, 0, bb, ii, jj)
    assert np.array_equal(e, C.reshape(p.M, p.ldc)[ii, jj])


def test_small_integers_exact_and_subnormal_products():
    # integers up to 8 are exact in binary16; the sum is an exact integer
    p = wl.make_problem("f16", 0, 1, 7, 5, 31, seed=2, dist="ints")
    C = p.C0.copy()
    og.gemm("f16", 0, 1, p.M, p.N, p.K, 1.0, p.A, p.lda, p.B, p.ldb, 0.0, C, p.ldc)
    As, Bs, _ = operand_matrices(p)
    assert np.array_equal(c_views(p, C)[0], (As[0] @ Bs[0]).astype(np.float32))
    # a subnormal operand: 2^-24 * 2^10 = 2^-14
    A = np.array([0x0001], dtype=np.uint16); B = np.array([0x6400], dtype=np.uint16)   # 2^-24, 1024
    C = np.zeros(1, dtype=np.float32)
    og.gemm("f16", 0, 0, 1, 1, 1, 1.0, A, 1, B, 1, 0.0, C, 1)
    assert C[0] == np.float32(2.0 ** -14)
