"""numpy-facing wrapper of the C GEMM oracle (oracle/gemm_oracle.c).

TEST INFRASTRUCTURE ONLY.  The definition implemented is the general matrix
multiply of the paper's Section II, C = alpha*op(A)*op(B) + beta*C, batched with
element strides, row-major, fp64 accumulation in increasing k.

All arrays are flat or shaped numpy buffers; the caller states the logical
problem (M, N, K, leading dimensions, strides) exactly as the C ABI of the
product does, so the two can be driven from the same argument tuple.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None

_i64 = ctypes.c_int64
_f32 = ctypes.c_float
_ptr = ctypes.c_void_p


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        head = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _f32, _ptr, _i64, _ptr, _i64,
                _f32, _ptr, _i64, _i64, _i64, _i64, _i64]
        for name in ("oracle_gemm_f32", "oracle_gemm_bf16"):
            f = getattr(L, name)
            f.argtypes = head
            f.restype = ctypes.c_int
        for name in ("oracle_gemm_bias_f32", "oracle_gemm_bias_bf16", "oracle_gemm_bias_f16"):
            f = getattr(L, name)
            f.argtypes = head + [_ptr]
            f.restype = ctypes.c_int
        L.oracle_round_to_bf16.argtypes = [ctypes.c_double]
        L.oracle_round_to_bf16.restype = ctypes.c_uint16
        L.oracle_gemm_out_bf16.argtypes = [ctypes.c_int] + head + [_ptr]
        L.oracle_gemm_out_bf16.restype = ctypes.c_int
        L.oracle_widen_f16.argtypes = [ctypes.c_uint16]
        L.oracle_widen_f16.restype = ctypes.c_double
        for name in ("oracle_gemm_f32_entries", "oracle_gemm_bf16_entries", "oracle_gemm_f16_entries"):
            f = getattr(L, name)
            f.argtypes = head + [_i64, _ptr, _ptr, _ptr, _ptr]
            f.restype = ctypes.c_int
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))


def _p(a):
    return None if a is None else a.ctypes.data_as(_ptr)


def _check_in(a, dtype):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("oracle operands must be C-contiguous %s buffers" % np.dtype(dtype).name)


def gemm(dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
         batch=1, strideA=0, strideB=0, strideC=0):
    """In-place on C (float32 numpy buffer).  dtype is 'f32', 'bf16' or 'f16' (A, B uint16 bits)."""
    in_t = np.float32 if dtype == "f32" else np.uint16
    _check_in(A, in_t)
    _check_in(B, in_t)
    _check_in(C, np.float32)
    if dtype == "f16":
        return gemm_bias(dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, None,
                         batch, strideA, strideB, strideC)
    fn = lib().oracle_gemm_f32 if dtype == "f32" else lib().oracle_gemm_bf16
    rc = fn(int(transA), int(transB), M, N, K, alpha, _p(A), lda, _p(B), ldb, beta, _p(C), ldc,
            batch, strideA, strideB, strideC)
    if rc != 0:
        raise ValueError("oracle gemm: invalid arguments")
    return C


def gemm_bias(dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, bias,
              batch=1, strideA=0, strideB=0, strideC=0):
    """gemm() with a length-N fp32 vector added to every row: alpha*op(A)*op(B) + beta*C + bias[j]
    (fully-connected layer, Section II-A), summed in fp64 and rounded once.  In place on C."""
    in_t = np.float32 if dtype == "f32" else np.uint16
    _check_in(A, in_t)
    _check_in(B, in_t)
    _check_in(C, np.float32)
    if bias is not None:
        _check_in(bias, np.float32)
        if bias.size < N:
            raise ValueError("bias shorter than N")
    fn = {"f32": lib().oracle_gemm_bias_f32, "bf16": lib().oracle_gemm_bias_bf16,
          "f16": lib().oracle_gemm_bias_f16}[dtype]
    rc = fn(int(transA), int(transB), M, N, K, alpha, _p(A), lda, _p(B), ldb, beta, _p(C), ldc,
            batch, strideA, strideB, strideC, _p(bias))
    if rc != 0:
        raise ValueError("oracle gemm_bias: invalid arguments")
    return C


def gemm_entries(dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C0, ldc,
                 batch, strideA, strideB, strideC, bb, ii, jj):
    """Values of the listed output entries (b, i, j) by the same definition."""
    in_t = np.float32 if dtype == "f32" else np.uint16
    _check_in(A, in_t)
    _check_in(B, in_t)
    if C0 is not None:
        _check_in(C0, np.float32)
    bb = np.ascontiguousarray(bb, dtype=np.int64)
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    out = np.empty(bb.shape[0], dtype=np.float32)
    fn = {"f32": lib().oracle_gemm_f32_entries, "bf16": lib().oracle_gemm_bf16_entries,
          "f16": lib().oracle_gemm_f16_entries}[dtype]
    rc = fn(int(transA), int(transB), M, N, K, alpha, _p(A), lda, _p(B), ldb, beta, _p(C0), ldc,
            batch, strideA, strideB, strideC, bb.shape[0], _p(bb), _p(ii), _p(jj), _p(out))
    if rc != 0:
        raise ValueError("oracle gemm_entries: invalid arguments")
    return out


def widen_f16(bits):
    """The oracle's own binary16 -> float64 conversion of one bit pattern."""
    return lib().oracle_widen_f16(int(bits))


def round_to_bf16(x):
    """The oracle's own float64 -> bf16 (bit pattern) rounding of one value."""
    return lib().oracle_round_to_bf16(float(x))


def gemm_out_bf16(dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C16, ldc, bias=None,
                  batch=1, strideA=0, strideB=0, strideC=0):
    """C kept in bf16 (uint16 bit patterns, in place): bf16(alpha*op(A)*op(B) + beta*C + bias[j]),
    the sum formed in fp64 and rounded once to nearest even."""
    in_t = np.float32 if dtype == "f32" else np.uint16
    _check_in(A, in_t)
    _check_in(B, in_t)
    _check_in(C16, np.uint16)
    if bias is not None:
        _check_in(bias, np.float32)
        if bias.size < N:
            raise ValueError("bias shorter than N")
    rc = lib().oracle_gemm_out_bf16({"f32": 0, "bf16": 1, "f16": 2}[dtype], int(transA), int(transB), M, N, K,
                                    alpha, _p(A), lda, _p(B), ldb, beta, _p(C16), ldc, batch, strideA,
                                    strideB, strideC, _p(bias))
    if rc != 0:
        raise ValueError("oracle gemm_out_bf16: invalid arguments")
    return C16
