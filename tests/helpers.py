"""Test-side helpers: views of a workloads.Problem as numpy matrices, tolerances."""
import numpy as np

import workloads as wl


def operand_matrices(p):
    """Lists (per batch item) of op(A) [M x K], op(B) [K x N] as float64 and C0 [M x N] float32 views."""
    a = wl.operand_as_f32(p.dtype, p.A)
    b = wl.operand_as_f32(p.dtype, p.B)
    As, Bs, Cs = [], [], []
    for t in range(p.batch):
        ra, ca = (p.K, p.M) if p.transA else (p.M, p.K)
        rb, cb = (p.N, p.K) if p.transB else (p.K, p.N)
        Am = a[t * p.strideA: t * p.strideA + ra * p.lda].reshape(ra, p.lda)[:, :ca].astype(np.float64)
        Bm = b[t * p.strideB: t * p.strideB + rb * p.ldb].reshape(rb, p.ldb)[:, :cb].astype(np.float64)
        As.append(Am.T if p.transA else Am)
        Bs.append(Bm.T if p.transB else Bm)
        Cs.append(p.C0[t * p.strideC: t * p.strideC + p.M * p.ldc].reshape(p.M, p.ldc)[:, :p.N])
    return As, Bs, Cs


def c_views(p, Cbuf):
    """Per-batch [M x N] views of a flat output buffer laid out like p.C0."""
    return [Cbuf[t * p.strideC: t * p.strideC + p.M * p.ldc].reshape(p.M, p.ldc)[:, :p.N]
            for t in range(p.batch)]


def c_padding_mask(p):
    """Boolean mask over the flat C buffer: True where no logical entry lives."""
    m = np.ones(p.C0.shape[0], dtype=bool)
    for t in range(p.batch):
        v = m[t * p.strideC: t * p.strideC + p.M * p.ldc].reshape(p.M, p.ldc)
        v[:, :p.N] = False
    return m


def tolerance(p):
    """Largest allowed |C_gpu - C_oracle|.

    fp32:  |alpha| * 1e-5 * K * max|A| * max|B|       + 1e-6 * |beta| * max|C0|
    bf16:  |alpha| * 1e-2 * sqrt(K) * max|A| * max|B| + 1e-6 * |beta| * max|C0|
    (the stated bounds at alpha = 1, beta = 0, extended linearly; plus one fp32
    rounding of the stored value, which matters only when K == 0).
    """
    ma, mb, mc = p.max_abs()
    if p.dtype == "f32":
        t = abs(p.alpha) * 1e-5 * p.K * ma * mb
    else:
        t = abs(p.alpha) * 1e-2 * np.sqrt(p.K) * ma * mb
    t += 1e-6 * abs(p.beta) * mc
    return t + 1.2e-7 * abs(p.beta) * mc
