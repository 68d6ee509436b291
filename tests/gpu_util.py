"""Helpers for the GPU parity tests: upload a workloads.Problem, run it through the C ABI
(via the thin binding), and bring C back."""
import numpy as np
import torch

import paper_2003_06795_amd.binding as ks
from oracle import gemm as og

DT = {"f32": ks.F32, "bf16": ks.BF16, "f16": ks.F16}
GEMM = {"f32": ks.gemm_f32, "bf16": ks.gemm_bf16, "f16": ks.gemm_f16}
GEMM_K = {"f32": ks.gemm_f32_with_kernel, "bf16": ks.gemm_bf16_with_kernel, "f16": ks.gemm_f16_with_kernel}


GUARD = 64                  # canary floats kept in front of and behind every output buffer
CANARY = -7777.25


class DeviceProblem:
    def __init__(self, p):
        self.p = p
        dev = torch.device("cuda:0")
        a = p.A if p.dtype == "f32" else p.A.view(np.int16)
        b = p.B if p.dtype == "f32" else p.B.view(np.int16)
        # at least one element so data_ptr() is a real allocation even for empty operands
        self.A = torch.from_numpy(np.concatenate([a, a[:0]]) if a.size else np.zeros(1, a.dtype)).to(dev)
        self.B = torch.from_numpy(b if b.size else np.zeros(1, b.dtype)).to(dev)
        self.C0 = torch.from_numpy(p.C0 if p.C0.size else np.zeros(1, np.float32)).to(dev)

    def run(self, kernel_id=None, C=None):
        """Returns the flat C buffer after the call as numpy (same length as p.C0).  The output the
        library sees sits between two runs of canary values, which must come back untouched."""
        p = self.p
        guarded = None
        if C is None:
            n = self.C0.numel()
            guarded = torch.full((n + 2 * GUARD,), CANARY, dtype=torch.float32, device=self.C0.device)
            guarded[GUARD:GUARD + n] = self.C0
            C = guarded[GUARD:GUARD + n]
        args = (p.transA, p.transB, p.M, p.N, p.K, p.alpha, self.A, p.lda, self.B, p.ldb, p.beta, C,
                p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
        if kernel_id is None:
            GEMM[p.dtype](*args)
        else:
            GEMM_K[p.dtype](kernel_id, *args)
        torch.cuda.synchronize()
        if guarded is not None:
            edges = torch.cat([guarded[:GUARD], guarded[GUARD + self.C0.numel():]])
            assert bool((edges == CANARY).all()), "kernel %s wrote outside the output buffer" % (kernel_id,)
        return C.cpu().numpy()[:p.C0.size]


def oracle_full(p):
    C = p.C0.copy()
    og.gemm(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb, p.beta, C,
            p.ldc, p.batch, p.strideA, p.strideB, p.strideC)
    return C


def oracle_entries(p, bb, ii, jj):
    return og.gemm_entries(p.dtype, p.transA, p.transB, p.M, p.N, p.K, p.alpha, p.A, p.lda, p.B, p.ldb,
                           p.beta, p.C0, p.ldc, p.batch, p.strideA, p.strideB, p.strideC, bb, ii, jj)


def sample_entries(p, n, seed, tile=256):
    """Seeded (b, i, j) sample that always holds the four corners and one entry of every edge tile."""
    r = np.random.default_rng(seed)
    bb = r.integers(0, p.batch, n)
    ii = r.integers(0, p.M, n)
    jj = r.integers(0, p.N, n)
    extra = [(0, 0, 0), (p.batch - 1, p.M - 1, p.N - 1), (0, 0, p.N - 1), (0, p.M - 1, 0)]
    for t in range(0, p.M, tile):
        extra.append((0, min(t + int(r.integers(0, tile)), p.M - 1), p.N - 1))
    for t in range(0, p.N, tile):
        extra.append((p.batch - 1, p.M - 1, min(t + int(r.integers(0, tile)), p.N - 1)))
    e = np.array(extra, dtype=np.int64)
    return (np.concatenate([bb, e[:, 0]]), np.concatenate([ii, e[:, 1]]), np.concatenate([jj, e[:, 2]]))


def ensure_workspace(nbytes, _cache={}):
    """One growing torch buffer registered as the split-K workspace."""
    buf = _cache.get("buf")
    if buf is None or buf.numel() * 4 < nbytes:
        buf = torch.empty(max(nbytes // 4 + 1, 1 << 20), dtype=torch.float32, device="cuda:0")
        _cache["buf"] = buf
        ks.set_workspace(buf)
    return buf
