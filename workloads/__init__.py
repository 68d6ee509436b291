"""Seeded synthetic workloads: shape sets and input tensors.

This module holds no arithmetic of the method (no GEMM, no tree, no scoring):
only the shape lists of the five benchmark configurations and the seeded
generators of their operand values.  Both the GPU tests/benchmark and the CPU
oracle draw their inputs from here so that they see identical bits.

The shape sets stand in for the GEMM sizes the paper extracted from VGG, ResNet
and MobileNet (Section II-A), which are not available: config 2 is a log-uniform
sweep, config 3 enumerates im2col-style convolution shapes, config 4 is batched
small GEMMs, config 5 is large/skinny bf16 GEMMs.
"""
from dataclasses import dataclass, field
import itertools

import numpy as np

__all__ = [
    "Problem", "make_problem", "uniform_pm1", "normal_scaled", "f32_to_bf16_rne",
    "bf16_to_f32", "f32_to_f16_bits", "f16_bits_to_f32", "operand_as_f32", "config1_problem", "CONFIG1_TILES", "config2_shapes", "config2_split",
    "config2_rows", "config2_extra_rows", "config3_shapes", "config4_shapes", "config4_extra_rows", "config5_shapes", "bf16_tuning_shapes",
    "bf16_tuning_split",
]


# --------------------------------------------------------------------------- values

def _rng(seed, *key):
    return np.random.default_rng([int(seed)] + [int(k) for k in key])


def uniform_pm1(n, seed, *key):
    """n i.i.d. float32 values uniform in [-1, 1)."""
    r = _rng(seed, *key)
    x = r.random(int(n), dtype=np.float32)
    x *= 2.0
    x -= 1.0
    return x


def normal_scaled(n, scale, seed, *key):
    """n i.i.d. float32 normal(0, 1) values multiplied by `scale`."""
    r = _rng(seed, *key)
    x = r.standard_normal(int(n), dtype=np.float32)
    x *= np.float32(scale)
    return x


def f32_to_bf16_rne(x):
    """Round float32 to bfloat16 bit patterns (uint16), round-to-nearest-even.

    Inputs are finite in every workload here; NaN handling is not needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_to_f16_bits(x):
    """float32 -> IEEE binary16 bit patterns (uint16), round to nearest even (numpy's conversion)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b):
    """binary16 bit patterns -> float32 (exact)."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def operand_as_f32(dtype, buf):
    """The operand buffer of a Problem as float32 values, whatever its storage type."""
    if dtype == "f32":
        return buf
    return bf16_to_f32(buf) if dtype == "bf16" else f16_bits_to_f32(buf)


def bf16_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- problems

@dataclass
class Problem:
    """One GEMM call, in the argument order of the C ABI, with host buffers."""
    dtype: str                    # 'f32' | 'bf16' | 'f16'
    transA: int
    transB: int
    M: int
    N: int
    K: int
    alpha: float
    A: np.ndarray                 # flat; float32 or uint16 (bf16 bits)
    lda: int
    B: np.ndarray
    ldb: int
    beta: float
    C0: np.ndarray                # flat float32, the output buffer before the call
    ldc: int
    batch: int
    strideA: int
    strideB: int
    strideC: int
    meta: dict = field(default_factory=dict)

    @property
    def flops(self):
        return 2.0 * self.M * self.N * self.K * self.batch

    def max_abs(self):
        """(max|A|, max|B|, max|C0|) over the logical entries' buffers, as float."""
        a = operand_as_f32(self.dtype, self.A)
        b = operand_as_f32(self.dtype, self.B)
        f = lambda v: float(np.max(np.abs(v))) if v.size else 0.0
        c = self.C0[np.isfinite(self.C0)]
        return f(a), f(b), f(c)


def make_problem(dtype, transA, transB, M, N, K, batch=1, alpha=1.0, beta=0.0, seed=0, key=0,
                 pad=(0, 0, 0), batch_pad=(0, 0, 0), broadcast=(False, False),
                 dist="uniform", c_fill="uniform"):
    """Seeded operands for one GEMM.

    pad       extra elements added to each leading dimension (lda, ldb, ldc)
    batch_pad extra elements between consecutive batch items of A, B, C
    broadcast (A, B): use batch stride 0 for that operand
    dist      'uniform' -> U[-1,1); 'normal' -> N(0,1)/sqrt(K); 'ints' -> integers in [-8, 8]
    c_fill    'uniform' | 'nan' | 'zeros': what the output buffer holds before the call
    bf16 operands are produced by rounding the float32 draw once (RNE).
    """
    rowsA, colsA = (K, M) if transA else (M, K)
    rowsB, colsB = (N, K) if transB else (K, N)
    lda, ldb, ldc = max(colsA, 1) + pad[0], max(colsB, 1) + pad[1], max(N, 1) + pad[2]
    sizeA, sizeB, sizeC = rowsA * lda, rowsB * ldb, M * ldc
    strideA = 0 if broadcast[0] else sizeA + batch_pad[0]
    strideB = 0 if broadcast[1] else sizeB + batch_pad[1]
    strideC = sizeC + batch_pad[2]
    nA = sizeA + strideA * max(batch - 1, 0)
    nB = sizeB + strideB * max(batch - 1, 0)
    nC = sizeC + strideC * max(batch - 1, 0)

    def draw(n, t):
        if dist == "uniform":
            return uniform_pm1(n, seed, key, t)
        if dist == "normal":
            return normal_scaled(n, 1.0 / np.sqrt(max(K, 1)), seed, key, t)
        if dist == "ints":
            return _rng(seed, key, t).integers(-8, 9, size=int(n)).astype(np.float32)
        raise ValueError(dist)

    A, B = draw(nA, 0), draw(nB, 1)
    if dtype == "bf16":
        A, B = f32_to_bf16_rne(A), f32_to_bf16_rne(B)
    elif dtype == "f16":
        A, B = f32_to_f16_bits(A), f32_to_f16_bits(B)
    if c_fill == "uniform":
        C0 = uniform_pm1(nC, seed, key, 2)
    elif c_fill == "nan":
        C0 = np.full(nC, np.nan, dtype=np.float32)
    else:
        C0 = np.zeros(nC, dtype=np.float32)
    return Problem(dtype, int(transA), int(transB), M, N, K, float(alpha), A, lda, B, ldb,
                   float(beta), C0, ldc, batch, strideA, strideB, strideC,
                   meta=dict(seed=seed, key=key, dist=dist))


# --------------------------------------------------------------------------- config 1

# (work-group tile rows, cols, register tile rows, cols, K-step)
CONFIG1_TILES = [(32, 32, 2, 2, 8), (32, 32, 4, 4, 8), (64, 64, 2, 2, 8), (64, 64, 4, 4, 8)]


def config1_problem():
    return make_problem("f32", 0, 0, 128, 128, 128, alpha=1.0, beta=0.0, seed=0)


# --------------------------------------------------------------------------- config 2

def config2_shapes(n=200, seed=1, lo=16, hi=4096, multiple=8):
    """n (M, N, K) triples, each dimension log-uniform in [lo, hi], rounded to `multiple`.

    One generator, draw order M, N, K per shape.
    """
    r = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dims = []
        for _d in range(3):
            v = float(np.exp(r.uniform(np.log(lo), np.log(hi))))
            q = int(round(v / multiple)) * multiple
            dims.append(min(max(q, lo), hi))
        out.append(tuple(dims))
    return out


def config2_extra_rows(n=400, seed=11):
    """More rows of the same distribution as config 2 (other seed), used only to train the fp32
    selector on a larger table; never part of a held-out set."""
    rows = []
    for s, (M, N, K) in enumerate(config2_shapes(n, seed)):
        for tA, tB in itertools.product((0, 1), (0, 1)):
            rows.append((s, tA, tB, M, N, K, 1))
    return rows


def large_fp32_rows(n=24, seed=16, lo=2048, hi=8192, cap=2 ** 37):
    """Large fp32 GEMMs, for training the fp32 selector only (the tuning set stops at 4096 and holds
    few shapes that are large in all three dimensions): M, N, K log-uniform in [lo, hi], multiples
    of 64, M*N*K at most `cap`; all four layouts."""
    r = np.random.default_rng(seed)
    rows, s = [], 0
    while s < n:
        M, N, K = (int(round(np.exp(r.uniform(np.log(lo), np.log(hi))) / 64.0)) * 64 for _ in range(3))
        if M * N * K > cap:
            continue
        for tA, tB in itertools.product((0, 1), (0, 1)):
            rows.append((s, tA, tB, M, N, K, 1))
        s += 1
    return rows


def medium_large_fp32_rows():
    """72 more shapes between the top of the tuning set and the large ones (dimensions 1024 .. 8192,
    M*N*K at most 2^36, seed 17): training rows for the pruning step, which otherwise sees too few
    problems of several rounds of large tiles to give them a leaf of their own."""
    return large_fp32_rows(n=72, seed=17, lo=1024, hi=8192, cap=2 ** 36)


def config2_split(n=200, seed=1, train_fraction=0.7):
    """Indices of the train and test shapes (shapes, not rows: the four transpose
    combinations of one shape stay on the same side)."""
    perm = np.random.default_rng([seed, 0x5917]).permutation(n)
    n_train = int(round(train_fraction * n))
    return sorted(int(i) for i in perm[:n_train]), sorted(int(i) for i in perm[n_train:])


def config2_rows(n=200, seed=1):
    """Rows of the tuning table: (shape_index, transA, transB, M, N, K, batch)."""
    rows = []
    for s, (M, N, K) in enumerate(config2_shapes(n, seed)):
        for tA, tB in itertools.product((0, 1), (0, 1)):
            rows.append((s, tA, tB, M, N, K, 1))
    return rows


# --------------------------------------------------------------------------- config 3

def config3_shapes():
    """Distinct im2col GEMM shapes (M, N, K): M = batch*H*W, N = out channels, K = kh*kw*Cin."""
    seen, out = set(), []
    for b, hw, n, ks, cin in itertools.product((1, 8, 32), (7, 14, 28, 56, 112),
                                               (32, 64, 128, 256, 512, 1024, 2048),
                                               (1, 3), (3, 32, 64, 128, 256, 512)):
        t = (b * hw * hw, n, ks * ks * cin)
        if t not in seen:
            seen.add(t)
            out.append(t)
    return out


# --------------------------------------------------------------------------- config 4

def config4_shapes():
    """(M, N, K) in {8,16,32,64}^3, each run as 1024 contiguous strided batch items."""
    return list(itertools.product((8, 16, 32, 64), repeat=3))


CONFIG4_BATCH = 1024
CONFIG4_ALPHA, CONFIG4_BETA = 1.0, 0.5


def config4_extra_rows(n=240, seed=14):
    """More batched small GEMMs for training the fp32 selector only: (M, N, K, batch) with every
    dimension a multiple of 8 in [8, 64] and batch in {256, 512, 1024, 2048, 4096}; triples that
    config 4 contains (all three dimensions powers of two) are left out, so its held-out shapes
    stay unseen."""
    r = np.random.default_rng(seed)
    pow2 = {8, 16, 32, 64}
    seen, out = set(), []
    while len(out) < n:
        M, N, K = (int(v) for v in 8 * r.integers(1, 9, size=3))
        b = int(r.choice([256, 512, 1024, 2048, 4096]))
        if ({M, N, K} <= pow2) or (M, N, K, b) in seen:
            continue
        seen.add((M, N, K, b))
        out.append((M, N, K, b))
    return out


# --------------------------------------------------------------------------- config 5

def config5_shapes():
    """bf16 (M, N, K) cells, each run in NN and NT layouts."""
    sq = [(s, s, s) for s in (2048, 4096, 8192)]
    skinny = [(8192, n, 8192) for n in (16, 64, 256)]
    tall_k = [(256, 256, 65536)]
    return sq + skinny + tall_k


CONFIG5_LAYOUTS = [(0, 0), (0, 1)]


# --------------------------------------------------------------------------- bf16 tuning set

def bf16_tuning_shapes(n=160, seed=5, lo=64, hi=16384, max_mnk=2 ** 39):
    """(M, N, K) triples for tuning the bf16 family: each dimension log-uniform in [lo, hi],
    M and N rounded to multiples of 64 and K to a multiple of 128 (the sizes transformer-style
    layers produce); triples with M*N*K above max_mnk are redrawn.  Each is run as NN and NT."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        dims = []
        for d in range(3):
            mult = 128 if d == 2 else 64
            v = float(np.exp(r.uniform(np.log(lo), np.log(hi))))
            dims.append(min(max(int(round(v / mult)) * mult, mult), hi))
        if dims[0] * dims[1] * dims[2] <= max_mnk:
            out.append(tuple(dims))
    return out


def bf16_tuning_split(n=160, seed=5, train_fraction=0.7):
    perm = np.random.default_rng([seed, 0x5917]).permutation(n)
    n_train = int(round(train_fraction * n))
    return sorted(int(i) for i in perm[:n_train]), sorted(int(i) for i in perm[n_train:])
