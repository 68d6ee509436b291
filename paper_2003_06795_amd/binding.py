"""ctypes binding of libks_gemm.so: argument marshalling only, same names as the C ABI
(include/ks_gemm.h without the ks_ prefix).  Every compute step runs inside the library's HIP
kernels; if the library has not been built this module raises on first use.

Device operands may be torch tensors (their data_ptr() is passed) or integer device addresses.
Host arrays are numpy.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# KS_GEMM_LIBRARY=libks_gemm_kept.so loads the pruned build (kept members only) instead
LIB_PATH = os.path.join(_HERE, os.environ.get("KS_GEMM_LIBRARY", "libks_gemm.so"))

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_LAUNCH, ERR_WORKSPACE = 0, -1, -2, -3, -4
F32, BF16, F16 = 0, 1, 2
CORE_NAMES = {0: "fma", 1: "mfma16", 2: "mfma32", 3: "direct", 4: "kslice"}
NUM_RAW_FEATURES, NUM_FEATURES, MAX_TREE_NODES = 6, 10, 4096
FEATURE_NAMES = ["M", "N", "K", "batch", "transA", "transB", "M*N", "M*N*K", "min(M,N)", "max(M,N)"]


class KernelInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("id", "dtype", "core", "bm", "bn", "bk", "wm", "wn", "tm", "tn", "threads",
                 "split_k", "lds_bytes", "k_waves", "band_rows", "available", "balanced_per_cu")]

    def as_dict(self):
        d = {n: int(getattr(self, n)) for n, _ in self._fields_}
        d["core_name"] = CORE_NAMES[d["core"]]
        return d


class LaunchPlan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("kernel_id", "split_k", "path", "vector_loads", "grid_3d", "tiles_per_workgroup")] + \
               [("workgroups", ctypes.c_int64), ("balanced_groups", ctypes.c_int32), ("divided_tiles", ctypes.c_int32),
                ("tail_split", ctypes.c_int32), ("k_remainder", ctypes.c_int32)]


class TreeNode(ctypes.Structure):
    _fields_ = [("feature", ctypes.c_int32), ("left", ctypes.c_int32), ("right", ctypes.c_int32),
                ("value", ctypes.c_int32), ("threshold", ctypes.c_int64)]


TREE_DTYPE = np.dtype([("feature", "<i4"), ("left", "<i4"), ("right", "<i4"), ("value", "<i4"),
                       ("threshold", "<i8")], align=True)
assert TREE_DTYPE.itemsize == ctypes.sizeof(TreeNode)


class KsError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, status_string(status), status))


_lib = None
_i, _i64, _f, _p = ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
_GEMM = [_i, _i, _i64, _i64, _i64, _f, _p, _i64, _p, _i64, _f, _p, _i64, _i64, _i64, _i64, _i64, _p]

EXPORTS = [
    "ks_gemm_f32", "ks_gemm_bf16", "ks_gemm_f32_with_kernel", "ks_gemm_bf16_with_kernel",
    "ks_gemm_f16", "ks_gemm_f16_with_kernel", "ks_gemm_bias", "ks_gemm_out_bf16", "ks_gemm_static_scratch", "ks_gemm_with_workspace", "ks_gemm_plan", "ks_time_gemm", "ks_calibration_copy", "ks_mfma_sustained", "ks_bf16_ablation", "ks_num_kernels", "ks_kernel_info", "ks_select", "ks_features",
    "ks_set_selector", "ks_get_selector", "ks_set_fast_path", "ks_set_tiles_per_workgroup", "ks_set_balanced_groups", "ks_set_tail_split", "ks_set_split_partitions", "ks_set_workspace", "ks_workspace_bytes_needed",
    "ks_tune_performance", "ks_tune_normalise", "ks_tune_prune_tree", "ks_tune_achievable", "ks_tune_fit_selector",
    "ks_tune_predict", "ks_tune_selector_score", "ks_tune_prune_top_n", "ks_tune_prune_kmeans", "ks_tune_prune_hdbscan",
    "ks_tune_pca_variance", "ks_status_string",
]


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libks_gemm.so is not built: run `python -m paper_2003_06795_amd.build` "
                           "(there is no fallback path)")
    # PyTorch owns device memory and streams here, so its HIP runtime must be the one this process
    # uses: load it before the library (whichever copy of the runtime is loaded first serves both).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    L.ks_gemm_f32.argtypes = _GEMM
    L.ks_gemm_bf16.argtypes = _GEMM
    L.ks_gemm_f16.argtypes = _GEMM
    L.ks_gemm_f16_with_kernel.argtypes = [_i] + _GEMM
    L.ks_gemm_f32_with_kernel.argtypes = [_i] + _GEMM
    L.ks_gemm_bf16_with_kernel.argtypes = [_i] + _GEMM
    L.ks_gemm_bias.argtypes = [_i, _i] + _GEMM[:13] + [_p] + _GEMM[13:]
    L.ks_gemm_out_bf16.argtypes = [_i, _i] + _GEMM[:13] + [_p] + _GEMM[13:]
    L.ks_gemm_static_scratch.argtypes = [_i, _i] + _GEMM
    L.ks_gemm_with_workspace.argtypes = [_i, _i] + _GEMM[:-1] + [_p, ctypes.c_size_t, _p]
    L.ks_gemm_plan.argtypes = [_i, _i] + _GEMM[:-1] + [ctypes.POINTER(LaunchPlan)]
    L.ks_time_gemm.argtypes = [_i, _i] + _GEMM + [_i, _i, _i, _p]
    L.ks_num_kernels.argtypes = [_i]
    L.ks_kernel_info.argtypes = [_i, _i, ctypes.POINTER(KernelInfo)]
    L.ks_select.argtypes = [_i, _i64, _i64, _i64, _i64, _i, _i]
    L.ks_features.argtypes = [_i64, _i64, _i64, _i64, _i, _i, _p]
    L.ks_set_selector.argtypes = [_i, _p, _i]
    L.ks_get_selector.argtypes = [_i, _p, _i]
    L.ks_calibration_copy.argtypes = [_p, _p, ctypes.c_size_t, _p]
    L.ks_mfma_sustained.argtypes = [_i, _i, _p, ctypes.c_size_t, _i, _p, _p, _p]
    L.ks_bf16_ablation.argtypes = [_i, _p, _p, _p, _i64, _i64, _i64, _p, _i, _p, _p]
    L.ks_set_fast_path.argtypes = [_i]
    L.ks_set_tiles_per_workgroup.argtypes = [_i]
    L.ks_set_balanced_groups.argtypes = [_i]
    L.ks_set_tail_split.argtypes = [_i]
    L.ks_set_split_partitions.argtypes = [_i]
    L.ks_set_workspace.argtypes = [_p, ctypes.c_size_t]
    L.ks_workspace_bytes_needed.argtypes = [_i, _i, _i64, _i64, _i64]
    L.ks_workspace_bytes_needed.restype = ctypes.c_size_t
    L.ks_tune_performance.argtypes = [_p, _p, _i, _i, _p]
    L.ks_tune_normalise.argtypes = [_p, _i, _i, _p]
    L.ks_tune_prune_tree.argtypes = [_p, _i, _p, _i, _i, _i, _i, _p, _p, _p]
    L.ks_tune_achievable.argtypes = [_p, _i, _i, _p, _i, _p]
    L.ks_tune_fit_selector.argtypes = [_p, _i, _p, _i, _i, _p, _i, _i, _i, _p, _p, _i]
    L.ks_tune_predict.argtypes = [_p, _i, _p, _i, _i, _p]
    L.ks_tune_selector_score.argtypes = [_p, _i, _i, _p, _p]
    L.ks_tune_prune_top_n.argtypes = [_p, _i, _i, _i, _p]
    L.ks_tune_prune_kmeans.argtypes = [_p, _i, _i, _i, _i, _i, _p]
    L.ks_tune_prune_hdbscan.argtypes = [_p, _i, _i, _i, _i, _p, _i, _p]
    L.ks_tune_pca_variance.argtypes = [_p, _i, _i, _p]
    L.ks_status_string.argtypes = [_i]
    L.ks_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


def status_string(status):
    return lib().ks_status_string(int(status)).decode()


def _check(rc, what):
    if rc != OK:
        raise KsError(rc, what)


def _dev(x):
    """Device address of a torch tensor, or the integer itself."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return getattr(stream, "cuda_stream", stream)


def _np(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(_p)


# ------------------------------------------------------------------------------ GEMM

def _gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch, strideA,
               strideB, strideC, stream):
    return (int(transA), int(transB), M, N, K, alpha, _dev(A), lda, _dev(B), ldb, beta, _dev(C), ldc,
            batch, strideA, strideB, strideC, _stream(stream))


def gemm_f32(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch=1, strideA=0,
             strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_f32(*_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                         batch, strideA, strideB, strideC, stream)), "ks_gemm_f32")


def gemm_bf16(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch=1, strideA=0,
              strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_bf16(*_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                          batch, strideA, strideB, strideC, stream)), "ks_gemm_bf16")


def gemm_f16(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch=1, strideA=0,
             strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_f16(*_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                         batch, strideA, strideB, strideC, stream)), "ks_gemm_f16")


def gemm_f16_with_kernel(kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                         batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_f16_with_kernel(
        int(kernel_id), *_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                    batch, strideA, strideB, strideC, stream)), "ks_gemm_f16_with_kernel")


def gemm_f32_with_kernel(kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                         batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_f32_with_kernel(
        int(kernel_id), *_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                    batch, strideA, strideB, strideC, stream)), "ks_gemm_f32_with_kernel")


def gemm_bf16_with_kernel(kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                          batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    _check(lib().ks_gemm_bf16_with_kernel(
        int(kernel_id), *_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                    batch, strideA, strideB, strideC, stream)), "ks_gemm_bf16_with_kernel")


def gemm_bias(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, bias,
              batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    """C = alpha*op(A)*op(B) + beta*C + bias[j] per column; kernel_id < 0 lets the deployed tree choose."""
    a = _gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch, strideA,
                   strideB, strideC, stream)
    _check(lib().ks_gemm_bias(int(dtype), int(kernel_id), *a[:13], _dev(bias) if bias is not None else None,
                              *a[13:]), "ks_gemm_bias")


def gemm_out_bf16(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C16, ldc,
                  bias=None, batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    """C16 (bf16 bit patterns) = bf16(alpha*op(A)*op(B) + beta*C16 + bias[j]); kernel_id < 0 selects."""
    a = _gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C16, ldc, batch, strideA,
                   strideB, strideC, stream)
    _check(lib().ks_gemm_out_bf16(int(dtype), int(kernel_id), *a[:13],
                                  _dev(bias) if bias is not None else None, *a[13:]), "ks_gemm_out_bf16")


def gemm_static_scratch(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                        batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    """GEMM whose split-K scratch is the library's static device array; allocates nothing."""
    _check(lib().ks_gemm_static_scratch(
        int(dtype), int(kernel_id), *_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                                                batch, strideA, strideB, strideC, stream)), "ks_gemm_static_scratch")


def gemm_with_workspace(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
                        workspace, batch=1, strideA=0, strideB=0, strideC=0, stream=None):
    """GEMM whose scratch (split-K partial sums, divided tiles) is `workspace` (torch tensor or None),
    not the registered one."""
    a = _gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch, strideA, strideB,
                   strideC, stream)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().ks_gemm_with_workspace(int(dtype), int(kernel_id), *a[:-1],
                                        _dev(workspace) if workspace is not None else None, nbytes, a[-1]),
           "ks_gemm_with_workspace")


def gemm_plan(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
              batch=1, strideA=0, strideB=0, strideC=0):
    """What the call would launch (dict of ks_launch_plan_t), without launching."""
    out = LaunchPlan()
    a = _gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, batch, strideA, strideB,
                   strideC, 0)
    _check(lib().ks_gemm_plan(int(dtype), int(kernel_id), *a[:-1], ctypes.byref(out)), "ks_gemm_plan")
    return {n: int(getattr(out, n)) for n, _ in LaunchPlan._fields_}


def time_gemm(dtype, kernel_id, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc,
              batch=1, strideA=0, strideB=0, strideC=0, stream=None, warmup=3, iters=10, reps=1):
    """Per-launch milliseconds of `iters` samples (numpy float32)."""
    out = np.zeros(iters, dtype=np.float32)
    _check(lib().ks_time_gemm(
        int(dtype), int(kernel_id), *_gemm_args(transA, transB, M, N, K, alpha, A, lda, B, ldb, beta,
                                                C, ldc, batch, strideA, strideB, strideC, stream),
        int(warmup), int(iters), int(reps), out.ctypes.data_as(_p)), "ks_time_gemm")
    return out


# ------------------------------------------------------------------------------ registry / selection

def num_kernels(dtype):
    n = lib().ks_num_kernels(int(dtype))
    if n < 0:
        raise KsError(n, "ks_num_kernels")
    return n


def kernel_info(dtype, kernel_id):
    ki = KernelInfo()
    _check(lib().ks_kernel_info(int(dtype), int(kernel_id), ctypes.byref(ki)), "ks_kernel_info")
    return ki.as_dict()


def select(dtype, M, N, K, batch=1, transA=0, transB=0):
    rc = lib().ks_select(int(dtype), M, N, K, batch, int(transA), int(transB))
    if rc < 0:
        raise KsError(rc, "ks_select")
    return rc


def features(M, N, K, batch=1, transA=0, transB=0):
    out = np.zeros(NUM_FEATURES, dtype=np.int64)
    _check(lib().ks_features(M, N, K, batch, int(transA), int(transB), out.ctypes.data_as(_p)),
           "ks_features")
    return out


def set_selector(dtype, nodes):
    """nodes: numpy structured array of TREE_DTYPE (or None / empty to restore the built-in tree)."""
    if nodes is None or len(nodes) == 0:
        _check(lib().ks_set_selector(int(dtype), None, 0), "ks_set_selector")
        return
    a, p = _np(nodes, TREE_DTYPE)
    _check(lib().ks_set_selector(int(dtype), p, len(a)), "ks_set_selector")


def get_selector(dtype):
    a = np.zeros(MAX_TREE_NODES, dtype=TREE_DTYPE)
    n = lib().ks_get_selector(int(dtype), a.ctypes.data_as(_p), MAX_TREE_NODES)
    if n < 0:
        raise KsError(n, "ks_get_selector")
    return a[:n].copy()


def calibration_copy(dst, src, nbytes, stream=None):
    _check(lib().ks_calibration_copy(_dev(dst), _dev(src), int(nbytes), _stream(stream)), "ks_calibration_copy")


MFMA_PROBE_BYTES = 64 * 8 * 12 * 1024


def mfma_sustained(dtype, operands, nbytes=None, rounds=2000, stream=None, fragment=32):
    """(TFLOP/s, shader MHz) of a pure MFMA loop on the values in `operands` (device buffer);
    fragment 32: 32x32 MFMAs, 16 (16-bit types only): 16x16x32."""
    if nbytes is None:
        nbytes = operands.numel() * operands.element_size()
    tf, mhz = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().ks_mfma_sustained(int(dtype), int(fragment), _dev(operands), int(nbytes), int(rounds), _stream(stream),
                                   ctypes.byref(tf), ctypes.byref(mhz)), "ks_mfma_sustained")
    return tf.value, mhz.value


def bf16_ablation(mode, A, B, C, M, N, K, iters=10, stream=None):
    """Milliseconds of `iters` launches of the two-group bf16 kernel with data paths left out (mode 0-3);
    mode 4 is the whole kernel and returns (milliseconds, shader MHz during the last launch)."""
    out = np.zeros(iters, dtype=np.float32)
    mhz = ctypes.c_double(0.0)
    _check(lib().ks_bf16_ablation(int(mode), _dev(A), _dev(B), _dev(C), M, N, K, _stream(stream), int(iters),
                                  out.ctypes.data_as(_p), ctypes.byref(mhz)), "ks_bf16_ablation")
    return (out, float(mhz.value)) if int(mode) >= 4 else out


def set_fast_path(enabled):
    _check(lib().ks_set_fast_path(int(bool(enabled))), "ks_set_fast_path")


def set_tiles_per_workgroup(n):
    """0: chosen per call; 1..64: forced (large-tile fp32 MFMA members, 1-D launches without split-K)."""
    _check(lib().ks_set_tiles_per_workgroup(int(n)), "ks_set_tiles_per_workgroup")


def set_balanced_groups(per_cu):
    """0: each member's own count; 1..8: forced work-groups per compute unit of the balanced persistent form."""
    _check(lib().ks_set_balanced_groups(int(per_cu)), "ks_set_balanced_groups")


def set_tail_split(partitions):
    """-1: hybrid launches of the 16-bit per-call-split members chosen per call; 0: never; 2..16: forced."""
    _check(lib().ks_set_tail_split(int(partitions)), "ks_set_tail_split")


def set_split_partitions(partitions):
    """0: per-call split members take the library's estimate; 1..256: forced K partitions (1 = no split)."""
    _check(lib().ks_set_split_partitions(int(partitions)), "ks_set_split_partitions")


def set_workspace(buf, nbytes=None):
    """buf: torch tensor (kept alive by the caller), integer address, or None."""
    if buf is None:
        _check(lib().ks_set_workspace(None, 0), "ks_set_workspace")
        return
    if nbytes is None:
        nbytes = buf.numel() * buf.element_size()
    _check(lib().ks_set_workspace(_dev(buf), nbytes), "ks_set_workspace")


def workspace_bytes_needed(dtype, kernel_id, M, N, batch=1):
    return int(lib().ks_workspace_bytes_needed(int(dtype), int(kernel_id), M, N, batch))


# ------------------------------------------------------------------------------ offline tuner (host)

def tune_performance(sizes, seconds):
    """flop/s table from (M, N, K, batch) rows and the measured seconds [rows x kernels]."""
    z, zp = _np(sizes, np.int64)
    t, tp = _np(seconds, np.float64)
    out = np.empty_like(t)
    _check(lib().ks_tune_performance(zp, tp, t.shape[0], t.shape[1], out.ctypes.data_as(_p)), "ks_tune_performance")
    return out


def tune_normalise(perf):
    a, p = _np(perf, np.float64)
    out = np.empty_like(a)
    _check(lib().ks_tune_normalise(p, a.shape[0], a.shape[1], out.ctypes.data_as(_p)), "ks_tune_normalise")
    return out


def tune_prune_tree(features_, normalised, max_leaves, min_samples_leaf=1):
    """Returns (kept ids, regression tree as TREE_DTYPE array)."""
    X, xp = _np(features_, np.int64)
    Y, yp = _np(normalised, np.float64)
    kept = np.zeros(max_leaves, dtype=np.int32)
    tree = np.zeros(2 * max_leaves - 1, dtype=TREE_DTYPE)
    n_nodes = ctypes.c_int(0)
    n = lib().ks_tune_prune_tree(xp, X.shape[1], yp, Y.shape[0], Y.shape[1], int(max_leaves),
                                 int(min_samples_leaf), kept.ctypes.data_as(_p),
                                 tree.ctypes.data_as(_p), ctypes.byref(n_nodes))
    if n < 0:
        raise KsError(n, "ks_tune_prune_tree")
    return kept[:n].copy(), tree[:n_nodes.value].copy()


def tune_achievable(normalised, kept):
    Y, yp = _np(normalised, np.float64)
    k, kp = _np(kept, np.int32)
    out = ctypes.c_double(0)
    _check(lib().ks_tune_achievable(yp, Y.shape[0], Y.shape[1], kp, len(k), ctypes.byref(out)),
           "ks_tune_achievable")
    return out.value


def tune_fit_selector(features_, perf, kept, max_depth=12, min_samples_leaf=1, row_weight=None):
    X, xp = _np(features_, np.int64)
    P, pp = _np(perf, np.float64)
    k, kp = _np(kept, np.int32)
    w = wp = None
    if row_weight is not None:
        w, wp = _np(row_weight, np.float64)
    tree = np.zeros(MAX_TREE_NODES, dtype=TREE_DTYPE)
    n = lib().ks_tune_fit_selector(xp, X.shape[1], pp, P.shape[0], P.shape[1], kp, len(k),
                                   int(max_depth), int(min_samples_leaf), wp,
                                   tree.ctypes.data_as(_p), MAX_TREE_NODES)
    if n < 0:
        raise KsError(n, "ks_tune_fit_selector")
    return tree[:n].copy()


def tune_predict(tree, features_):
    t, tp = _np(tree, TREE_DTYPE)
    X, xp = _np(features_, np.int64)
    out = np.zeros(X.shape[0], dtype=np.int32)
    _check(lib().ks_tune_predict(tp, len(t), xp, X.shape[1], X.shape[0], out.ctypes.data_as(_p)),
           "ks_tune_predict")
    return out


def tune_selector_score(normalised, chosen):
    Y, yp = _np(normalised, np.float64)
    c, cp = _np(chosen, np.int32)
    out = ctypes.c_double(0)
    _check(lib().ks_tune_selector_score(yp, Y.shape[0], Y.shape[1], cp, ctypes.byref(out)),
           "ks_tune_selector_score")
    return out.value


def tune_prune_top_n(normalised, n):
    Y, yp = _np(normalised, np.float64)
    kept = np.zeros(n, dtype=np.int32)
    m = lib().ks_tune_prune_top_n(yp, Y.shape[0], Y.shape[1], int(n), kept.ctypes.data_as(_p))
    if m < 0:
        raise KsError(m, "ks_tune_prune_top_n")
    return kept[:m].copy()


def tune_prune_kmeans(normalised, n, pca_dims=0, max_iter=100):
    Y, yp = _np(normalised, np.float64)
    kept = np.zeros(n, dtype=np.int32)
    m = lib().ks_tune_prune_kmeans(yp, Y.shape[0], Y.shape[1], int(n), int(pca_dims), int(max_iter),
                                   kept.ctypes.data_as(_p))
    if m < 0:
        raise KsError(m, "ks_tune_prune_kmeans")
    return kept[:m].copy()


def tune_prune_hdbscan(normalised, min_cluster_size, min_samples=None):
    """Returns (kept ids, cluster label of every row; -1 = noise)."""
    Y, yp = _np(normalised, np.float64)
    kept = np.zeros(Y.shape[1], dtype=np.int32)
    labels = np.zeros(Y.shape[0], dtype=np.int32)
    m = lib().ks_tune_prune_hdbscan(yp, Y.shape[0], Y.shape[1], int(min_cluster_size),
                                    int(min_samples if min_samples is not None else min_cluster_size),
                                    kept.ctypes.data_as(_p), len(kept), labels.ctypes.data_as(_p))
    if m < 0:
        raise KsError(m, "ks_tune_prune_hdbscan")
    return kept[:m].copy(), labels


def tune_pca_variance(normalised):
    Y, yp = _np(normalised, np.float64)
    out = np.zeros(Y.shape[1], dtype=np.float64)
    _check(lib().ks_tune_pca_variance(yp, Y.shape[0], Y.shape[1], out.ctypes.data_as(_p)), "ks_tune_pca_variance")
    return out
