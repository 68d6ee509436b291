"""MI355X-native tiled GEMM family with learned kernel selection (arXiv 2003.06795).

The product is libks_gemm.so (hand-written HIP kernels for gfx950 behind a C ABI, declared in
include/ks_gemm.h); this package is its thin Python binding plus the offline tuning drivers.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
