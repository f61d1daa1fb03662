"""Ternary linear layer for MI355X: y = gamma * (x @ What^T) with packed ternary weights.

The work is done by hand-written gfx950 kernels in libtl.so (see include/tl.h);
this package is the thin binding above that C ABI.
"""
from .binding import *  # noqa: F401,F403
from .binding import TlError, EXPORTS, LIB_PATH, raw, tl_gemm_job, make_jobs  # noqa: F401
