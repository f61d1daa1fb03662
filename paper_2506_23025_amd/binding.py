"""ctypes binding of libtl.so: same names as include/tl.h, argument marshalling only.

Host entry points take and return numpy arrays.  Device entry points take torch
tensors (or raw integer device addresses) and a stream; torch is used for nothing
but device memory and streams.  There is no CPU fallback: if the shared library
is missing, importing this module raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# TL_LIB_PATH: another build of the same library (the host-sanitizer build, see README)
LIB_PATH = os.environ.get("TL_LIB_PATH") or os.path.join(_HERE, "libtl.so")

TL_OK = 0
TL_ERR_NULL, TL_ERR_SHAPE, TL_ERR_VALUE, TL_ERR_ALIGN, TL_ERR_UNSUPPORTED, TL_ERR_HIP = 1, 2, 3, 4, 5, 6
TL_FMT_2BIT, TL_FMT_1P6BIT, TL_FMT_1P6BIT_FX = 0, 1, 2
TL_PATH_AUTO, TL_PATH_GENERIC, TL_PATH_GEMV, TL_PATH_MFMA = 0, 1, 2, 3

EXPORTS = (
    "tl_status_str", "tl_row_stride_bytes", "tl_packed_bytes", "tl_quantize", "tl_pack_2bit", "tl_pack_1p6bit",
    "tl_pack_1p6bit_fx", "tl_unpack_1p6bit_fx", "tl_unpack", "tl_unpack_dev", "tl_ternary_gemm",
    "tl_ternary_gemm_path", "tl_ternary_gemm_grouped", "tl_ternary_gemm_1p6", "tl_ternary_gemm_1p6_fx",
    "tl_ternary_gemm_gs", "tl_ternary_gemm_1p6_grouped", "tl_ternary_gemm_gs_grouped",
    "tl_ternary_gemm_which",
    "tl_init",
    "tl_probe_copy",
    "tl_probe_read",
    "tl_probe_mfma",
)


class tl_gemm_job(ctypes.Structure):
    """Mirror of struct tl_gemm_job in include/tl.h."""
    _fields_ = [("x", ctypes.c_void_p), ("Wpacked", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("gamma_fp16_bits", ctypes.c_uint16)]


class tl_gemm_gs_job(ctypes.Structure):
    """Mirror of struct tl_gemm_gs_job in include/tl.h."""
    _fields_ = [("x", ctypes.c_void_p), ("Wpacked", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("y", ctypes.c_void_p),
                ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("group", ctypes.c_int64)]


class TlError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {tl_status_str(status)} (tl_status {int(status)})")


def _load():
    # torch ships its own copy of the HIP runtime under the same soname.  Importing torch
    # first makes libtl.so bind to that copy, so that torch's streams and device memory
    # and this library's kernels live in one runtime instead of two.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2506_23025_amd.build); "
            "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    i64, vp, u16, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_uint16, ctypes.c_size_t
    ci = ctypes.c_int
    L.tl_status_str.argtypes = [ci]
    L.tl_status_str.restype = ctypes.c_char_p
    L.tl_row_stride_bytes.argtypes = [ci, i64]
    L.tl_row_stride_bytes.restype = sz
    L.tl_packed_bytes.argtypes = [ci, i64, i64]
    L.tl_packed_bytes.restype = sz
    for name in ("tl_pack_2bit", "tl_pack_1p6bit", "tl_pack_1p6bit_fx", "tl_unpack_1p6bit_fx"):
        getattr(L, name).argtypes = [vp, i64, i64, vp]
        getattr(L, name).restype = ci
    L.tl_quantize.argtypes = [vp, i64, i64, ctypes.c_double, vp, vp, vp]
    L.tl_quantize.restype = ci
    L.tl_unpack.argtypes = [ci, vp, i64, i64, vp]
    L.tl_unpack.restype = ci
    L.tl_unpack_dev.argtypes = [ci, vp, i64, i64, vp, vp]
    L.tl_unpack_dev.restype = ci
    L.tl_ternary_gemm.argtypes = [vp, vp, u16, vp, i64, i64, i64, vp]
    L.tl_ternary_gemm.restype = ci
    L.tl_ternary_gemm_path.argtypes = [vp, vp, u16, vp, i64, i64, i64, vp, ci]
    L.tl_ternary_gemm_path.restype = ci
    L.tl_ternary_gemm_grouped.argtypes = [ctypes.POINTER(tl_gemm_job), i64, vp]
    L.tl_ternary_gemm_grouped.restype = ci
    L.tl_ternary_gemm_1p6.argtypes = [vp, vp, u16, vp, i64, i64, i64, vp]
    L.tl_ternary_gemm_1p6.restype = ci
    L.tl_ternary_gemm_1p6_fx.argtypes = [vp, vp, u16, vp, i64, i64, i64, vp]
    L.tl_ternary_gemm_1p6_fx.restype = ci
    L.tl_ternary_gemm_gs.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, vp]
    L.tl_ternary_gemm_gs.restype = ci
    L.tl_ternary_gemm_1p6_grouped.argtypes = [ctypes.POINTER(tl_gemm_job), i64, ci, vp]
    L.tl_ternary_gemm_1p6_grouped.restype = ci
    L.tl_ternary_gemm_gs_grouped.argtypes = [ctypes.POINTER(tl_gemm_gs_job), i64, vp]
    L.tl_ternary_gemm_gs_grouped.restype = ci
    L.tl_ternary_gemm_which.argtypes = [i64, i64, i64]
    L.tl_ternary_gemm_which.restype = ci
    L.tl_init.argtypes = []
    L.tl_init.restype = ci
    L.tl_probe_copy.argtypes = [vp, vp, sz, vp]
    L.tl_probe_copy.restype = ci
    L.tl_probe_read.argtypes = [vp, sz, vp, vp]
    L.tl_probe_read.restype = ci
    L.tl_probe_mfma.argtypes = [vp, i64, vp, i64, i64, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.tl_probe_mfma.restype = ci
    return L


_lib = _load()


def raw():
    """The ctypes library object (for callers that time raw calls)."""
    return _lib


def _check(status, where):
    if status != TL_OK:
        raise TlError(status, where)


def _ptr(t):
    """Device address of a torch tensor, or the integer itself."""
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _host_w(W):
    W = np.ascontiguousarray(W, dtype=np.int8)
    if W.ndim != 2:
        raise ValueError("W must be [N][K]")
    return W


# ---- geometry ------------------------------------------------------------------

def tl_status_str(status):
    return _lib.tl_status_str(int(status)).decode()


def tl_row_stride_bytes(fmt, K):
    return int(_lib.tl_row_stride_bytes(fmt, K))


def tl_packed_bytes(fmt, N, K):
    return int(_lib.tl_packed_bytes(fmt, N, K))


# ---- host packers / unpackers ----------------------------------------------------

def tl_pack_2bit(W):
    W = _host_w(W)
    N, K = W.shape
    out = np.empty((N, tl_row_stride_bytes(TL_FMT_2BIT, K) // 4), dtype=np.uint32)
    _check(_lib.tl_pack_2bit(W.ctypes.data, N, K, out.ctypes.data), "tl_pack_2bit")
    return out


def tl_pack_1p6bit(W):
    W = _host_w(W)
    N, K = W.shape
    out = np.empty((N, tl_row_stride_bytes(TL_FMT_1P6BIT, K)), dtype=np.uint8)
    _check(_lib.tl_pack_1p6bit(W.ctypes.data, N, K, out.ctypes.data), "tl_pack_1p6bit")
    return out


def tl_quantize(W, eps=1e-5):
    """float32 [N][K] -> (What int8 [N][K], gamma float, gamma_fp16_bits int)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    What = np.empty((N, K), dtype=np.int8)
    g = ctypes.c_double(0.0)
    gb = ctypes.c_uint16(0)
    _check(_lib.tl_quantize(W.ctypes.data, N, K, float(eps), What.ctypes.data, ctypes.addressof(g),
                            ctypes.addressof(gb)), "tl_quantize")
    return What, g.value, gb.value


def tl_pack_1p6bit_fx(W):
    W = _host_w(W)
    N, K = W.shape
    out = np.empty((N, tl_row_stride_bytes(TL_FMT_1P6BIT, K)), dtype=np.uint8)
    _check(_lib.tl_pack_1p6bit_fx(W.ctypes.data, N, K, out.ctypes.data), "tl_pack_1p6bit_fx")
    return out


def tl_unpack_1p6bit_fx(packed, N, K):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    if packed.size != tl_packed_bytes(TL_FMT_1P6BIT, N, K):
        raise ValueError("packed size does not match N, K")
    out = np.empty((N, K), dtype=np.int8)
    _check(_lib.tl_unpack_1p6bit_fx(packed.ctypes.data, N, K, out.ctypes.data), "tl_unpack_1p6bit_fx")
    return out


def tl_unpack(fmt, packed, N, K):
    packed = np.ascontiguousarray(packed)
    if packed.nbytes != tl_packed_bytes(fmt, N, K):
        raise ValueError("packed size does not match fmt, N, K")
    out = np.empty((N, K), dtype=np.int8)
    _check(_lib.tl_unpack(fmt, packed.ctypes.data, N, K, out.ctypes.data), "tl_unpack")
    return out


# ---- device entry points ---------------------------------------------------------

def tl_unpack_dev(fmt, packed, N, K, W_out, stream=None):
    _check(_lib.tl_unpack_dev(fmt, _ptr(packed), N, K, _ptr(W_out), _stream(stream)), "tl_unpack_dev")


def tl_ternary_gemm(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream=None):
    _check(_lib.tl_ternary_gemm(_ptr(x), _ptr(Wpacked), gamma_fp16_bits, _ptr(y), M, N, K,
                                _stream(stream)), "tl_ternary_gemm")


def tl_ternary_gemm_path(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream=None, path=TL_PATH_AUTO):
    _check(_lib.tl_ternary_gemm_path(_ptr(x), _ptr(Wpacked), gamma_fp16_bits, _ptr(y), M, N, K,
                                     _stream(stream), path), "tl_ternary_gemm_path")


def make_jobs(jobs):
    """[(x, Wpacked, gamma_fp16_bits, y, M, N, K), ...] -> ctypes array of tl_gemm_job."""
    arr = (tl_gemm_job * len(jobs))()
    for a, (x, Wp, gbits, y, M, N, K) in zip(arr, jobs):
        a.x, a.Wpacked, a.y = _ptr(x), _ptr(Wp), _ptr(y)
        a.M, a.N, a.K, a.gamma_fp16_bits = M, N, K, gbits
    return arr


def tl_ternary_gemm_grouped(jobs, stream=None):
    """jobs: list of (x, Wpacked, gamma_fp16_bits, y, M, N, K), or an array made by make_jobs."""
    arr = jobs if isinstance(jobs, ctypes.Array) else make_jobs(jobs)
    _check(_lib.tl_ternary_gemm_grouped(arr, len(arr), _stream(stream)), "tl_ternary_gemm_grouped")


def tl_ternary_gemm_1p6(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream=None):
    _check(_lib.tl_ternary_gemm_1p6(_ptr(x), _ptr(Wpacked), gamma_fp16_bits, _ptr(y), M, N, K,
                                    _stream(stream)), "tl_ternary_gemm_1p6")


def tl_ternary_gemm_1p6_fx(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream=None):
    _check(_lib.tl_ternary_gemm_1p6_fx(_ptr(x), _ptr(Wpacked), gamma_fp16_bits, _ptr(y), M, N, K,
                                       _stream(stream)), "tl_ternary_gemm_1p6_fx")


def tl_init():
    _check(_lib.tl_init(), "tl_init")


def tl_ternary_gemm_which(M, N, K):
    return int(_lib.tl_ternary_gemm_which(M, N, K))


def tl_ternary_gemm_gs(x, Wpacked, scales, group, y, M, N, K, stream=None):
    _check(_lib.tl_ternary_gemm_gs(_ptr(x), _ptr(Wpacked), _ptr(scales), group, _ptr(y), M, N, K,
                                   _stream(stream)), "tl_ternary_gemm_gs")


def tl_ternary_gemm_1p6_grouped(jobs, fmt=TL_FMT_1P6BIT, stream=None):
    """jobs: list of (x, Wpacked, gamma_fp16_bits, y, M, N, K) with 1.6-bit weights, or an array made by make_jobs."""
    arr = jobs if isinstance(jobs, ctypes.Array) else make_jobs(jobs)
    _check(_lib.tl_ternary_gemm_1p6_grouped(arr, len(arr), fmt, _stream(stream)), "tl_ternary_gemm_1p6_grouped")


def make_gs_jobs(jobs):
    """[(x, Wpacked, scales, group, y, M, N, K), ...] -> ctypes array of tl_gemm_gs_job."""
    arr = (tl_gemm_gs_job * len(jobs))()
    for a, (x, Wp, sc, group, y, M, N, K) in zip(arr, jobs):
        a.x, a.Wpacked, a.scales, a.y = _ptr(x), _ptr(Wp), _ptr(sc), _ptr(y)
        a.M, a.N, a.K, a.group = M, N, K, group
    return arr


def tl_ternary_gemm_gs_grouped(jobs, stream=None):
    """jobs: list of (x, Wpacked, scales, group, y, M, N, K), or an array made by make_gs_jobs."""
    arr = jobs if isinstance(jobs, ctypes.Array) else make_gs_jobs(jobs)
    _check(_lib.tl_ternary_gemm_gs_grouped(arr, len(arr), _stream(stream)), "tl_ternary_gemm_gs_grouped")


def tl_probe_copy(dst, src, nbytes, stream=None):
    _check(_lib.tl_probe_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "tl_probe_copy")


def tl_probe_read(src, nbytes, sink, stream=None):
    _check(_lib.tl_probe_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "tl_probe_read")


def tl_probe_mfma(x, x_elems, Wpacked, w_words, iters, sink, stream=None):
    """Returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(_lib.tl_probe_mfma(_ptr(x), x_elems, _ptr(Wpacked), w_words, iters, _ptr(sink), ctypes.byref(flops),
                              _stream(stream)), "tl_probe_mfma")
    return flops.value
