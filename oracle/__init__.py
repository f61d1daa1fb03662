"""CPU oracle for the ternary linear layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to oracle/ternary_oracle.c (plain C, fp64, written from the
paper's definitions; see that file's header for the passage each routine follows).
Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package; the product path never does and never falls back to it.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None

_i8p = np.ctypeslib.ndpointer(np.int8, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(np.uint64, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_i64 = ctypes.c_int64


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.orc_pack2.argtypes = [_i8p, _i64, ctypes.c_int, _u64p]
        L.orc_pack2.restype = ctypes.c_int
        L.orc_unpack2.argtypes = [_u64p, _i64, ctypes.c_int, _i8p]
        L.orc_unpack2.restype = ctypes.c_int
        L.orc_pack2_matrix.argtypes = [_i8p, _i64, _i64, _u32p]
        L.orc_pack2_matrix.restype = ctypes.c_int
        L.orc_unpack2_matrix.argtypes = [_u32p, _i64, _i64, _i8p]
        L.orc_unpack2_matrix.restype = ctypes.c_int
        L.orc_pack_fx_block.argtypes = [_i8p, ctypes.c_int, ctypes.c_int]
        L.orc_pack_fx_block.restype = _i64
        L.orc_unpack_fx_div_block.argtypes = [_i64, ctypes.c_int, ctypes.c_int, _i8p]
        L.orc_unpack_fx_div_block.restype = None
        L.orc_unpack_fx_alg1_block.argtypes = [ctypes.c_int, _i8p]
        L.orc_unpack_fx_alg1_block.restype = None
        L.orc_stride3le.argtypes = [_i64]
        L.orc_stride3le.restype = _i64
        L.orc_pack3le_matrix.argtypes = [_i8p, _i64, _i64, _u8p]
        L.orc_pack3le_matrix.restype = ctypes.c_int
        L.orc_unpack3le_matrix.argtypes = [_u8p, _i64, _i64, _i8p]
        L.orc_unpack3le_matrix.restype = ctypes.c_int
        L.orc_half_to_double.argtypes = [ctypes.c_uint16]
        L.orc_half_to_double.restype = ctypes.c_double
        L.orc_gemm.argtypes = [_u16p, _i8p, ctypes.c_uint16, _f64p, _i64, _i64, _i64]
        L.orc_gemm.restype = None
        L.orc_gemm_packed2.argtypes = [_u16p, _u32p, ctypes.c_uint16, _f64p, _i64, _i64, _i64, _i8p]
        L.orc_gemm_packed2.restype = ctypes.c_int
        L.orc_gemm_packed3le.argtypes = [_u16p, _u8p, ctypes.c_uint16, _f64p, _i64, _i64, _i64, _i8p]
        L.orc_gemm_packed3le.restype = ctypes.c_int
        L.orc_gemm_fixed.argtypes = [_u16p, _i8p, _i64p, _i64, _i64, _i64]
        L.orc_gemm_fixed.restype = ctypes.c_int
        L.orc_num_threads.argtypes = []
        L.orc_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _w(W):
    W = np.ascontiguousarray(W, dtype=np.int8)
    assert W.ndim == 2
    return W


def _xbits(x):
    """fp16 array (or raw uint16 bits) [M][K] -> contiguous uint16 bits."""
    x = np.asarray(x)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    assert x.dtype == np.uint16 and x.ndim == 2
    return np.ascontiguousarray(x)


def _gbits(gamma):
    """gamma given as np.float16 scalar or raw int bits -> int bits."""
    if isinstance(gamma, (np.float16,)):
        return int(np.array(gamma, dtype=np.float16).view(np.uint16))
    return int(gamma)


# --- Sec. 3.1 ---------------------------------------------------------------

def pack2_seq(d, k=16):
    """P of Sec. 3.1 on one digit sequence; returns ceil(n/k) blocks as uint64."""
    d = np.ascontiguousarray(d, dtype=np.int8)
    out = np.zeros((len(d) + k - 1) // k, dtype=np.uint64)
    if lib().orc_pack2(d, len(d), k, out) != 0:
        raise ValueError("digit outside {-1,0,1}")
    return out


def unpack2_seq(blocks, n, k=16):
    blocks = np.ascontiguousarray(blocks, dtype=np.uint64)
    d = np.zeros(n, dtype=np.int8)
    if lib().orc_unpack2(blocks, n, k, d) != 0:
        raise ValueError("digit 3 in packed data")
    return d


def pack2(W):
    W = _w(W)
    N, K = W.shape
    out = np.zeros((N, (K + 15) // 16), dtype=np.uint32)
    if lib().orc_pack2_matrix(W, N, K, out) != 0:
        raise ValueError("weight outside {-1,0,1}")
    return out


def unpack2(packed, K):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    N = packed.shape[0]
    assert packed.shape[1] == (K + 15) // 16
    W = np.zeros((N, K), dtype=np.int8)
    if lib().orc_unpack2_matrix(packed, N, K, W) != 0:
        raise ValueError("code 3 in packed data")
    return W


# --- Sec. 3.2 / App. E / App. F ---------------------------------------------

def pack_fx_block(d, k=5, p=8):
    d = np.ascontiguousarray(d, dtype=np.int8)
    assert len(d) == k
    return int(lib().orc_pack_fx_block(d, k, p))


def unpack_fx_div_block(b, k=5, p=8):
    d = np.zeros(k, dtype=np.int8)
    lib().orc_unpack_fx_div_block(int(b), k, p, d)
    return d


def unpack_fx_alg1_block(b):
    d = np.zeros(5, dtype=np.int8)
    lib().orc_unpack_fx_alg1_block(int(b), d)
    return d


def stride3le(K):
    return int(lib().orc_stride3le(K))


def pack3le(W):
    W = _w(W)
    N, K = W.shape
    out = np.zeros((N, stride3le(K)), dtype=np.uint8)
    if lib().orc_pack3le_matrix(W, N, K, out) != 0:
        raise ValueError("weight outside {-1,0,1}")
    return out


def unpack3le(packed, K):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    N = packed.shape[0]
    assert packed.shape[1] == stride3le(K)
    W = np.zeros((N, K), dtype=np.int8)
    if lib().orc_unpack3le_matrix(packed, N, K, W) != 0:
        raise ValueError("byte > 242 in packed data")
    return W


def pack3fx(W):
    """Rows of the fixed-point 1.6-bit code (Sec. 3.2, k = 5, p = 8): per block of five weights,
    big-endian value Nval = sum_j (w_j + 1) 3^(4-j), byte = ceil(256 Nval / 243) written as
    floor((256 Nval + 242) / 243); a short last block is filled with weight 0; row stride as for
    the plain 1.6-bit form, padding zero."""
    W = _w(W)
    N, K = W.shape
    nb = (K + 4) // 5
    d = np.ones((N, nb * 5), dtype=np.int64)              # digit 1 = weight 0
    d[:, :K] = W.astype(np.int64) + 1
    if d.min() < 0 or d.max() > 2:
        raise ValueError("weight outside {-1,0,1}")
    d = d.reshape(N, nb, 5)
    nval = np.zeros((N, nb), dtype=np.int64)
    for j in range(5):
        nval += d[:, :, j] * 3 ** (4 - j)
    out = np.zeros((N, stride3le(K)), dtype=np.uint8)
    out[:, :nb] = ((nval * 256 + 242) // 243).astype(np.uint8)
    return out


def unpack3fx(packed, K):
    """Digits of the fixed-point code by the closed form of App. E: d'_j = floor(b 3^(j+1) / 2^8) mod 3."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    N = packed.shape[0]
    assert packed.shape[1] == stride3le(K)
    nb = (K + 4) // 5
    b = packed[:, :nb].astype(np.int64)
    W = np.zeros((N, nb, 5), dtype=np.int8)
    for j in range(5):
        W[:, :, j] = ((b * 3 ** (j + 1)) >> 8) % 3 - 1
    return np.ascontiguousarray(W.reshape(N, nb * 5)[:, :K])


def gemm_packed3fx(x, Wp, gamma, K):
    return gemm(x, unpack3fx(Wp, K), gamma)


# --- App. B: ternarisation of trained weights ---------------------------------------

def quantize(W, eps=1e-5):
    """gamma = eps + mean |W| (exactly rounded fp64 sum), What = round(clip(W / gamma, -1, 1)),
    round half to even.  Returns (What int8, gamma float)."""
    import math
    W64 = np.asarray(W, dtype=np.float64)
    gamma = float(eps) + math.fsum(np.abs(W64).ravel().tolist()) / W64.size
    if gamma > 0.0:
        q = np.clip(W64 / gamma, -1.0, 1.0)
    else:
        q = np.zeros_like(W64)
    return np.rint(q).astype(np.int8), gamma


# --- numbers and GEMM ---------------------------------------------------------

def half_to_double(bits):
    return float(lib().orc_half_to_double(int(bits)))


def gemm(x, W, gamma):
    """y[m][n] = gamma * sum_k x[m][k] W[n][k] in fp64 (App. B, Inference). Unrounded."""
    xb = _xbits(x)
    W = _w(W)
    M, K = xb.shape
    N = W.shape[0]
    assert W.shape[1] == K
    y = np.zeros((M, N), dtype=np.float64)
    lib().orc_gemm(xb, W, _gbits(gamma), y, M, N, K)
    return y


def gemm_packed2(x, Wp, gamma, K):
    """The oracle proper: unpack the 2-bit words, then fp64 dot products."""
    xb = _xbits(x)
    Wp = np.ascontiguousarray(Wp, dtype=np.uint32)
    M = xb.shape[0]
    N = Wp.shape[0]
    assert xb.shape[1] == K and Wp.shape[1] == (K + 15) // 16
    y = np.zeros((M, N), dtype=np.float64)
    scratch = np.zeros((N, K), dtype=np.int8)
    if lib().orc_gemm_packed2(xb, Wp, _gbits(gamma), y, M, N, K, scratch) != 0:
        raise ValueError("code 3 in packed data")
    return y


def gemm_packed3le(x, Wp, gamma, K):
    xb = _xbits(x)
    Wp = np.ascontiguousarray(Wp, dtype=np.uint8)
    M = xb.shape[0]
    N = Wp.shape[0]
    assert xb.shape[1] == K and Wp.shape[1] == stride3le(K)
    y = np.zeros((M, N), dtype=np.float64)
    scratch = np.zeros((N, K), dtype=np.int8)
    if lib().orc_gemm_packed3le(xb, Wp, _gbits(gamma), y, M, N, K, scratch) != 0:
        raise ValueError("byte > 242 in packed data")
    return y


def gemm_group_scales(x, W, scales, group):
    """y[m][n] = sum_g scales[g][n] * sum_{k in group g} x[m][k] W[n][k], fp64, unrounded.
    One scale per block of `group` consecutive weights along K and per output row (Sec. 3.3,
    CPU inference: a block of the 2-bit format carries its own fp16 scale, and a block is
    reconstructed as scale times its ternary values; the GPU kernel reads its scales from a
    separate buffer).  scales: fp16 [ceil(K / group)][N]; the last group may be short.
    The definition written out: one fp64 matrix product per group (each exact), scaled, summed."""
    x64 = np.asarray(x, dtype=np.float16).astype(np.float64)
    W64 = _w(W).astype(np.float64)
    s64 = np.asarray(scales, dtype=np.float16).astype(np.float64)
    M, K = x64.shape
    N = W64.shape[0]
    G = (K + group - 1) // group
    assert W64.shape[1] == K and s64.shape == (G, N)
    y = np.zeros((M, N), dtype=np.float64)
    for g in range(G):
        k0, k1 = g * group, min(K, (g + 1) * group)
        y += (x64[:, k0:k1] @ W64[:, k0:k1].T) * s64[g][None, :]
    return y


def gemm_packed2_group_scales(x, Wp, scales, group, K):
    return gemm_group_scales(x, unpack2(Wp, K), scales, group)


def gemm_fixed(x, W):
    """Exact integer S * 2^24, S[m][n] = sum_k x[m][k] W[n][k]."""
    xb = _xbits(x)
    W = _w(W)
    M, K = xb.shape
    N = W.shape[0]
    S = np.zeros((M, N), dtype=np.int64)
    if lib().orc_gemm_fixed(xb, W, S, M, N, K) != 0:
        raise ValueError("inf/nan in x")
    return S


def num_threads():
    return int(lib().orc_num_threads())


def to_fp16(y64):
    """fp64 -> fp16, round-to-nearest-even (numpy converts double to half in one rounding)."""
    return np.asarray(y64, dtype=np.float64).astype(np.float16)
