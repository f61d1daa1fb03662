"""CPU tests of the library's host side: exports, geometry, packers against the oracle."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import oracle
import paper_2506_23025_amd as tl
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tl_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    L = ctypes.CDLL(tl.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} declared in tl.h but not exported"
    assert declared == set(tl.EXPORTS)


def test_geometry():
    assert tl.tl_row_stride_bytes(tl.TL_FMT_2BIT, 4096) == 1024
    assert tl.tl_row_stride_bytes(tl.TL_FMT_2BIT, 17) == 8
    assert tl.tl_row_stride_bytes(tl.TL_FMT_1P6BIT, 4096) == 832
    assert tl.tl_row_stride_bytes(tl.TL_FMT_1P6BIT, 11008) == 2208
    assert tl.tl_row_stride_bytes(tl.TL_FMT_2BIT, 0) == 0
    assert tl.tl_row_stride_bytes(7, 64) == 0
    assert tl.tl_packed_bytes(tl.TL_FMT_2BIT, 14336, 4096) == 14336 * 1024
    assert tl.tl_packed_bytes(tl.TL_FMT_2BIT, 0, 4096) == 0
    for K in (1, 5, 79, 80, 81, 4096):
        assert tl.tl_row_stride_bytes(tl.TL_FMT_1P6BIT, K) == oracle.stride3le(K)


@pytest.mark.parametrize("N,K", [(1, 1), (3, 15), (4, 16), (5, 17), (2, 100), (7, 4096), (3, 11008)])
def test_pack_2bit_bit_exact_against_oracle(N, K):
    W = si.ternary_weights(np.random.default_rng(N * 100003 + K), N, K)
    P = tl.tl_pack_2bit(W)
    assert P.dtype == np.uint32 and P.shape == (N, (K + 15) // 16)
    assert np.array_equal(P, oracle.pack2(W))
    assert np.array_equal(tl.tl_unpack(tl.TL_FMT_2BIT, P, N, K), W)
    assert np.array_equal(oracle.unpack2(P, K), W)


@pytest.mark.parametrize("N,K", [(1, 1), (3, 4), (4, 5), (5, 6), (2, 81), (7, 4096), (3, 11008)])
def test_pack_1p6bit_bit_exact_against_oracle(N, K):
    W = si.ternary_weights(np.random.default_rng(N * 100003 + K), N, K)
    P = tl.tl_pack_1p6bit(W)
    assert P.dtype == np.uint8 and P.shape == (N, oracle.stride3le(K))
    assert np.array_equal(P, oracle.pack3le(W))
    assert np.array_equal(tl.tl_unpack(tl.TL_FMT_1P6BIT, P, N, K), W)


def test_pack_1p6bit_fx_matches_paper_code_and_alg1_decode():
    all5 = np.array(list(itertools.product((-1, 0, 1), repeat=5)), dtype=np.int8)
    P = tl.tl_pack_1p6bit_fx(all5)
    want = [oracle.pack_fx_block(d, 5, 8) for d in all5]
    assert P[:, 0].tolist() == want
    assert np.array_equal(tl.tl_unpack_1p6bit_fx(P, 243, 5), all5)
    # ragged rows
    W = si.ternary_weights(np.random.default_rng(8), 3, 4096)
    assert np.array_equal(tl.tl_unpack_1p6bit_fx(tl.tl_pack_1p6bit_fx(W), 3, 4096), W)
    # each byte decodes like the oracle's Alg. 1
    Pw = tl.tl_pack_1p6bit_fx(W)
    for b in range(0, 819, 97):
        assert oracle.unpack_fx_alg1_block(int(Pw[1, b])).tolist() == W[1, 5 * b:5 * b + 5].tolist()


def test_unpack_1p6bit_fx_closed_form_equals_alg1_on_every_byte():
    # the library inverts the code in closed form (V = floor(243 b / 256), then base-3 digits);
    # App. F, Alg. 1 (in the oracle) peels digits with multiplications by 3: same digits for all
    # 256 byte values, also the 13 that no block produces
    P = np.zeros((256, 16), dtype=np.uint8)
    P[:, 0] = np.arange(256)
    got = tl.tl_unpack_1p6bit_fx(P, 256, 5)
    want = np.array([oracle.unpack_fx_alg1_block(b) for b in range(256)], dtype=np.int8)
    assert np.array_equal(got, want)


def test_fx_format_through_the_format_enum():
    # TL_FMT_1P6BIT_FX: same geometry as the plain 1.6-bit form; host unpack = Alg. 1 decode;
    # the library's rows equal the oracle's rows byte for byte
    for K in (5, 64, 4096, 11008):
        assert tl.tl_row_stride_bytes(tl.TL_FMT_1P6BIT_FX, K) == tl.tl_row_stride_bytes(tl.TL_FMT_1P6BIT, K)
    W = si.ternary_weights(np.random.default_rng(9), 5, 643)
    P = tl.tl_pack_1p6bit_fx(W)
    assert np.array_equal(P, oracle.pack3fx(W))
    assert np.array_equal(tl.tl_unpack(tl.TL_FMT_1P6BIT_FX, P, 5, 643), W)


def test_quantize_hand_worked_and_invariants():
    # App. B: gamma = eps + mean|W|, What = round(clip(W / gamma, -1, 1))
    W = np.array([[0.5, -0.5, 0.1, 2.0]], dtype=np.float32)        # mean |W| = 0.775
    What, g, gb = tl.tl_quantize(W, eps=0.0)
    assert g == pytest.approx(0.775, rel=1e-7) and What.tolist() == [[1, -1, 0, 1]]
    assert gb == int(np.float16(g).view(np.uint16))
    # eps enters additively; all-zero weights give gamma = eps and What = 0
    What, g, _ = tl.tl_quantize(np.zeros((3, 5), np.float32), eps=1e-5)
    assert g == 1e-5 and not What.any()
    What, g, _ = tl.tl_quantize(np.zeros((3, 5), np.float32), eps=0.0)
    assert g == 0.0 and not What.any()
    # scaling W by a power of two scales gamma and leaves What alone (eps = 0)
    rng = np.random.default_rng(3)
    W = rng.standard_normal((64, 96)).astype(np.float32)
    Wh1, g1, _ = tl.tl_quantize(W, eps=0.0)
    Wh2, g2, _ = tl.tl_quantize(W * np.float32(8.0), eps=0.0)
    assert g2 == 8.0 * g1 and np.array_equal(Wh1, Wh2)
    # near-Gaussian weights: |W| < gamma / 2 becomes 0, i.e. P(0) = 2 Phi(0.5 sqrt(2 / pi)) - 1 = 0.31
    W = rng.standard_normal((512, 512)).astype(np.float32)
    Wh, g, _ = tl.tl_quantize(W, eps=0.0)
    assert abs(g - np.sqrt(2 / np.pi)) < 5e-3
    assert abs((Wh == 0).mean() - 0.310) < 5e-3 and abs((Wh == 1).mean() - (Wh == -1).mean()) < 5e-3
    assert set(np.unique(Wh).tolist()) == {-1, 0, 1}


def test_quantize_against_oracle_and_fp16_gamma():
    rng = np.random.default_rng(4)
    for shape, eps in (((7, 33), 1e-5), ((128, 257), 0.0), ((1, 4096), 1e-3)):
        W = (rng.standard_normal(shape) * rng.uniform(0.01, 3.0)).astype(np.float32)
        Wh, g, gb = tl.tl_quantize(W, eps=eps)
        Wo, go = oracle.quantize(W, eps)
        assert abs(g - go) <= 4e-16 * go
        away_from_tie = np.abs(np.abs(W.astype(np.float64) / go) - 0.5) > 1e-9
        assert np.array_equal(Wh[away_from_tie], Wo[away_from_tie])
        assert gb == int(np.float16(g).view(np.uint16))
    # the fp64 -> fp16 rounding of gamma, through 1 x 1 matrices (gamma = |w|): normal, subnormal,
    # halfway cases, overflow
    vals = [1.0, 0.02, 65504.0, 65519.9, 65520.0, 1e6, 6.1035e-5, 6.0e-8, 2.98e-8, 2.9802322387695312e-8,
            8.940696716308594e-08, 0.333251953125, 0.3333740234375, 1.00048828125, 1.0009765625 * 1.5]
    vals += list(np.abs(rng.standard_normal(200)) * 10.0 ** rng.integers(-8, 5, 200))
    for v in vals:
        w = np.array([[v]], dtype=np.float32)
        _, g, gb = tl.tl_quantize(w, eps=0.0)
        assert g == float(w[0, 0])
        with np.errstate(over="ignore"):
            assert gb == int(np.float64(g).astype(np.float16).view(np.uint16)), v
    with pytest.raises(tl.TlError):
        tl.tl_quantize(np.array([[np.nan]], np.float32))
    with pytest.raises(tl.TlError):
        tl.tl_quantize(np.ones((2, 2), np.float32), eps=-1.0)


def test_error_codes():
    L = tl.raw()
    W = np.zeros((2, 16), dtype=np.int8)
    out = np.zeros((2, 1), dtype=np.uint32)
    assert L.tl_pack_2bit(None, 2, 16, out.ctypes.data) == tl.TL_ERR_NULL
    assert L.tl_pack_2bit(W.ctypes.data, 2, 16, None) == tl.TL_ERR_NULL
    assert L.tl_pack_2bit(W.ctypes.data, 0, 16, out.ctypes.data) == tl.TL_ERR_SHAPE
    assert L.tl_pack_2bit(W.ctypes.data, 2, -1, out.ctypes.data) == tl.TL_ERR_SHAPE
    W[1, 3] = 2
    assert L.tl_pack_2bit(W.ctypes.data, 2, 16, out.ctypes.data) == tl.TL_ERR_VALUE
    W[1, 3] = -2
    out8 = np.zeros((2, 16), dtype=np.uint8)
    assert L.tl_pack_1p6bit(W.ctypes.data, 2, 16, out8.ctypes.data) == tl.TL_ERR_VALUE
    assert L.tl_pack_1p6bit_fx(W.ctypes.data, 2, 16, out8.ctypes.data) == tl.TL_ERR_VALUE
    # invalid codes on unpack
    bad = np.array([[0x55555557]], dtype=np.uint32)
    o = np.zeros((1, 16), dtype=np.int8)
    assert L.tl_unpack(tl.TL_FMT_2BIT, bad.ctypes.data, 1, 16, o.ctypes.data) == tl.TL_ERR_VALUE
    bad8 = np.zeros((1, 16), dtype=np.uint8)
    bad8[0, 0] = 243
    assert L.tl_unpack(tl.TL_FMT_1P6BIT, bad8.ctypes.data, 1, 5, o.ctypes.data) == tl.TL_ERR_VALUE
    assert L.tl_unpack(9, bad8.ctypes.data, 1, 5, o.ctypes.data) == tl.TL_ERR_UNSUPPORTED
    # device entry points validate before touching the GPU
    assert L.tl_ternary_gemm(None, None, 0, None, 1, 1, 16, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm(16, 16, 0, 16, 0, 1, 16, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm(24, 16, 0, 16, 1, 1, 16, None) == tl.TL_ERR_ALIGN
    assert L.tl_ternary_gemm_path(16, 16, 0, 16, 1, 1, 16, None, 99) == tl.TL_ERR_UNSUPPORTED
    assert L.tl_ternary_gemm_1p6(None, 16, 0, 16, 1, 1, 16, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_grouped(None, 2, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_grouped(tl.make_jobs([(16, 16, 0, 16, 0, 1, 16)]), 1, None) == tl.TL_ERR_SHAPE
    assert L.tl_unpack_dev(tl.TL_FMT_2BIT, None, 1, 16, None, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_gs(16, 16, None, 256, 16, 1, 1, 16, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_gs(16, 16, 16, 24, 16, 1, 1, 16, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_gs(16, 16, 16, 0, 16, 1, 1, 16, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_gs(16, 16, 8, 256, 16, 1, 1, 16, None) == tl.TL_ERR_ALIGN
    # the grouped forms check every job before anything is launched
    ok = tl.make_jobs([(16, 16, 0, 32, 1, 16, 64)])
    assert L.tl_ternary_gemm_1p6_grouped(None, 0, tl.TL_FMT_1P6BIT, None) == tl.TL_OK
    assert L.tl_ternary_gemm_1p6_grouped(None, 2, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_1p6_grouped(ok, 1, tl.TL_FMT_2BIT, None) == tl.TL_ERR_VALUE
    assert L.tl_ternary_gemm_1p6_grouped(ok, 1, 7, None) == tl.TL_ERR_VALUE
    assert L.tl_ternary_gemm_1p6_grouped(ok, -1, tl.TL_FMT_1P6BIT_FX, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_1p6_grouped(tl.make_jobs([(16, 16, 0, 32, 1, 16, 64), (16, 16, 0, 0, 1, 16, 64)]), 2,
                                         tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_1p6_grouped(tl.make_jobs([(16, 24, 0, 32, 1, 16, 64)]), 1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_ALIGN
    assert L.tl_ternary_gemm_1p6_grouped(tl.make_jobs([(16, 16, 0, 32, 1, 0, 64)]), 1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_gs_grouped(None, 0, None) == tl.TL_OK
    assert L.tl_ternary_gemm_gs_grouped(None, 2, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_gs_grouped(tl.make_gs_jobs([(16, 16, 0, 256, 32, 1, 16, 64)]), 1, None) == tl.TL_ERR_NULL
    assert L.tl_ternary_gemm_gs_grouped(tl.make_gs_jobs([(16, 16, 24, 256, 32, 1, 16, 64)]), 1, None) == tl.TL_ERR_ALIGN
    assert L.tl_ternary_gemm_gs_grouped(tl.make_gs_jobs([(16, 16, 32, 24, 48, 1, 16, 64)]), 1, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_gs_grouped(tl.make_gs_jobs([(16, 16, 32, 256, 48, 1, 16, 64)]), 5000, None) == tl.TL_ERR_SHAPE
    assert L.tl_probe_copy(16, 16, 24, None) == tl.TL_ERR_SHAPE
    assert L.tl_probe_read(16, 24, 16, None) == tl.TL_ERR_SHAPE
    assert L.tl_probe_read(16, 32, None, None) == tl.TL_ERR_NULL
    assert L.tl_probe_read(16, 32, 18, None) == tl.TL_ERR_ALIGN
    assert L.tl_probe_mfma(None, 8, 16, 8, 1, 16, None, None) == tl.TL_ERR_NULL
    assert L.tl_probe_mfma(16, 0, 16, 8, 1, 16, None, None) == tl.TL_ERR_SHAPE
    assert L.tl_probe_mfma(16, 8, 16, 8, 0, 16, None, None) == tl.TL_ERR_SHAPE
    assert L.tl_probe_mfma(16, 8, 18, 8, 1, 16, None, None) == tl.TL_ERR_ALIGN
    for s in range(8):
        assert tl.tl_status_str(s)


def test_padding_bits_and_bytes():
    W = np.ones((1, 19), dtype=np.int8)
    P = tl.tl_pack_2bit(W)
    assert P.tolist() == [[0xAAAAAAAA, 0x5555556A]]
    P3 = tl.tl_pack_1p6bit(W)
    assert P3[0, :4].tolist() == [242, 242, 242, 2 + 6 + 18 + 54 + 81]
    assert not P3[0, 4:].any()


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    # include/tl.h under a strict C99 compiler, a C program linked against libtl.so
    import os
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    cc = shutil.which("gcc") or shutil.which("cc")
    assert cc, "no C compiler"
    libdir = os.path.dirname(tl.LIB_PATH)
    exe = str(tmp_path / "abi_host")
    cmd = [cc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
           os.path.join(root, "tests", "c", "abi_host.c"), "-o", exe, "-L", libdir, "-ltl",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr)


def test_workgroup_allocator_invariants(tmp_path):
    # csrc/tl_deal.hpp is host logic without an entry point of its own: a small C++ program checks its
    # invariants (every job served, counts add up, monotone in cost, no single move helps)
    import os
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    cxx = shutil.which("g++") or shutil.which("c++")
    assert cxx, "no C++ compiler"
    exe = str(tmp_path / "deal_host")
    cmd = [cxx, "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "paper_2506_23025_amd", "csrc"),
           os.path.join(root, "tests", "c", "deal_host.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr)


def test_kernel_choice_is_a_pure_function_of_the_shape():
    # decode batch sizes stream the weights; the prefill sizes of the workloads use the tiled MFMA
    # kernel; shapes neither fast kernel takes fall back; invalid sizes give no path
    for M in (1, 2, 4, 8, 16):
        for N, K in ((2048, 2048), (4096, 4096), (14336, 4096), (4096, 11008)):
            assert tl.tl_ternary_gemm_which(M, N, K) == tl.TL_PATH_GEMV
    for M in (1024, 2048):
        assert tl.tl_ternary_gemm_which(M, 14336, 4096) == tl.TL_PATH_MFMA
    assert tl.tl_ternary_gemm_which(3, 70, 100) == tl.TL_PATH_GENERIC      # K not a multiple of 64
    assert tl.tl_ternary_gemm_which(0, 16, 64) == tl.TL_PATH_AUTO
    assert tl.tl_ternary_gemm_which(1, 16, -64) == tl.TL_PATH_AUTO
    # the model follows the measured crossovers (small-M kernel up to M = 768 at 4096 -> 14336)
    assert tl.tl_ternary_gemm_which(512, 14336, 4096) == tl.TL_PATH_GEMV
    assert tl.tl_ternary_gemm_which(1024, 4096, 11008) == tl.TL_PATH_MFMA
