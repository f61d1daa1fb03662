"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest

import oracle
import paper_2506_23025_amd as tl
import synth_inputs as si
from parity import REL_TOL, assert_close, dev_u32, floors, to_dev

pytestmark = pytest.mark.gpu


def run_gemm(x, Wp, g, N, K, path=tl.TL_PATH_AUTO):
    import torch
    M = x.shape[0]
    xd, wd = to_dev(x.view(np.uint16).view(np.int16)), dev_u32(Wp)
    yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")   # poison
    tl.tl_ternary_gemm_path(xd, wd, si.gamma_bits(g), yd, M, N, K, path=path)
    torch.cuda.synchronize()
    return yd.cpu().numpy().view(np.float16)


def run_gemm3(x, Wp, g, N, K):
    import torch
    M = x.shape[0]
    xd, wd = to_dev(x.view(np.uint16).view(np.int16)), to_dev(Wp)
    yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
    tl.tl_ternary_gemm_1p6(xd, wd, si.gamma_bits(g), yd, M, N, K)
    torch.cuda.synchronize()
    return yd.cpu().numpy().view(np.float16)


@pytest.mark.parametrize("N,K", [(1, 1), (5, 17), (33, 100), (64, 4096), (7, 11008)])
def test_unpack_dev_2bit_bit_exact(N, K):
    import torch
    W = si.ternary_weights(np.random.default_rng(N + K), N, K)
    P = oracle.pack2(W)
    out = torch.full((N, K), 77, dtype=torch.int8, device="cuda")
    tl.tl_unpack_dev(tl.TL_FMT_2BIT, dev_u32(P), N, K, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), W)


@pytest.mark.parametrize("N,K", [(1, 1), (5, 17), (33, 101), (64, 4096), (7, 11008)])
def test_unpack_dev_1p6bit_bit_exact(N, K):
    import torch
    W = si.ternary_weights(np.random.default_rng(N + K), N, K)
    P = oracle.pack3le(W)
    out = torch.full((N, K), 77, dtype=torch.int8, device="cuda")
    tl.tl_unpack_dev(tl.TL_FMT_1P6BIT, to_dev(P), N, K, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), W)


GENERIC_SHAPES = [(1, 1, 1), (1, 3, 16), (2, 5, 17), (3, 70, 100), (5, 129, 4096), (1, 2048, 2048),
                  (4, 64, 11008), (17, 33, 1000), (33, 100, 2047), (16, 4096, 4095), (40, 50, 2050)]


@pytest.mark.parametrize("M,N,K", GENERIC_SHAPES)
def test_gemm_generic_matches_oracle(M, N, K):
    x, W, g = si.layer(1000 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    assert np.array_equal(Wp, oracle.pack2(W))
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GENERIC)
    assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"generic {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", GENERIC_SHAPES)
def test_gemm_1p6_matches_oracle(M, N, K):
    x, W, g = si.layer(2000 + M + N + K, M, N, K)
    Wp = tl.tl_pack_1p6bit(W)
    assert np.array_equal(Wp, oracle.pack3le(W))
    y = run_gemm3(x, Wp, g, N, K)
    assert_close(y, oracle.gemm_packed3le(x, Wp, g, K), x, g, f"1.6-bit {M}x{N}x{K}")


def test_gemm_exact_cases_generic():
    K = 128
    rng = np.random.default_rng(4)
    x = si.activations(rng, 3, K)
    g = np.float16(0.02)
    eye = np.eye(K, dtype=np.int8)
    y = run_gemm(x, tl.tl_pack_2bit(eye), g, K, K, tl.TL_PATH_GENERIC)
    assert np.array_equal(y, oracle.to_fp16(oracle.gemm(x, eye, g)))      # single product: exact
    y0 = run_gemm(x, tl.tl_pack_2bit(np.zeros((K, K), dtype=np.int8)), g, K, K, tl.TL_PATH_GENERIC)
    assert not y0.view(np.uint16).any()


# ---------------------------------------------------------------- fast small-M kernel

GEMV_SHAPES = [
    (1, 16, 64), (1, 1, 64), (3, 17, 128), (16, 100, 512), (5, 33, 576), (2, 48, 1024),
    (1, 2048, 2048), (7, 272, 4096), (16, 4099, 4096), (4, 40, 11008), (1, 4112, 4160),
    (17, 64, 1024), (33, 130, 2048), (64, 96, 4096), (9, 2100, 8192),
]


@pytest.mark.parametrize("M,N,K", GEMV_SHAPES)
def test_gemv_matches_oracle(M, N, K):
    x, W, g = si.layer(3000 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"gemv {M}x{N}x{K}")


LONGK_SHAPES = [
    # lone calls with 4096 < K <= 16384 and at most two tiles per workgroup: the long-K form (passes of a
    # wave one slice of 512 apart in blocks of 8).  Two, three and four passes, a ninth slice of 64
    # weights only, a ragged last slice, one and two tiles per workgroup, several blocks of 16 rows,
    # and the sizes around its limits (8192 columns; 16384 = 32 slices; beyond both the other kernels)
    (1, 4096, 11008), (16, 4096, 14336), (3, 272, 4160), (5, 16, 4608), (1, 8192, 8192), (16, 8192, 5120),
    (7, 4112, 8192), (40, 1024, 11008), (2, 512, 16384), (4, 8208, 8192), (9, 64, 16448), (16, 4096, 16384),
    (33, 2048, 12288), (1, 48, 12352),
]


@pytest.mark.parametrize("M,N,K", LONGK_SHAPES)
def test_gemv_long_k_lone_calls(M, N, K):
    x, W, g = si.layer(5600 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    if N * K <= 4096 * 4096:
        assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"long K {M}x{N}x{K}")
    else:
        cols = np.sort(np.random.default_rng(5).choice(N, 384, replace=False))
        cols = np.unique(np.concatenate([cols, np.arange(0, N, 16), np.arange(15, N, 16)[:64]]))[:640]
        assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g, f"long K {M}x{N}x{K} sampled")
        assert not (y.view(np.int16) == -21555).all(axis=0).any()


def test_gemv_rejects_k_not_multiple_of_64():
    import torch
    t = torch.zeros(4096, dtype=torch.int16, device="cuda")
    with pytest.raises(tl.TlError) as e:
        tl.tl_ternary_gemm_path(t, t, 0, t, 1, 16, 48, path=tl.TL_PATH_GEMV)
    assert e.value.status == tl.TL_ERR_UNSUPPORTED


def test_gemv_structured_weights():
    # zero, identity, dense +-1: the kernel's time and correctness do not depend on the values
    K = N = 512
    rng = np.random.default_rng(11)
    x = si.activations(rng, 6, K)
    g = np.float16(0.03)
    for W in (np.zeros((N, K), np.int8), np.eye(K, dtype=np.int8), -np.eye(K, dtype=np.int8),
              np.ones((N, K), np.int8), -np.ones((N, K), np.int8),
              (rng.integers(0, 2, (N, K)) * 2 - 1).astype(np.int8)):
        Wp = tl.tl_pack_2bit(W)
        y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
        assert_close(y, oracle.gemm(x, W, g), x, g, "structured")


def test_gemv_large_and_tiny_activations():
    # |x| up to the fp16 maximum and down to subnormals must not disturb the decode trick
    K, N = 1024, 64
    rng = np.random.default_rng(12)
    W = si.ternary_weights(rng, N, K)
    g = np.float16(1.0)
    big = (rng.standard_normal((2, K)) * 40).astype(np.float16)
    tiny = (rng.standard_normal((2, K)) * 1e-6).astype(np.float16)
    x = np.concatenate([big, tiny])
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    assert_close(y, oracle.gemm(x, W, g), x, g, "range")


def test_gemv_is_deterministic():
    M, N, K = 8, 4096, 4096
    x, W, g = si.layer(99, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y0 = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    for _ in range(5):
        assert np.array_equal(run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV).view(np.uint16), y0.view(np.uint16))


def test_gemv_odd_symmetry_within_tolerance():
    # y(-W) = -y holds exactly for the oracle.  The small-M kernel computes sum (w + 1) x - sum x in
    # fp32, which is not an odd function of W bit for bit, so the two GPU results are compared at
    # the tolerance (each against its own oracle value) and their disagreement is bounded by two
    # output roundings plus the accumulation floor; the generic kernel (w x summed directly) is odd
    # bit for bit.
    M, N, K = 8, 1024, 4096
    x, W, g = si.layer(98, M, N, K)
    ref = oracle.gemm(x, W, g)
    assert np.array_equal(oracle.gemm(x, -W, g), -ref)
    yp = run_gemm(x, tl.tl_pack_2bit(W), g, N, K, tl.TL_PATH_GEMV)
    yn = run_gemm(x, tl.tl_pack_2bit(-W), g, N, K, tl.TL_PATH_GEMV)
    assert_close(yp, ref, x, g, "y(W)")
    assert_close(yn, -ref, x, g, "y(-W)")
    d = np.abs(yp.astype(np.float64) + yn.astype(np.float64))
    assert np.all(d <= 2 * REL_TOL * np.maximum(np.abs(ref), floors(x, g, K)))
    gp = run_gemm(x, tl.tl_pack_2bit(W), g, N, K, tl.TL_PATH_GENERIC)
    gn = run_gemm(x, tl.tl_pack_2bit(-W), g, N, K, tl.TL_PATH_GENERIC)
    assert np.array_equal(gp.view(np.uint16) ^ np.uint16(0x8000), gn.view(np.uint16))


def test_gemv_exact_cases_error_in_floor_units():
    # W = 0 and W = I have exact answers (0 and fp16(gamma x)).  The small-M kernel reaches them
    # through sum (w + 1) x - sum x, so what is left is fp32 accumulation noise of the two sums:
    # measured here in units of the accumulation floor 2^-24 sqrt(K) ||x||_2 gamma (the tolerance
    # allows 4 of them), for a short and a long K.
    rng = np.random.default_rng(97)
    g = np.float16(0.03)
    for K in (512, 4096, 32768):
        x = si.activations(rng, 4, K)
        unit = float(g) * 2.0 ** -24 * np.sqrt(K) * np.sqrt((x.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
        y0 = run_gemm(x, tl.tl_pack_2bit(np.zeros((64, K), np.int8)), g, 64, K, tl.TL_PATH_GEMV)
        worst0 = float(np.max(np.abs(y0.astype(np.float64)) / unit))
        assert worst0 <= 4.0, f"W = 0, K = {K}: {worst0:.2f} floor units"
        N = min(K, 1024)
        I = np.zeros((N, K), np.int8)
        I[np.arange(N), np.arange(N)] = 1
        yi = run_gemm(x, tl.tl_pack_2bit(I), g, N, K, tl.TL_PATH_GEMV)
        exact = float(g) * x[:, :N].astype(np.float64)
        err = np.abs(yi.astype(np.float64) - exact)
        # fp16 rounding of the output (half an ulp of |exact|, at most 2^-11 relative) plus the floor
        assert np.all(err <= 2.0 ** -11 * np.abs(exact) + 4.0 * unit + 2.0 ** -25), f"W = I, K = {K}"
        print(f"K={K}: W=0 worst {worst0:.2f} floor units; W=I worst excess "
              f"{float(np.max((err - 2.0 ** -11 * np.abs(exact)) / unit)):.2f} floor units")


def test_auto_path_full_size_sampled_columns():
    # 4096 -> 14336 at M = 16 through tl_ternary_gemm itself; the oracle checks 512 sampled columns
    M, N, K = 16, 14336, 4096
    x, W, g = si.layer(si.SEEDS["c2"], M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K)
    cols = np.sort(np.random.default_rng(0).choice(N, 512, replace=False))
    ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
    assert_close(y[:, cols], ref, x, g, "full size sampled")


@pytest.mark.parametrize("M", [17, 33, 48])
def test_large_w_just_over_16_rows_sampled_columns(M):
    # W of 18.9 MB: the small-M kernel takes M > 16 in blocks of 32 rows from M = 17 on (a job of
    # 17 rows is one full block of 16 and one block with a single row); 384 sampled columns
    N, K = 18432, 4096
    x, W, g = si.layer(31000 + M, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K)
    cols = np.sort(np.random.default_rng(M).choice(N, 384, replace=False))
    cols[-1] = N - 1
    ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
    assert_close(y[:, cols], ref, x, g, f"large W, M={M}")


@pytest.mark.parametrize("M,N,K", [(1, 1 << 20, 64), (2, 16, 1 << 20), (100000, 16, 64), (3, 33, 262144 + 64)])
def test_extreme_dimensions_sampled(M, N, K):
    # one dimension near what the entry point takes, the others small: a million output rows, a
    # million-long K (2048 slices through the general kernel), a hundred thousand activation rows
    x, W, g = si.layer(9900 + M % 97 + N % 89 + K % 83, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K)
    rows = np.unique(np.concatenate([[0, M - 1], np.random.default_rng(1).integers(0, M, 6)]))
    cols = np.unique(np.concatenate([[0, N - 1], np.random.default_rng(2).integers(0, N, 300)]))
    xs = np.ascontiguousarray(x[rows])
    ref = oracle.gemm(xs, np.ascontiguousarray(W[cols]), g)
    assert_close(y[np.ix_(rows, cols)], ref, xs, g, f"extreme {M}x{N}x{K}")


def test_generic_kernels_take_more_row_blocks_than_one_grid_holds():
    # the plain kernels keep their row blocks on grid.y (65535 of them): 16 rows per block for the
    # 2-bit form (K not a multiple of 64), 4 for the 1.6-bit form (K not a multiple of 8); more
    # rows than that go out as several launches.  Checked on sampled rows, the last ones included.
    rng = np.random.default_rng(65535)
    for fmt, M, N, K in (("2bit", 65535 * 16 + 40, 3, 16), ("1p6", 65535 * 4 + 9, 2, 5)):
        x = si.activations(rng, M, K)
        W = si.ternary_weights(rng, N, K)
        g = np.float16(0.02)
        y = run_gemm(x, tl.tl_pack_2bit(W), g, N, K) if fmt == "2bit" else run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K)
        rows = np.unique(np.concatenate([rng.choice(M, 4096, replace=False), np.arange(M - 64, M), np.arange(64)]))
        xs = np.ascontiguousarray(x[rows])
        assert_close(y[rows], oracle.gemm(xs, W, g), xs, g, f"{fmt} M={M}")


def test_config1_square_2048():
    # config 1: 2048 -> 2048, M = 1, gamma = fp16(0.02); the whole matrix against the oracle
    M, N, K = 1, 2048, 2048
    x, W, g = si.layer(si.SEEDS["c1"], M, N, K, fixed_gamma=0.02)
    Wp = tl.tl_pack_2bit(W)
    assert np.array_equal(Wp, oracle.pack2(W))
    y = run_gemm(x, Wp, g, N, K)
    assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, "config 1")


@pytest.mark.parametrize("M", [1, 16, 64])
def test_config3_block_single_and_grouped(M):
    # config 3: the four linears of a block (QKV, O, gate+up, down) at their full shapes, each as
    # its own call and all four in one grouped call; 256 sampled columns per matrix
    import torch
    rng = np.random.default_rng(si.SEEDS["c3"] + M)
    host, dev, jobs = [], [], []
    for name in si.BLOCK_SHAPES:
        K, N = si.SHAPES[name]
        W = si.ternary_weights(rng, N, K)
        g = si.gamma_uniform(rng)
        x = si.activations(rng, M, K)
        Wp = tl.tl_pack_2bit(W)
        cols = np.sort(np.random.default_rng(N + M).choice(N, 256, replace=False))
        ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
        y1 = run_gemm(x, Wp, g, N, K)
        assert_close(y1[:, cols], ref, x, g, f"block {name} M={M}, single call")
        xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
        yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
        host.append((name, N, K, x, g, cols, ref, y1))
        dev.append((xd, wd, yd))
        jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    for (name, N, K, x, g, cols, ref, y1), (_, _, yd) in zip(host, dev):
        y = yd.cpu().numpy().view(np.float16)
        assert_close(y[:, cols], ref, x, g, f"block {name} M={M}, grouped call")
        assert_close(y, y1.astype(np.float64), x, g, f"block {name} M={M}, grouped against single")


@pytest.mark.parametrize("M,N,K", [(77, 8200, 4096), (390, 130, 1024), (64, 14336, 4096), (400, 33, 2048),
                                   (64, 4096, 11008), (390, 520, 8704), (80, 8192, 6144), (45, 65552, 4608),
                                   (600, 4099, 16384)])
def test_small_m_kernel_blocks_of_32_rows(M, N, K):
    # shapes the small-M kernel takes in blocks of 32 activation rows (two row blocks per wave):
    # ragged last block (77 = 32 + 32 + 13, 390 = 12 x 32 + 6), ragged N, several launches (M = 400);
    # K beyond one pass (sums of both row blocks kept in LDS between passes), a K that ends inside a
    # slice (8704 = 17 x 512), launches cut short so that the runs fit (600 rows of 257 tiles), and
    # a matrix too tall for that form (65552 rows: back to blocks of 16)
    x, W, g = si.layer(8800 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    if N * K <= 4096 * 1024:
        assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"blocks of 32 rows {M}x{N}x{K}")
    else:
        cols = np.sort(np.random.default_rng(M).choice(N, 300, replace=False))
        cols[0], cols[-1] = 0, N - 1
        assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g,
                     f"blocks of 32 rows {M}x{N}x{K} sampled")
    # bit for bit the same on a second run
    assert np.array_equal(y.view(np.uint16), run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV).view(np.uint16))


# ---------------------------------------------------------------- MFMA prefill kernel

MFMA_SHAPES = [
    (256, 256, 64), (1, 16, 64), (300, 200, 128), (128, 128, 4096), (512, 384, 1024),
    (257, 130, 192), (64, 1000, 2048), (1024, 512, 512), (31, 257, 11008),
    # 128 x 128 tiles: K % 128 == 0 runs two sets of waves per tile (1 and 2 steps each), else one
    (4, 33, 128), (130, 260, 256), (100, 140, 320), (384, 4096, 4096),
]


@pytest.mark.parametrize("M,N,K", MFMA_SHAPES)
def test_mfma_matches_oracle(M, N, K):
    x, W, g = si.layer(5000 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_MFMA)
    assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"mfma {M}x{N}x{K}")


def test_mfma_exact_cases():
    # identity / zero weights: every output is a single product (or nothing), so fp16(gamma x) exactly
    K = N = 256
    rng = np.random.default_rng(21)
    x = si.activations(rng, 40, K)
    g = np.float16(0.02)
    eye = np.eye(K, dtype=np.int8)
    y = run_gemm(x, tl.tl_pack_2bit(eye), g, N, K, tl.TL_PATH_MFMA)
    assert np.array_equal(y, oracle.to_fp16(oracle.gemm(x, eye, g)))
    y = run_gemm(x, tl.tl_pack_2bit(-eye), g, N, K, tl.TL_PATH_MFMA)
    assert np.array_equal(y, oracle.to_fp16(oracle.gemm(x, -eye, g)))
    y0 = run_gemm(x, tl.tl_pack_2bit(np.zeros((N, K), np.int8)), g, N, K, tl.TL_PATH_MFMA)
    assert not (y0.view(np.uint16) & 0x7FFF).any()


@pytest.mark.parametrize("M", [256, 1024, 2048])
def test_prefill_full_size_sampled(M):
    # 4096 -> 14336 through the LDS-tiled MFMA kernel; 256 sampled columns
    N, K = 14336, 4096
    x, W, g = si.layer(si.SEEDS["c4"] + M, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_MFMA)
    cols = np.sort(np.random.default_rng(1).choice(N, 256, replace=False))
    ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
    assert_close(y[:, cols], ref, x, g, f"prefill full size M={M}")
    # whichever kernel tl_ternary_gemm picks for this M on its own
    ya = run_gemm(x, Wp, g, N, K)
    assert_close(ya[:, cols], ref, x, g, f"full size, kernel picked by the library, M={M}")
    # y(-W) = -y: the matrix core's internal alignment is not exactly sign-symmetric, so a
    # few outputs may land on the neighbouring fp16 value; nothing may be further off
    y2 = run_gemm(x, tl.tl_pack_2bit(-W), g, N, K, tl.TL_PATH_MFMA)
    assert_close(-y2[:, cols], ref, x, g, f"prefill full size, negated W, M={M}")
    a = y.view(np.int16).astype(np.int32)
    b = (y2.view(np.uint16) ^ 0x8000).view(np.int16).astype(np.int32)
    differs = a != b
    assert np.abs(a - b)[differs & (y != 0)].max(initial=0) <= 1
    assert differs.mean() < 1e-3


@pytest.mark.parametrize("M,N,K", [(4096, 12288, 256), (8192, 2048, 128), (4096, 3840, 192), (512, 14336, 128),
                                   (1024, 2560, 128), (2048, 2560, 64), (5120, 2048, 64)])
def test_mfma_tile_order_covers_every_tile(M, N, K):
    # grids of 32 and 64 row blocks (one region of the tile grid per XCD, walked in bands of four row
    # blocks), of 4, 8 and 16 row blocks (XCDs side by side along the columns), and grids the region
    # scheme does not take (column count not divisible, 40 row blocks): every output written, once,
    # and right on sampled columns (short K keeps the oracle quick)
    import torch
    x, W, g = si.layer(5200 + M + N + K, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm(x, Wp, g, N, K, tl.TL_PATH_MFMA)
    assert not (y.view(np.int16) == -21555).all(axis=0).any()         # no column left at the poison value
    cols = np.sort(np.random.default_rng(4).choice(N, 192, replace=False))
    cols = np.unique(np.concatenate([cols, np.arange(0, N, 256), np.arange(255, N, 256)]))   # both edges of every column block
    assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g, f"mfma tile order {M}x{N}x{K}")


# ---------------------------------------------------------------- grouped launch

def test_grouped_matches_oracle_and_single_calls():
    import torch
    # mixed bag: different shapes, M values (one above 16, one above the small-M limit) and a K
    # the fast kernel cannot take, so that fused and one-by-one launches both occur
    specs = [(1, 4096, 4096), (16, 1000, 1024), (3, 272, 11008), (40, 130, 512), (2, 33, 100),
             (8, 14336, 4096), (200, 96, 256), (5, 48, 64)]
    host, dev, jobs = [], [], []
    for i, (M, N, K) in enumerate(specs):
        x, W, g = si.layer(7000 + i, M, N, K)
        Wp = tl.tl_pack_2bit(W)
        xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
        yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
        host.append((x, W, Wp, g))
        dev.append((xd, wd, yd))
        jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    for (M, N, K), (x, W, Wp, g), (xd, wd, yd) in zip(specs, host, dev):
        y = yd.cpu().numpy().view(np.float16)
        if N * K <= 4096 * 4096:
            assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"grouped {M}x{N}x{K}")
        else:
            cols = np.sort(np.random.default_rng(2).choice(N, 512, replace=False))
            assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g,
                         f"grouped {M}x{N}x{K} sampled")
        # the grouped call and the single call agree bit for bit where they use the same arithmetic
        y1 = run_gemm(x, Wp, g, N, K)
        assert_close(y1, y.astype(np.float64), x, g, "grouped vs single")


@pytest.mark.parametrize("M", [1, 3, 4, 5])
def test_grouped_long_k_several_passes(M):
    # K beyond one pass of 8 slices, enough tiles in the call for the streaming form: passes whose
    # last one has 1, 2, 6 or 8 active waves, a K that ends inside a slice, ragged N; up to 4 rows
    # the next pass's activations are fetched ahead, M = 5 takes the plain path
    import torch
    specs = [(M, 4096, 4160), (M, 4100, 5120), (M, 4096, 11008), (M, 2048, 8192), (M, 1000, 9024)]
    host, dev, jobs = [], [], []
    for i, (m, N, K) in enumerate(specs):
        x, W, g = si.layer(7700 + 10 * M + i, m, N, K)
        Wp = tl.tl_pack_2bit(W)
        xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
        yd = torch.full((m, N), -21555, dtype=torch.int16, device="cuda")
        host.append((x, Wp, g))
        dev.append(yd)
        jobs.append((xd, wd, si.gamma_bits(g), yd, m, N, K))
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    for (m, N, K), (x, Wp, g), yd in zip(specs, host, dev):
        y = yd.cpu().numpy().view(np.float16)
        assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"grouped long K {m}x{N}x{K}")


def test_grouped_many_small_k_jobs():
    # more jobs than one launch carries, all of them short enough in K for the kernel form that
    # keeps a wave's activations in registers: ragged N and M, a K slice that ends inside a
    # 512-block, one-tile jobs next to jobs that give every workgroup a run of several items
    import torch
    specs = [(1, 14336, 4096), (16, 4099, 4096), (3, 17, 576), (9, 1, 64), (2, 300, 1024), (16, 16, 4096),
             (5, 2048, 2048), (1, 12288, 4096), (12, 33, 3136), (4, 640, 512), (1, 4096, 4096), (7, 95, 128),
             (16, 22016, 4096), (2, 48, 2048), (13, 1000, 1600), (1, 31, 4096), (8, 777, 960), (6, 16, 64),
             (24, 130, 1024), (1, 5000, 2560),
             # K longer than one pass of the register-resident form: several passes, sums kept in LDS
             (5, 300, 6144), (16, 64, 11008), (1, 1000, 14336), (3, 17, 32768)]
    host, dev, jobs = [], [], []
    for i, (M, N, K) in enumerate(specs):
        x, W, g = si.layer(7100 + i, M, N, K)
        Wp = tl.tl_pack_2bit(W)
        xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
        yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
        host.append((x, W, Wp, g))
        dev.append((xd, wd, yd))
        jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    first = [yd.cpu().numpy().copy() for _, _, yd in dev]
    for (M, N, K), (x, W, Wp, g), y16 in zip(specs, host, first):
        y = y16.view(np.float16)
        if N * K <= 4096 * 4096:
            assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"grouped {M}x{N}x{K}")
        else:
            cols = np.sort(np.random.default_rng(3).choice(N, 512, replace=False))
            assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g,
                         f"grouped {M}x{N}x{K} sampled")
    # same call again: bit for bit the same
    for _, _, yd in dev:
        yd.fill_(-21555)
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    for (M, N, K), y16, (_, _, yd) in zip(specs, first, dev):
        assert np.array_equal(y16, yd.cpu().numpy()), f"grouped {M}x{N}x{K} not deterministic"


def test_grouped_decode_sweep_as_benchmarked():
    # the benchmark's step, exactly as bench.py launches it: the ten GEMMs of the decode sweep
    # (K = 4096; N = 4096 and 14336; M = 1, 2, 4, 8, 16) in one tl_ternary_gemm_grouped call, each
    # with its own weights; 384 sampled columns per GEMM against the oracle, all rows
    import torch
    K = 4096
    rng = np.random.default_rng(si.SEEDS["c2"] + 77)
    host, dev, jobs = [], [], []
    for name in si.DECODE_SWEEP_SHAPES:
        k, N = si.SHAPES[name]
        assert k == K
        for M in si.DECODE_SWEEP_M:
            W = si.ternary_weights(rng, N, K)
            g = si.gamma_uniform(rng)
            x = si.activations(rng, M, K)
            Wp = tl.tl_pack_2bit(W)
            xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
            yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
            host.append((M, N, x, W, g))
            dev.append((xd, wd, yd))
            jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
    tl.tl_ternary_gemm_grouped(jobs)
    torch.cuda.synchronize()
    for (M, N, x, W, g), (_, _, yd) in zip(host, dev):
        y = yd.cpu().numpy().view(np.float16)
        cols = np.sort(np.random.default_rng(M + N).choice(N, 384, replace=False))
        cols[0], cols[-1] = 0, N - 1                       # first and last column of the matrix
        assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g,
                     f"sweep {M}x{N}x{K}")
        assert not (y.view(np.int16) == -21555).all(axis=0).any()   # every column was written


def test_grouped_empty_and_errors():
    L = tl.raw()
    assert L.tl_ternary_gemm_grouped(None, 0, None) == tl.TL_OK
    assert L.tl_ternary_gemm_grouped(None, 3, None) == tl.TL_ERR_NULL
    bad = tl.make_jobs([(16, 16, 0, 0, 1, 16, 64)])
    assert L.tl_ternary_gemm_grouped(bad, 1, None) == tl.TL_ERR_NULL
    bad = tl.make_jobs([(16, 16, 0, 24, 1, 16, 64)])
    assert L.tl_ternary_gemm_grouped(bad, 1, None) == tl.TL_ERR_ALIGN


# ---------------------------------------------------------------- 1.6-bit small-M kernel

GEMV3_SHAPES = [(1, 16, 8), (1, 1, 640), (4, 272, 640), (3, 17, 1280), (16, 100, 648), (7, 33, 4096),
                (16, 4099, 4096), (3, 40, 11008), (33, 130, 2048), (2, 512, 8192), (64, 48, 4096),
                (300, 272, 4096), (1000, 64, 1280), (5000, 16, 640), (130, 4100, 4480), (70, 100, 4488)]


@pytest.mark.parametrize("M,N,K", GEMV3_SHAPES)
def test_gemv_1p6_matches_oracle(M, N, K):
    x, W, g = si.layer(9000 + M + N + K, M, N, K)
    Wp = tl.tl_pack_1p6bit(W)
    assert np.array_equal(Wp, oracle.pack3le(W))
    y = run_gemm3(x, Wp, g, N, K)
    assert_close(y, oracle.gemm_packed3le(x, Wp, g, K), x, g, f"1.6-bit small-M {M}x{N}x{K}")


# ------------------------------------------------- the paper's fixed-point 1.6-bit code on the GPU

@pytest.mark.parametrize("N,K", [(1, 1), (5, 17), (33, 101), (64, 4096), (7, 11008)])
def test_unpack_dev_1p6bit_fx_bit_exact(N, K):
    # Alg. 1 (App. F) on the GPU against the closed-form decode of App. E in the oracle
    import torch
    W = si.ternary_weights(np.random.default_rng(N + K + 1), N, K)
    P = oracle.pack3fx(W)
    out = torch.full((N, K), 77, dtype=torch.int8, device="cuda")
    tl.tl_unpack_dev(tl.TL_FMT_1P6BIT_FX, to_dev(P), N, K, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), W)
    # every byte value, not only the 243 the packer produces
    every = np.zeros((256, 16), dtype=np.uint8)
    every[:, 0] = np.arange(256)
    out = torch.full((256, 5), 77, dtype=torch.int8, device="cuda")
    tl.tl_unpack_dev(tl.TL_FMT_1P6BIT_FX, to_dev(every), 256, 5, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.unpack3fx(every, 5))


FX_SHAPES = [(1, 16, 8), (4, 272, 640), (3, 17, 1280), (16, 100, 648), (7, 33, 4096), (16, 4099, 4096),
             (3, 40, 11008), (33, 130, 2048), (2, 5, 17), (5, 129, 4095), (200, 48, 640)]


@pytest.mark.parametrize("M,N,K", FX_SHAPES)
def test_gemm_1p6_fx_matches_oracle(M, N, K):
    # small-M kernel (table filled by Alg. 1) where K % 8 == 0 and M <= 4096, generic kernel otherwise
    import torch
    x, W, g = si.layer(9500 + M + N + K, M, N, K)
    Wp = tl.tl_pack_1p6bit_fx(W)
    assert np.array_equal(Wp, oracle.pack3fx(W))
    xd, wd = to_dev(x.view(np.uint16).view(np.int16)), to_dev(Wp)
    yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
    tl.tl_ternary_gemm_1p6_fx(xd, wd, si.gamma_bits(g), yd, M, N, K)
    torch.cuda.synchronize()
    y = yd.cpu().numpy().view(np.float16)
    assert_close(y, oracle.gemm_packed3fx(x, Wp, g, K), x, g, f"1.6-bit fixed-point code {M}x{N}x{K}")
    # the same weights in the plain base-3 form give the same bits: only the byte code differs
    y3 = run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K)
    assert np.array_equal(y.view(np.uint16), y3.view(np.uint16))


@pytest.mark.parametrize("M", [1, 4, 16])
def test_gemv_1p6_full_size_agrees_with_2bit_path(M):
    # config 5: the same weights through both formats; 512 sampled columns against the oracle
    N, K = 14336, 4096
    x, W, g = si.layer(si.SEEDS["c5"] + M, M, N, K)
    y3 = run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K)
    y2 = run_gemm(x, tl.tl_pack_2bit(W), g, N, K)
    cols = np.sort(np.random.default_rng(3).choice(N, 512, replace=False))
    ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
    assert_close(y3[:, cols], ref, x, g, "1.6-bit full size")
    assert_close(y2[:, cols], ref, x, g, "2-bit full size")
    assert_close(y3, y2.astype(np.float64), x, g, "1.6-bit vs 2-bit")
    # deterministic
    assert np.array_equal(run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K).view(np.uint16), y3.view(np.uint16))


# --- per-group scales --------------------------------------------------------------------

def run_gemm_gs(x, Wp, sc, group, N, K):
    import torch
    M = x.shape[0]
    xd, wd = to_dev(x.view(np.uint16).view(np.int16)), dev_u32(Wp)
    sd = to_dev(sc.view(np.uint16).view(np.int16))
    yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
    tl.tl_ternary_gemm_gs(xd, wd, sd, group, yd, M, N, K)
    torch.cuda.synchronize()
    return yd.cpu().numpy().view(np.float16)


GS_SHAPES = [
    # small-M stream kernel: group % 128 == 0, K % 64 == 0, N % 4 == 0
    (1, 64, 512, 256), (3, 100, 1024, 256), (16, 4096, 4096, 256), (5, 272, 4096, 512), (16, 144, 4096, 1024),
    (7, 48, 4096, 4096), (1, 4100, 4096, 256), (33, 128, 2048, 256), (4, 40, 11008, 256), (2, 64, 8192, 768),
    (300, 64, 1024, 256), (2, 1152, 1344, 256), (1, 14336, 4096, 256),
    # the same kernel with scale units of 128 weights: group % 128 == 0 but not % 256
    (1, 64, 512, 128), (3, 100, 1024, 128), (16, 4096, 4096, 128), (5, 272, 4096, 384), (4, 40, 11008, 128),
    (33, 128, 2048, 128), (2, 1152, 1344, 128), (1, 14336, 4096, 128), (7, 48, 4096, 640), (16, 64, 8192, 1152),
    # plain kernel: any other group (multiple of 16), N or K
    (3, 7, 100, 16), (2, 33, 4096, 64), (5, 6, 4096, 256), (4, 12, 1000, 256),
    (16, 4096, 4096, 64), (17, 300, 4000, 80), (1, 64, 1001, 16), (35, 21, 2047, 32), (3, 30, 4096, 128),
]


@pytest.mark.parametrize("M,N,K,group", GS_SHAPES)
def test_gemm_group_scales_matches_oracle(M, N, K, group):
    rng = np.random.default_rng(7700 + M + N + K + group)
    x, W, _ = si.layer(7600 + M + N + K, M, N, K)
    sc = si.group_scales(rng, (K + group - 1) // group, N)
    Wp = tl.tl_pack_2bit(W)
    y = run_gemm_gs(x, Wp, sc, group, N, K)
    ref = oracle.gemm_packed2_group_scales(x, Wp, sc, group, K)
    assert_close(y, ref, x, float(sc.max()), f"group scales {M}x{N}x{K} / {group}")


def test_gemm_group_scales_equal_scales_reproduce_the_single_gamma_kernel_bits():
    # every scale equal to gamma: the two halves of a slice are scaled apart and added, which is
    # the single-gamma result up to the rounding of that one addition
    M, N, K = 4, 512, 4096
    x, W, g = si.layer(7801, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    sc = np.full((K // 256, N), g, dtype=np.float16)
    y = run_gemm_gs(x, Wp, sc, 256, N, K)
    y1 = run_gemm(x, Wp, g, N, K, tl.TL_PATH_GEMV)
    assert_close(y, y1.astype(np.float64), x, g, "equal scales against the single-gamma kernel")
    assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, "equal scales against the oracle")


# --- seeded random shapes through every dispatch rule --------------------------------------

def _random_shape(rng):
    M = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 31, 32, 33, 64, 70, 130, 300]))
    N = int(rng.choice([1, 3, 4, 15, 16, 17, 100, 256, 272, 513, 1000, 2049]))
    K = int(rng.choice([16, 17, 64, 100, 128, 448, 512, 576, 1024, 2048, 3136, 4096, 4160, 6144, 11008]))
    return M, N, K


def test_random_shapes_single_calls():
    rng = np.random.default_rng(20250623)
    for case in range(36):
        M, N, K = _random_shape(rng)
        x, W, g = si.layer(880000 + case, M, N, K)
        Wp = tl.tl_pack_2bit(W)
        print(f"case {case}: {M}x{N}x{K}", flush=True)
        y = run_gemm(x, Wp, g, N, K)
        assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"random shape {M}x{N}x{K}")


def test_random_grouped_calls():
    import torch
    rng = np.random.default_rng(20250624)
    for call in range(6):
        count = int(rng.integers(2, 21))
        host, dev, jobs, specs = [], [], [], []
        for i in range(count):
            M, N, K = _random_shape(rng)
            x, W, g = si.layer(890000 + 100 * call + i, M, N, K)
            Wp = tl.tl_pack_2bit(W)
            xd, wd = to_dev(x.view(np.int16)), dev_u32(Wp)
            yd = torch.full((M, N), -21555, dtype=torch.int16, device="cuda")
            host.append((x, Wp, g))
            dev.append(yd)
            specs.append((M, N, K))
            jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
        print(f"call {call}: {specs}", flush=True)
        tl.tl_ternary_gemm_grouped(jobs)
        torch.cuda.synchronize()
        for (M, N, K), (x, Wp, g), yd in zip(specs, host, dev):
            y = yd.cpu().numpy().view(np.float16)
            assert_close(y, oracle.gemm_packed2(x, Wp, g, K), x, g, f"random grouped call {call}: {M}x{N}x{K}")


def test_random_shapes_other_formats_and_group_scales():
    rng = np.random.default_rng(20250625)
    for case in range(16):
        M, N, K = _random_shape(rng)
        x, W, g = si.layer(895000 + case, M, N, K)
        print(f"case {case}: {M}x{N}x{K}", flush=True)
        # 1.6-bit, plain base 3
        y3 = run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K)
        assert_close(y3, oracle.gemm(x, W, g), x, g, f"random 1.6-bit {M}x{N}x{K}")
        # per-group scales, group sizes on both sides of the fast kernel's conditions
        group = int(rng.choice([16, 64, 256, 512, 1024]))
        sc = si.group_scales(rng, (K + group - 1) // group, N)
        Wp = tl.tl_pack_2bit(W)
        ys = run_gemm_gs(x, Wp, sc, group, N, K)
        assert_close(ys, oracle.gemm_packed2_group_scales(x, Wp, sc, group, K), x, float(sc.max()),
                     f"random group scales {M}x{N}x{K} / {group}")


def test_probe_kernels_run_and_leave_memory_alone():
    import torch
    n = (1 << 20) + 16
    src = torch.arange(n, dtype=torch.int32, device="cuda")
    dst = torch.zeros(n, dtype=torch.int32, device="cuda")
    sink = torch.full((4,), 7, dtype=torch.int32, device="cuda")
    tl.tl_probe_read(src, n * 4, sink)
    tl.tl_probe_copy(dst, src, n * 4)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert sink.tolist() == [7, 7, 7, 7]          # the fold of 0..n-1 is not the value that triggers the store
    # the matrix-pipe probe: reports its flops, touches nothing but (possibly) the sink
    x = to_dev(si.activations(np.random.default_rng(5), 1, 4096).view(np.int16))
    wp = dev_u32(tl.tl_pack_2bit(si.ternary_weights(np.random.default_rng(6), 4, 4096)))
    fsink = torch.full((4,), 3.0, dtype=torch.float32, device="cuda")
    flops = tl.tl_probe_mfma(x, 4096, wp, 1024, 10, fsink)
    torch.cuda.synchronize()
    assert flops == 256 * 8 * 10 * 8 * 2 * 32 * 32 * 16
    assert fsink.tolist() == [3.0, 3.0, 3.0, 3.0]


def test_init_is_idempotent_and_calls_work_after_it():
    tl.tl_init()
    tl.tl_init()
    x, W, g = si.layer(31337, 3, 272, 4096)
    Wp = tl.tl_pack_2bit(W)
    assert_close(run_gemm(x, Wp, g, 272, 4096), oracle.gemm_packed2(x, Wp, g, 4096), x, g, "after tl_init")


def test_non_finite_activations_stay_in_their_row():
    # a NaN and an infinity in two rows of x: those rows of y are non-finite, every other row is
    # exactly what it is without them
    M, N, K = 5, 272, 4096
    x, W, g = si.layer(4242, M, N, K)
    Wp = tl.tl_pack_2bit(W)
    clean = run_gemm(x, Wp, g, N, K)
    bad = x.copy()
    bad[1, 100] = np.float16(np.nan)
    bad[3, 2000] = np.float16(np.inf)
    y = run_gemm(bad, Wp, g, N, K)
    for m in (0, 2, 4):
        assert np.array_equal(y[m].view(np.uint16), clean[m].view(np.uint16))
    assert not np.isfinite(y[1].astype(np.float32)).any()
    assert not np.isfinite(y[3].astype(np.float32)).any()


# --- the workload configurations under the floor first proposed for the comparison ---------------

def _rms_floor_err(y_gpu, y_ref):
    """max |y_gpu - y_ref| / max(|y_ref|, 1e-2 rms_n(y_ref[m, :])): the relative error with a floor of
    one hundredth of the row's rms, which needs no model of the accumulation; and the plain
    relative error over the entries that are at least as large as the row's rms."""
    yg, yr = y_gpu.astype(np.float64), np.asarray(y_ref, dtype=np.float64)
    rms = np.sqrt(np.mean(yr ** 2, axis=1, keepdims=True))
    e_floor = float(np.max(np.abs(yg - yr) / np.maximum(np.abs(yr), 1e-2 * rms)))
    big = np.abs(yr) >= rms
    e_big = float(np.max(np.abs(yg - yr)[big] / np.abs(yr)[big])) if big.any() else 0.0
    return e_floor, e_big


def _sample_cols(N, n, seed):
    if N <= n:
        return np.arange(N)
    cols = np.sort(np.random.default_rng(seed).choice(N, n, replace=False))
    cols[-1] = N - 1
    return cols


Q6_CASES = ([("c1", "2bit", 1, 2048, 2048)] +
            [("c2", "2bit", M, N, 4096) for N in (4096, 14336) for M in (1, 16)] +
            [("c3", "2bit", M, si.SHAPES[n][1], si.SHAPES[n][0]) for n in si.BLOCK_SHAPES for M in (1, 16, 64)] +
            [("c4", "2bit", 256, 14336, 4096)] +
            [("c5", "1p6", M, N, 4096) for N in (4096, 14336) for M in (1, 16)])


@pytest.mark.parametrize("cfg,fmt,M,N,K", Q6_CASES)
def test_workload_configs_under_the_rms_floor(cfg, fmt, M, N, K):
    # Every configuration of the workload definition with the iid weights it names, judged by a
    # floor that does not depend on the kernel: 2e-3 relative to max(|y|, 1e-2 rms of the row), and
    # plain 2e-3 wherever |y| >= rms.  (The tolerance of parity.py models fp32 accumulation instead
    # and coincides with this floor at K = 4096; this test shows that the model is not what lets
    # these cases pass.)  Large N: 384 sampled output columns.
    x, W, g = si.layer(si.SEEDS[cfg] + 7 * M + N % 1000, M, N, K)
    cols = _sample_cols(N, 384, N + M)
    ref = oracle.gemm(x, np.ascontiguousarray(W[cols]), g)
    if fmt == "2bit":
        y = run_gemm(x, tl.tl_pack_2bit(W), g, N, K)
    else:
        y = run_gemm3(x, tl.tl_pack_1p6bit(W), g, N, K)
    e_floor, e_big = _rms_floor_err(y[:, cols], ref)
    assert e_floor <= REL_TOL, f"{cfg} {fmt} M={M} {K}->{N}: {e_floor:.3e} with the rms floor"
    assert e_big <= REL_TOL, f"{cfg} {fmt} M={M} {K}->{N}: {e_big:.3e} on entries >= rms"
