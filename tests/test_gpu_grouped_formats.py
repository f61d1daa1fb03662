"""GPU parity of the grouped entry points for the 1.6-bit forms and for per-group scales: several
GEMMs per launch, against the CPU oracle and against the single calls they stand for."""
import numpy as np
import pytest

import oracle
import paper_2506_23025_amd as tl
import synth_inputs as si
from parity import assert_close, dev_u32, to_dev

pytestmark = pytest.mark.gpu

POISON = -21555


def _pack3(W, fmt):
    return tl.tl_pack_1p6bit(W) if fmt == tl.TL_FMT_1P6BIT else tl.tl_pack_1p6bit_fx(W)


def _ref3(x, Wp, g, K, fmt):
    return oracle.gemm_packed3le(x, Wp, g, K) if fmt == tl.TL_FMT_1P6BIT else oracle.gemm_packed3fx(x, Wp, g, K)


def _single3(xd, wd, g, M, N, K, fmt):
    import torch
    yd = torch.full((M, N), POISON, dtype=torch.int16, device="cuda")
    (tl.tl_ternary_gemm_1p6 if fmt == tl.TL_FMT_1P6BIT else tl.tl_ternary_gemm_1p6_fx)(xd, wd, si.gamma_bits(g), yd, M, N, K)
    torch.cuda.synchronize()
    return yd.cpu().numpy().view(np.float16)


def _run_1p6_grouped(specs, seed, fmt, check_single=True, sample=None):
    import torch
    host, dev, jobs = [], [], []
    for i, (M, N, K) in enumerate(specs):
        x, W, g = si.layer(seed + i, M, N, K)
        Wp = _pack3(W, fmt)
        xd, wd = to_dev(x.view(np.int16)), to_dev(Wp)
        yd = torch.full((M, N), POISON, dtype=torch.int16, device="cuda")
        host.append((x, W, Wp, g))
        dev.append((xd, wd, yd))
        jobs.append((xd, wd, si.gamma_bits(g), yd, M, N, K))
    tl.tl_ternary_gemm_1p6_grouped(jobs, fmt)
    torch.cuda.synchronize()
    for (M, N, K), (x, W, Wp, g), (xd, wd, yd) in zip(specs, host, dev):
        y = yd.cpu().numpy().view(np.float16)
        what = f"1.6-bit grouped fmt {fmt} {M}x{N}x{K}"
        if sample is None or N <= sample:
            assert_close(y, _ref3(x, Wp, g, K, fmt), x, g, what)
        else:
            cols = np.sort(np.random.default_rng(3).choice(N, sample, replace=False))
            assert_close(y[:, cols], oracle.gemm(x, np.ascontiguousarray(W[cols]), g), x, g, what + " sampled")
        if check_single:
            # same kernel body, same order of summation: the grouped call and the single call agree bit for bit
            assert np.array_equal(y.view(np.uint16), _single3(xd, wd, g, M, N, K, fmt).view(np.uint16)), what


@pytest.mark.parametrize("fmt", [tl.TL_FMT_1P6BIT, tl.TL_FMT_1P6BIT_FX])
def test_1p6_grouped_mixed_bag(fmt):
    # shapes that share launches (K % 8 == 0, one pass), N not a multiple of 16 or 4, M above 16, a K
    # too long for one pass (runs alone), a K the fast kernel cannot take (plain kernel), the longest
    # K of one pass with a ragged last slice, a single slice
    specs = [(1, 4096, 4096), (16, 1000, 1024), (3, 272, 11008), (40, 130, 512), (2, 33, 100),
             (8, 2050, 4096), (200, 96, 256), (5, 48, 64), (1, 4099, 4480), (7, 17, 4488), (2, 640, 640)]
    _run_1p6_grouped(specs, 11000, fmt)


@pytest.mark.parametrize("fmt", [tl.TL_FMT_1P6BIT, tl.TL_FMT_1P6BIT_FX])
def test_1p6_grouped_decode_sweep(fmt):
    # the benchmark's step in the 1.6-bit form: ten GEMMs in one launch, sampled columns of the large ones
    specs = [(M, N, 4096) for N in (4096, 14336) for M in (1, 2, 4, 8, 16)]
    _run_1p6_grouped(specs, 11100, fmt, check_single=False, sample=256)


def test_1p6_grouped_more_row_blocks_than_one_launch_holds():
    # 38 + 4 + 1 blocks of 16 rows: two launches, the second starting inside the first job
    _run_1p6_grouped([(600, 48, 1280), (50, 272, 640), (1, 16, 8)], 11200, tl.TL_FMT_1P6BIT)


def test_1p6_grouped_one_job_equals_the_single_call():
    _run_1p6_grouped([(4, 14336, 4096)], 11300, tl.TL_FMT_1P6BIT, sample=256)


def test_1p6_grouped_random_calls():
    rng = np.random.default_rng(11400)
    for call in range(6):
        specs = []
        for _ in range(int(rng.integers(1, 7))):
            K = int(rng.choice([8, 64, 640, 648, 1024, 2048, 4096, 4480, 5120, 100]))
            specs.append((int(rng.integers(1, 50)), int(rng.integers(1, 600)), K))
        _run_1p6_grouped(specs, 11400 + 10 * call, tl.TL_FMT_1P6BIT_FX if call % 2 else tl.TL_FMT_1P6BIT)


def test_1p6_grouped_empty_and_errors():
    L = tl.raw()
    assert L.tl_ternary_gemm_1p6_grouped(None, 0, tl.TL_FMT_1P6BIT, None) == tl.TL_OK
    assert L.tl_ternary_gemm_1p6_grouped(None, 2, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_NULL
    ok = tl.make_jobs([(16, 16, 0, 32, 1, 16, 64)])
    assert L.tl_ternary_gemm_1p6_grouped(ok, 1, tl.TL_FMT_2BIT, None) == tl.TL_ERR_VALUE
    assert L.tl_ternary_gemm_1p6_grouped(ok, 1, 7, None) == tl.TL_ERR_VALUE
    assert L.tl_ternary_gemm_1p6_grouped(ok, -1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_SHAPE
    bad = tl.make_jobs([(16, 16, 0, 0, 1, 16, 64)])
    assert L.tl_ternary_gemm_1p6_grouped(bad, 1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_NULL
    bad = tl.make_jobs([(16, 16, 0, 24, 1, 16, 64)])
    assert L.tl_ternary_gemm_1p6_grouped(bad, 1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_ALIGN
    bad = tl.make_jobs([(16, 16, 0, 32, 1, 0, 64)])
    assert L.tl_ternary_gemm_1p6_grouped(bad, 1, tl.TL_FMT_1P6BIT, None) == tl.TL_ERR_SHAPE


# ------------------------------------------------------------------ per-group scales

def _run_gs_grouped(specs, seed, check_single=True, sample=None):
    import torch
    host, dev, jobs = [], [], []
    for i, (M, N, K, group) in enumerate(specs):
        rng = np.random.default_rng(seed + 100 + i)
        x, W, _ = si.layer(seed + i, M, N, K)
        sc = si.group_scales(rng, (K + group - 1) // group, N)
        Wp = tl.tl_pack_2bit(W)
        xd, wd, sd = to_dev(x.view(np.int16)), dev_u32(Wp), to_dev(sc.view(np.int16))
        yd = torch.full((M, N), POISON, dtype=torch.int16, device="cuda")
        host.append((x, W, Wp, sc))
        dev.append((xd, wd, sd, yd))
        jobs.append((xd, wd, sd, group, yd, M, N, K))
    tl.tl_ternary_gemm_gs_grouped(jobs)
    torch.cuda.synchronize()
    for (M, N, K, group), (x, W, Wp, sc), (xd, wd, sd, yd) in zip(specs, host, dev):
        y = yd.cpu().numpy().view(np.float16)
        what = f"group scales grouped {M}x{N}x{K} / {group}"
        if sample is None or N <= sample:
            assert_close(y, oracle.gemm_packed2_group_scales(x, Wp, sc, group, K), x, float(sc.max()), what)
        else:
            cols = np.sort(np.random.default_rng(3).choice(N, sample, replace=False))
            ref = oracle.gemm_packed2_group_scales(x, np.ascontiguousarray(Wp[cols]), np.ascontiguousarray(sc[:, cols]), group, K)
            assert_close(y[:, cols], ref, x, float(sc.max()), what + " sampled")
        if check_single:
            y1 = torch.full((M, N), POISON, dtype=torch.int16, device="cuda")
            tl.tl_ternary_gemm_gs(xd, wd, sd, group, y1, M, N, K)
            torch.cuda.synchronize()
            assert np.array_equal(y.view(np.uint16), y1.cpu().numpy().view(np.uint16)), what


def test_gs_grouped_mixed_bag():
    # both kinds of scale unit (multiples of 256, odd multiples of 128), several passes over K, M above
    # 16, N not a multiple of 16, and jobs the stream kernel does not take (group 64, N % 4 != 0)
    specs = [(1, 4096, 4096, 256), (16, 1000, 1024, 128), (3, 272, 11008, 256), (40, 132, 512, 256),
             (2, 33, 4096, 256), (8, 2052, 4096, 384), (5, 48, 4096, 64), (4, 40, 11008, 128),
             (2, 64, 8192, 768), (7, 48, 4096, 4096), (1, 64, 512, 128)]
    _run_gs_grouped(specs, 12000)


@pytest.mark.parametrize("group", [256, 128])
def test_gs_grouped_decode_sweep(group):
    specs = [(M, N, 4096, group) for N in (4096, 14336) for M in (1, 2, 4, 8, 16)]
    _run_gs_grouped(specs, 12100 + group, check_single=False, sample=256)


def test_gs_grouped_more_row_blocks_than_one_launch_holds():
    _run_gs_grouped([(600, 48, 1024, 256), (50, 272, 512, 256), (1, 16, 64, 128)], 12200)


def test_gs_grouped_block_with_long_k():
    # the four linears of a block with per-group scales: K = 4096 and K = 11008 (several passes) in one call
    specs = [(4, 12288, 4096, 256), (4, 4096, 4096, 256), (4, 22016, 4096, 256), (4, 4096, 11008, 256)]
    _run_gs_grouped(specs, 12300, check_single=False, sample=192)


def test_gs_grouped_runs_too_long_for_one_launch_go_out_job_by_job():
    # two jobs with two passes over K (K = 4608) and 6250 tiles each: in one launch a workgroup's run
    # would not fit the LDS that keeps its sums between the passes, so the jobs are launched one by one
    import torch
    M, N, K, group = 2, 100000, 4608, 256
    rng = np.random.default_rng(12500)
    jobs, keep = [], []
    for i in range(2):
        W = si.ternary_weights(rng, N, K)
        x = si.activations(rng, M, K)
        sc = si.group_scales(rng, K // group, N)
        Wp = tl.tl_pack_2bit(W)
        cols = np.sort(rng.choice(N, 96, replace=False))
        ref = oracle.gemm_packed2_group_scales(x, np.ascontiguousarray(Wp[cols]), np.ascontiguousarray(sc[:, cols]), group, K)
        xd, wd, sd = to_dev(x.view(np.int16)), dev_u32(Wp), to_dev(sc.view(np.int16))
        yd = torch.full((M, N), POISON, dtype=torch.int16, device="cuda")
        jobs.append((xd, wd, sd, group, yd, M, N, K))
        keep.append((x, sc, cols, ref, yd))
        del W, Wp
    tl.tl_ternary_gemm_gs_grouped(jobs)
    torch.cuda.synchronize()
    for x, sc, cols, ref, yd in keep:
        y = yd.cpu().numpy().view(np.float16)
        # a tile that was never written would leave 16 neighbouring columns at the poison value (a
        # genuine output may equal that bit pattern here and there)
        hit = (y.view(np.int16) == POISON)
        assert not (hit[:, :-1] & hit[:, 1:]).any()
        assert_close(y[:, cols], ref, x, float(sc.max()), "group scales grouped, job by job")


def test_gs_grouped_random_calls():
    rng = np.random.default_rng(12400)
    for call in range(6):
        specs = []
        for _ in range(int(rng.integers(1, 7))):
            K = int(rng.choice([64, 512, 1024, 2048, 4096, 8192, 1344, 1000]))
            group = int(rng.choice([16, 64, 128, 256, 384, 512]))
            specs.append((int(rng.integers(1, 50)), 4 * int(rng.integers(1, 150)) + int(rng.integers(0, 2)), K, group))
        _run_gs_grouped(specs, 12400 + 10 * call)


def test_gs_grouped_empty_and_errors():
    L = tl.raw()
    assert L.tl_ternary_gemm_gs_grouped(None, 0, None) == tl.TL_OK
    assert L.tl_ternary_gemm_gs_grouped(None, 2, None) == tl.TL_ERR_NULL
    bad = tl.make_gs_jobs([(16, 16, 0, 256, 32, 1, 16, 64)])
    assert L.tl_ternary_gemm_gs_grouped(bad, 1, None) == tl.TL_ERR_NULL
    bad = tl.make_gs_jobs([(16, 16, 24, 256, 32, 1, 16, 64)])
    assert L.tl_ternary_gemm_gs_grouped(bad, 1, None) == tl.TL_ERR_ALIGN
    bad = tl.make_gs_jobs([(16, 16, 32, 24, 48, 1, 16, 64)])
    assert L.tl_ternary_gemm_gs_grouped(bad, 1, None) == tl.TL_ERR_SHAPE
    assert L.tl_ternary_gemm_gs_grouped(bad, 5000, None) == tl.TL_ERR_SHAPE
