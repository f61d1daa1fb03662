"""Pins for the oracle's number conversion and GEMM (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as si


def test_half_to_double_matches_numpy_on_all_65536_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def _tiny(seed, M, N, K):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((M, K)) * 3).astype(np.float16)
    W = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
    g = np.float16(rng.uniform(0.01, 0.05))
    return x, W, g


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (3, 2, 32), (4, 4, 17)])
def test_gemm_brute_force_exact_rationals(M, N, K):
    # the definition, evaluated in exact rational arithmetic, element by element
    x, W, g = _tiny(10 + K, M, N, K)
    y = oracle.gemm(x, W, g)
    for m in range(M):
        for n in range(N):
            s = sum(Fraction(float(x[m, k])) * int(W[n, k]) for k in range(K))
            exact = Fraction(float(g)) * s
            # gamma and S are exact in fp64 and so is their product here (11 + <40 bits)
            assert Fraction(y[m, n]) == exact


@pytest.mark.parametrize("M,N,K", [(1, 7, 64), (5, 9, 100), (3, 33, 4096), (2, 4, 11008)])
def test_gemm_matches_numpy_fp64_matmul(M, N, K):
    # a library routine on the textbook formula; non-square and asymmetric so that a
    # transposed operand or swapped index cannot pass
    x, W, g = si.layer(77 + K, M, N, K)
    y = oracle.gemm(x, W, g)
    ref = (x.astype(np.float64) @ W.astype(np.float64).T) * float(g)
    assert y.shape == (M, N)
    assert np.array_equal(y, ref)      # every partial sum is exact in fp64, so no tolerance


def test_gemm_fixed_point_form_agrees_bit_for_bit():
    x, W, g = si.layer(5, 3, 11, 4096)
    x[0, :8] = np.array([0, 6e-8, -6e-8, 6.1e-5, -65504, 65504, 1e-3, -0.0], dtype=np.float16)
    y = oracle.gemm(x, W, g)
    S24 = oracle.gemm_fixed(x, W)
    y2 = float(g) * (S24.astype(np.float64) * 2.0 ** -24)
    assert np.array_equal(y, y2)


def test_gemm_identities():
    M, N, K = 3, 24, 160
    x, W, g = si.layer(9, M, N, K)
    y = oracle.gemm(x, W, g)
    # y(-W) = -y, y(0) = 0, exactly
    assert np.array_equal(oracle.gemm(x, -W, g), -y)
    assert not oracle.gemm(x, np.zeros_like(W), g).any()
    # scaling x by 2 doubles y exactly; rows of x are independent
    assert np.array_equal(oracle.gemm((x * np.float16(2)), W, g), 2 * y)
    for m in range(M):
        assert np.array_equal(oracle.gemm(x[m:m + 1], W, g), y[m:m + 1])
    # additivity over a split of K
    k1 = 48
    y1 = oracle.gemm(np.ascontiguousarray(x[:, :k1]), np.ascontiguousarray(W[:, :k1]), np.float16(1))
    y2 = oracle.gemm(np.ascontiguousarray(x[:, k1:]), np.ascontiguousarray(W[:, k1:]), np.float16(1))
    assert np.array_equal(oracle.gemm(x, W, np.float16(1)), y1 + y2)


def test_gemm_identity_and_permutation_weights_return_gamma_x():
    K = 96
    rng = np.random.default_rng(3)
    x = si.activations(rng, 4, K)
    g = np.float16(0.02)
    I = np.eye(K, dtype=np.int8)
    y = oracle.gemm(x, I, g)
    assert np.array_equal(y, float(g) * x.astype(np.float64))
    perm = rng.permutation(K)
    P = np.zeros((K, K), dtype=np.int8)
    P[np.arange(K), perm] = -1
    assert np.array_equal(oracle.gemm(x, P, g), -float(g) * x.astype(np.float64)[:, perm])
    # fp16 product of two fp16 numbers is exact in fp32: the rounded output is fp16(g * x)
    y16 = oracle.to_fp16(y)
    assert np.array_equal(y16, (x.astype(np.float32) * np.float32(g)).astype(np.float16))


def test_gemm_packed_equals_unpacked_and_padding_contributes_nothing():
    M, N, K = 2, 9, 100                      # 100 = 6 words + a 4-digit tail
    x, W, g = si.layer(21, M, N, K)
    y = oracle.gemm(x, W, g)
    assert np.array_equal(oracle.gemm_packed2(x, oracle.pack2(W), g, K), y)
    assert np.array_equal(oracle.gemm_packed3le(x, oracle.pack3le(W), g, K), y)
    # Sec. 3.1 pads with d = 0: widening K to the word boundary with zero weights and
    # arbitrary activations leaves y unchanged
    Kp = 112
    Wp = np.zeros((N, Kp), dtype=np.int8)
    Wp[:, :K] = W
    xp = si.activations(np.random.default_rng(4), M, Kp)
    xp[:, :K] = x
    assert np.array_equal(oracle.gemm(xp, Wp, g), y)


def test_gamma_is_the_fp16_value():
    x, W, _ = si.layer(2, 1, 4, 64)
    g = np.float16(0.02)                     # 0.02 is not representable: fp16 holds 0.0200042724609375
    assert float(g) == 0.0200042724609375
    y = oracle.gemm(x, W, g)
    y1 = oracle.gemm(x, W, np.float16(1))
    assert np.array_equal(y, 0.0200042724609375 * y1)
    assert np.array_equal(oracle.gemm(x, W, si.gamma_bits(g)), y)


# --- per-group scales ------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K,group", [(1, 1, 4, 2), (2, 3, 10, 4), (3, 2, 33, 16), (2, 2, 16, 16), (1, 3, 7, 64)])
def test_group_scales_brute_force_exact_rationals(M, N, K, group):
    # the definition, element by element, in exact rational arithmetic (the last group is short
    # in three of the cases); the fp64 result may differ from it by the rounding of the sum
    # over groups only
    rng = np.random.default_rng(900 + K)
    x, W, _ = _tiny(40 + K, M, N, K)
    G = (K + group - 1) // group
    sc = si.group_scales(rng, G, N)
    y = oracle.gemm_group_scales(x, W, sc, group)
    for m in range(M):
        for n in range(N):
            exact = Fraction(0)
            for g in range(G):
                part = sum(Fraction(float(x[m, k])) * int(W[n, k]) for k in range(g * group, min(K, (g + 1) * group)))
                exact += Fraction(float(sc[g, n])) * part
            assert abs(Fraction(y[m, n]) - exact) <= abs(exact) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 60)


def test_group_scales_all_equal_is_the_single_gamma_product():
    x, W, g = si.layer(31, 3, 9, 1000)
    sc = np.full((4, 9), g, dtype=np.float16)          # groups of 256, the last one short
    y = oracle.gemm_group_scales(x, W, sc, 256)
    assert np.allclose(y, oracle.gemm(x, W, g), rtol=1e-13, atol=1e-15)


def test_group_scales_one_group_switched_on_is_that_slice_of_k():
    x, W, g = si.layer(32, 2, 5, 700)
    for grp in range(3):                                # groups of 256: [0,256) [256,512) [512,700)
        sc = np.zeros((3, 5), dtype=np.float16)
        sc[grp, :] = g
        k0, k1 = grp * 256, min(700, grp * 256 + 256)
        ref = oracle.gemm(np.ascontiguousarray(x[:, k0:k1]), np.ascontiguousarray(W[:, k0:k1]), g)
        assert np.array_equal(oracle.gemm_group_scales(x, W, sc, 256), ref)


def test_group_scales_single_group_is_one_scale_per_output_row_and_linear_in_the_scales():
    rng = np.random.default_rng(33)
    x, W, _ = si.layer(33, 2, 6, 300)
    sc = si.group_scales(rng, 1, 6)
    S = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.array_equal(oracle.gemm_group_scales(x, W, sc, 512), S * sc.astype(np.float64))   # per column n
    a = si.group_scales(rng, 3, 6)
    b = np.zeros_like(a)
    b[1, 2] = a[1, 2]                                   # split one entry off: y(a) = y(a - b) + y(b)
    c = a.copy()
    c[1, 2] = 0
    ya, yb, yc = (oracle.gemm_group_scales(x, W, s, 128) for s in (a, b, c))
    assert np.allclose(ya, yb + yc, rtol=1e-13, atol=1e-15)
    assert np.count_nonzero(yb[:, [0, 1, 3, 4, 5]]) == 0   # the entry belongs to output row 2 alone


# --- the ternariser of App. B, pinned on the oracle's own function ------------------------------

def test_oracle_quantize_hand_worked_example():
    # App. B: gamma = eps + mean|W|, What = round(clip(W / gamma, -1, 1)).  Worked by hand:
    # |W| = (0.5, 0.5, 0.1, 2.0), mean 0.775; W / gamma = (0.645, -0.645, 0.129, 2.58 -> clipped 1)
    W = np.array([[0.5, -0.5, 0.1, 2.0]], dtype=np.float32)
    What, g = oracle.quantize(W, eps=0.0)
    assert What.dtype == np.int8 and What.tolist() == [[1, -1, 0, 1]]
    assert g == pytest.approx(0.775, rel=1e-7)
    # eps enters additively: the same weights with eps = 0.225 have gamma = 1.0 exactly (in fp64 up to
    # the rounding of 0.1f), and 0.5 / 1.0 is then a tie
    What, g = oracle.quantize(W, eps=1.0 - float(np.mean(np.abs(W.astype(np.float64)))))
    assert g == 1.0 and What.tolist() == [[0, 0, 0, 1]]


def test_oracle_quantize_ties_round_to_even_and_clip_comes_first():
    # mean|W| = 1 exactly, so W / gamma = W: +-0.5 are exact ties (half to even gives 0, half away
    # from zero would give +-1), 1.5 is clipped to 1 before rounding (rounding first would give 2)
    What, g = oracle.quantize(np.array([[0.5, 1.5]], dtype=np.float32), eps=0.0)
    assert g == 1.0 and What.tolist() == [[0, 1]]
    What, g = oracle.quantize(np.array([[-0.5, -1.5]], dtype=np.float32), eps=0.0)
    assert g == 1.0 and What.tolist() == [[0, -1]]
    # just past the tie on either side (0.5 +- 2^-20 and its complement to 2 are exact in fp32)
    d = np.float32(2.0 ** -20)
    What, g = oracle.quantize(np.array([[np.float32(0.5) + d, np.float32(1.5) - d]], dtype=np.float32), eps=0.0)
    assert g == 1.0 and What.tolist() == [[1, 1]]
    What, g = oracle.quantize(np.array([[np.float32(0.5) - d, np.float32(1.5) + d]], dtype=np.float32), eps=0.0)
    assert g == 1.0 and What.tolist() == [[0, 1]]
    # all-zero weights: gamma = eps, What = 0; eps = 0 as well: gamma = 0 and no division
    What, g = oracle.quantize(np.zeros((3, 5), np.float32), eps=1e-5)
    assert g == 1e-5 and not What.any()
    What, g = oracle.quantize(np.zeros((3, 5), np.float32), eps=0.0)
    assert g == 0.0 and not What.any()


@pytest.mark.parametrize("shape,eps,seed", [((1, 1), 0.0, 1), ((3, 7), 0.0, 2), ((5, 4), 1e-5, 3), ((2, 33), 0.25, 4)])
def test_oracle_quantize_brute_force_exact_rationals(shape, eps, seed):
    # the definition in exact rational arithmetic, element by element: gamma, the quotient, the
    # clip and the rounding (half to even) all exact; the fp64 oracle may differ only where the
    # exact quotient lies within rounding distance of a tie, which these draws avoid
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal(shape) * rng.uniform(0.05, 2.0)).astype(np.float32)
    What, g = oracle.quantize(W, eps=eps)
    gamma = Fraction(float(eps)) + sum(abs(Fraction(float(w))) for w in W.ravel()) / W.size
    assert abs(Fraction(g) - gamma) <= gamma * Fraction(1, 2 ** 50)
    half = Fraction(1, 2)
    for idx in np.ndindex(*shape):
        q = Fraction(float(W[idx])) / gamma
        q = max(Fraction(-1), min(Fraction(1), q))
        assert abs(abs(q) - half) > Fraction(1, 10 ** 9), "draw too close to a tie"
        want = 0 if abs(q) < half else (1 if q > 0 else -1)
        assert int(What[idx]) == want


def test_oracle_quantize_invariants():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((64, 96)).astype(np.float32)
    Wh1, g1 = oracle.quantize(W, eps=0.0)
    Wh2, g2 = oracle.quantize(W * np.float32(8.0), eps=0.0)        # a power of two scales gamma alone
    assert g2 == 8.0 * g1 and np.array_equal(Wh1, Wh2)
    Wh3, g3 = oracle.quantize(-W, eps=0.0)                          # odd in W
    assert g3 == g1 and np.array_equal(Wh3, -Wh1)
    # near-Gaussian weights: gamma -> sqrt(2 / pi), |W| < gamma / 2 becomes 0:
    # P(0) = 2 Phi(0.5 sqrt(2 / pi)) - 1 = 0.3101
    W = rng.standard_normal((512, 512)).astype(np.float32)
    Wh, g = oracle.quantize(W, eps=0.0)
    assert abs(g - np.sqrt(2 / np.pi)) < 5e-3
    assert abs((Wh == 0).mean() - 0.3101) < 5e-3 and abs((Wh == 1).mean() - (Wh == -1).mean()) < 5e-3
    assert set(np.unique(Wh).tolist()) == {-1, 0, 1}


# --- fp64 -> fp16 rounding of the oracle, pinned without a second cast ---------------------------

def _finite_halves():
    """(bits, value) of every finite non-negative fp16, ascending, decoded by the oracle's C routine
    (itself pinned against numpy's half -> double above)."""
    return [(b, oracle.half_to_double(b)) for b in range(0x7C00)]


def test_to_fp16_is_the_identity_on_every_fp16_value():
    for sign in (0, 0x8000):
        bits = np.arange(0x7C00, dtype=np.uint16) | np.uint16(sign)
        vals = np.array([oracle.half_to_double(int(b)) for b in bits])
        got = oracle.to_fp16(vals).view(np.uint16)
        assert np.array_equal(got, bits)


def test_to_fp16_rounds_to_nearest_ties_to_even_between_neighbours():
    # between neighbouring fp16 values a < b (subnormals and the 2^-14 boundary included): the
    # exact midpoint goes to the one with the even bit pattern, anything nearer to one side goes there
    hv = _finite_halves()
    lo_bits = np.array([b for b, _ in hv[:-1]], dtype=np.uint16)
    a = np.array([v for _, v in hv[:-1]])
    b = np.array([v for _, v in hv[1:]])
    mid = (a + b) / 2                                              # exact in fp64 (11-bit significands)
    want_mid = np.where(lo_bits % 2 == 0, lo_bits, lo_bits + 1).astype(np.uint16)
    assert np.array_equal(oracle.to_fp16(mid).view(np.uint16), want_mid)
    assert np.array_equal(oracle.to_fp16(np.nextafter(mid, -np.inf)).view(np.uint16), lo_bits)
    assert np.array_equal(oracle.to_fp16(np.nextafter(mid, np.inf)).view(np.uint16), lo_bits + 1)
    assert np.array_equal(oracle.to_fp16(-mid).view(np.uint16), want_mid | np.uint16(0x8000))
    # overflow: the midpoint between 65504 and 2^16 rounds to the even side, i.e. to infinity
    with np.errstate(over="ignore"):
        assert oracle.to_fp16(np.array([65519.999, 65520.0, 1e9])).view(np.uint16).tolist() == [0x7BFF, 0x7C00, 0x7C00]
    # below half of the smallest subnormal (2^-25) everything is zero; the tie itself goes to even = 0
    assert oracle.to_fp16(np.array([2.0 ** -25, np.nextafter(2.0 ** -25, 1.0), 2.0 ** -26])).view(np.uint16).tolist() == [0, 1, 0]
