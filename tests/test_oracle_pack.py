"""Pins for the oracle's packing / unpacking routines (CPU only).

Each test checks the oracle against something that is not the oracle: values
derived by hand from the printed formulas (tests/golden), numpy's positional
base conversion, exhaustive enumeration, and the statements of Theorem 1.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            digits = [int(t) for t in parts[0].split(",")]
            out.append((digits, parts[1:]))
    return out


# ------------------------------------------------------------------ Sec. 3.1

@pytest.mark.parametrize("digits,rest", _rows("pack2_words.txt"))
def test_pack2_golden_words(digits, rest):
    word = int(rest[0], 16)
    got = oracle.pack2_seq(digits, k=16)
    assert len(got) == 1 and int(got[0]) == word
    # the matrix form packs a row the same way
    got_m = oracle.pack2(np.array([digits], dtype=np.int8))
    assert got_m.shape == (1, 1) and int(got_m[0, 0]) == word


def test_pack2_digits_are_base4_digits_of_the_word():
    # Sec. 3.1: b = sum_j d'_j 4^j, so numpy's base-4 expansion of b, read from the
    # least significant end, must give back d' = d + 1.
    rng = np.random.default_rng(1)
    for _ in range(200):
        d = rng.integers(-1, 2, size=16).astype(np.int8)
        b = int(oracle.pack2_seq(d, 16)[0])
        rep = np.base_repr(b, 4).rjust(16, "0")[::-1]
        assert [int(c) - 1 for c in rep] == d.tolist()


def test_pack2_k4_is_the_tq2_byte_and_four_bytes_make_the_word():
    # App. F (TQ2): q_packed = q0 + 4 q1 + 16 q2 + 64 q3 is the k = 4 instance; four such
    # bytes read little-endian are the k = 16 word ("each 32-bit integer encodes 16 values").
    rng = np.random.default_rng(2)
    d = rng.integers(-1, 2, size=16).astype(np.int8)
    q = d.astype(np.int64) + 1
    by = [int(q[4 * i] + 4 * q[4 * i + 1] + 16 * q[4 * i + 2] + 64 * q[4 * i + 3]) for i in range(4)]
    k4 = oracle.pack2_seq(d, k=4)
    assert [int(v) for v in k4] == by
    word = int(oracle.pack2_seq(d, k=16)[0])
    assert word == int.from_bytes(bytes(by), "little")


def test_pack2_block_boundaries_and_order():
    # element 16 i + j must land in word i, bits [2j+1:2j]
    for idx in (0, 1, 15, 16, 17, 31, 32, 47):
        d = np.zeros(48, dtype=np.int8)
        d[idx] = 1
        words = oracle.pack2_seq(d, 16)
        for i in range(3):
            expect = 0x55555555 + ((1 << (2 * (idx % 16))) if i == idx // 16 else 0)
            assert int(words[i]) == expect


def test_unpack2_roundtrip_exhaustive_half_word():
    # all 3^8 patterns in the low half-word, zeros elsewhere; then the same in the high half
    pats = np.array(list(itertools.product((-1, 0, 1), repeat=8)), dtype=np.int8)
    for half in (0, 1):
        W = np.zeros((len(pats), 16), dtype=np.int8)
        W[:, 8 * half:8 * half + 8] = pats
        P = oracle.pack2(W)
        assert len(np.unique(P)) == len(pats)            # injective
        assert np.array_equal(oracle.unpack2(P, 16), W)  # U(P(D)) = D


@pytest.mark.parametrize("K", [1, 5, 15, 16, 17, 31, 33, 64, 100, 4096])
def test_unpack2_roundtrip_random_and_ragged(K):
    rng = np.random.default_rng(K)
    W = rng.integers(-1, 2, size=(7, K)).astype(np.int8)
    P = oracle.pack2(W)
    assert P.shape == (7, (K + 15) // 16)
    assert np.array_equal(oracle.unpack2(P, K), W)
    # padding digits of the last word are all 1 (weight 0)
    if K % 16:
        tail = P[:, -1] >> np.uint32(2 * (K % 16))
        assert np.all(tail == (0x55555555 >> (2 * (K % 16))))


def test_pack2_rejects_bad_digit_and_unpack2_rejects_code3():
    with pytest.raises(ValueError):
        oracle.pack2(np.array([[0, 2, 0]], dtype=np.int8))
    with pytest.raises(ValueError):
        oracle.unpack2(np.array([[0x55555557]], dtype=np.uint32), 16)


# ----------------------------------------------- Sec. 3.2 / App. E / App. F

ALL5 = np.array(list(itertools.product((-1, 0, 1), repeat=5)), dtype=np.int8)


@pytest.mark.parametrize("digits,rest", _rows("fx_k5p8_bytes.txt"))
def test_fx_golden_bytes(digits, rest):
    assert oracle.pack_fx_block(digits, 5, 8) == int(rest[1])


def test_fx_theorem1_lossless_when_2p_exceeds_3k():
    # Theorem 1, sufficiency, exhaustively for (k, p) = (5, 8) and two more admissible pairs
    for k, p in ((5, 8), (3, 5), (2, 4), (6, 10)):
        seen = set()
        for d in itertools.product((-1, 0, 1), repeat=k):
            b = oracle.pack_fx_block(d, k, p)
            assert 0 <= b <= 2 ** p - 1
            seen.add(b)
            assert oracle.unpack_fx_div_block(b, k, p).tolist() == list(d)
        assert len(seen) == 3 ** k                       # corollary: injective


def test_fx_theorem1_necessity_collides_when_2p_below_3k():
    # Theorem 1, necessity: 2^7 < 3^5, so P cannot be injective and some block decodes wrongly
    codes = [oracle.pack_fx_block(d, 5, 7) for d in ALL5]
    assert len(set(codes)) < 243
    wrong = sum(oracle.unpack_fx_div_block(b, 5, 7).tolist() != d.tolist()
                for b, d in zip(codes, ALL5))
    assert wrong > 0


def test_fx_bytes_span_0_to_255_and_preserve_order():
    codes = [oracle.pack_fx_block(d, 5, 8) for d in ALL5]   # ALL5 is in increasing N order
    assert codes[0] == 0 and codes[-1] == 255
    assert all(a < b for a, b in zip(codes, codes[1:]))
    # floor((a + t - 1) / t) is ceil(a / t): the byte is ceil(256 N / 243)
    assert codes == [-(-(256 * n) // 243) for n in range(243)]


def test_fx_alg1_equals_division_decode_on_every_block():
    # App. F, Alg. 1 against the division form of Sec. 3.2: two different decoders
    for d in ALL5:
        b = oracle.pack_fx_block(d, 5, 8)
        a1 = oracle.unpack_fx_alg1_block(b).tolist()
        dv = oracle.unpack_fx_div_block(b, 5, 8).tolist()
        assert a1 == dv == d.tolist()                      # digits come out d_0 first


def test_fx_rows_agree_with_the_block_forms():
    # the row-level packer / decoder (numpy closed forms) against the block-level C forms,
    # on every block and on ragged rows; all 256 byte values decode like Alg. 1
    P = oracle.pack3fx(ALL5)
    assert P[:, 0].tolist() == [oracle.pack_fx_block(d, 5, 8) for d in ALL5]
    assert not P[:, 1:].any()                              # stride padding is zero
    assert np.array_equal(oracle.unpack3fx(P, 5), ALL5)
    every = np.zeros((256, 16), dtype=np.uint8)
    every[:, 0] = np.arange(256)
    got = oracle.unpack3fx(every, 5)
    for b in range(256):
        assert got[b].tolist() == oracle.unpack_fx_alg1_block(b).tolist()
    for K in (1, 4, 5, 6, 79, 80, 81, 4096):
        W = si.ternary_weights(np.random.default_rng(700 + K), 3, K)
        Pk = oracle.pack3fx(W)
        assert Pk.shape == (3, oracle.stride3le(K))
        assert np.array_equal(oracle.unpack3fx(Pk, K), W)
        assert not Pk[:, (K + 4) // 5:].any()
    with pytest.raises(ValueError):
        oracle.pack3fx(np.array([[0, 2, 0, 0, 0]], dtype=np.int8))


# -------------------------------------------- little-endian base-3 byte

@pytest.mark.parametrize("digits,rest", _rows("base3le_bytes.txt"))
def test_base3le_golden_bytes(digits, rest):
    P = oracle.pack3le(np.array([digits], dtype=np.int8))
    assert int(P[0, 0]) == int(rest[0])
    assert not P[0, 1:].any()


def test_base3le_exhaustive_roundtrip_and_base3_digits():
    P = oracle.pack3le(ALL5)
    assert P.shape == (243, 16)
    assert sorted(P[:, 0].tolist()) == list(range(243))    # bijection onto [0, 242]
    assert not P[:, 1:].any()                               # stride padding is zero
    assert np.array_equal(oracle.unpack3le(P, 5), ALL5)
    for row, d in zip(P, ALL5):
        rep = np.base_repr(int(row[0]), 3).rjust(5, "0")[::-1]
        assert [int(c) - 1 for c in rep] == d.tolist()


@pytest.mark.parametrize("K,stride", [(1, 16), (5, 16), (80, 16), (81, 32), (4096, 832), (11008, 2208)])
def test_base3le_stride_and_ragged_roundtrip(K, stride):
    assert oracle.stride3le(K) == stride
    rng = np.random.default_rng(K)
    W = rng.integers(-1, 2, size=(3, K)).astype(np.int8)
    P = oracle.pack3le(W)
    assert P.shape == (3, stride)
    assert P.max() <= 242
    assert np.array_equal(oracle.unpack3le(P, K), W)
    assert not P[:, (K + 4) // 5:].any()


def test_base3le_rejects_bad_values():
    with pytest.raises(ValueError):
        oracle.pack3le(np.array([[0, -2, 0, 0, 0]], dtype=np.int8))
    bad = np.zeros((1, 16), dtype=np.uint8)
    bad[0, 0] = 243
    with pytest.raises(ValueError):
        oracle.unpack3le(bad, 5)
