"""Pins for the oracle's rolling-family mode (flags bit 2).

Section 2.2 asks for H hash functions, Section 3.2 defines one (Eq. 1).  This mode takes Eq. 1
itself as the family: function k is Eq. 1 with a base q_k of its own.  Expected values come from
hand arithmetic, Python big integers (tests/pymirror), Eq. 2's reuse identity per base, and from
what the family's structure implies: shingles that differ only in their first character keep
their order under every function, which min-wise independence forbids.
"""
import random

import numpy as np
import pytest

import oracle
from tests import pymirror as pm

P = (1 << 61) - 1
RF = oracle.FLAG_ROLLING_FAMILY
BYTES = oracle.FLAG_BYTE_SHINGLES

TEXTS = [
    b"", b" ", b"one", b"one two", b"  one   two  ", b"a b c d e", b"a b c d e f",
    b"a  b\tc\nd\re\x0bf\x0cg", b"x\x00y z\x00 \x00", b"\xc3\xa9t\xc3\xa9 na\xc3\xafve \xff\xfe \x80",
    b"w1 w2 w3 w4 w5 w6 w7 w8 w9 w10 w11 w12", b"z" * 300 + b" " + b"y" * 70 + b" q",
]


def test_eq1_to_another_base_hand_values():
    assert oracle.base_hash_q(b"", 1000) == 0
    assert oracle.base_hash_q(b"a", 1000) == 97
    assert oracle.base_hash_q(b"ab", 1000) == 97 + 98 * 1000
    assert oracle.base_hash_q(b"abc", 1000) == 97 + 98_000 + 99_000_000
    assert oracle.base_hash_q(b"abc", 257) == oracle.base_hash(b"abc")
    # base p - 1 = -1: alternating sum
    assert oracle.base_hash_q(b"\x05\x03\x09", P - 1) == 5 - 3 + 9
    assert oracle.base_hash_q(b"\x01\x02", P - 1) == P - 1


def test_eq1_big_integers_and_reuse_identity():
    rng = random.Random(9)
    for _ in range(100):
        q = rng.randrange(257, P)
        s = bytes(rng.randrange(256) for _ in range(rng.randrange(0, 80)))
        assert oracle.base_hash_q(s, q) == pm.eq1(s, q)
    # Eq. 2 for a base of its own: h(t) = (h(s) - c_1) / q + c_{k+1} q^(k-1)
    for k in (1, 5, 13):
        q = rng.randrange(257, P)
        inv = pow(q, -1, P)
        s = bytes(rng.randrange(256) for _ in range(k + 20))
        h = oracle.base_hash_q(s[:k], q)
        for i in range(20):
            h = ((h - s[i]) * inv + s[i + k] * pow(q, k - 1, P)) % P
            assert h == oracle.base_hash_q(s[i + 1:i + 1 + k], q)


@pytest.mark.parametrize("seed", [0, 1, 12345, (1 << 64) - 1])
def test_bases_closed_form(seed):
    q = oracle.bases(seed, 40).tolist()
    assert q == pm.bases(seed, 40)
    assert all(257 <= x < P for x in q) and len(set(q)) == 40
    a, _ = oracle.coeffs(seed, 40)
    assert q == [257 + int(x) % (P - 257) for x in a]
    assert oracle.bases(seed, 7).tolist() == q[:7]           # prefix property


@pytest.mark.parametrize("byte_mode", [False, True])
@pytest.mark.parametrize("n", [1, 3, 5, 13])
def test_shingle_hashes_match_enumeration(n, byte_mode):
    for q in (257, 1000, 1 << 40, P - 1):
        for t in TEXTS:
            want = [pm.eq1(s, q) for s in pm.shingle_strings(t, n, byte_mode)]
            assert oracle.doc_shingles_q(t, n, q, byte_mode).tolist() == want, (t, n, q)


@pytest.mark.parametrize("byte_mode", [False, True])
@pytest.mark.parametrize("seed", [0, 99])
def test_signatures_match_enumeration(byte_mode, seed):
    n, K = (13 if byte_mode else 5), 12
    data = b"".join(TEXTS)
    off = np.cumsum([0] + [len(t) for t in TEXTS]).astype(np.uint64)
    got = oracle.minhash(data, off, n, K, seed, RF | (BYTES if byte_mode else 0))
    for d, t in enumerate(TEXTS):
        assert got[d].tolist() == pm.signature_rf(t, n, K, seed, byte_mode), (d, t)
    assert (got[0] == 0xFFFFFFFF).all()
    # K-prefix, whitespace-run invariance in word mode
    assert np.array_equal(oracle.minhash(data, off, n, 5, seed, RF | (BYTES if byte_mode else 0)),
                          got[:, :5])
    if not byte_mode:
        a, b = b"alpha beta gamma delta epsilon zeta", b" alpha\tbeta\n\ngamma delta  epsilon zeta "
        s = oracle.minhash(a + b, [0, len(a), len(a) + len(b)], 5, K, seed, RF)
        assert np.array_equal(s[0], s[1])


def test_flag_bits_are_checked():
    for flags in (6, 7, 8, 12):
        with pytest.raises(oracle.OracleError):
            oracle.minhash(b"a b", [0, 3], 5, 4, 0, flags)
    t = b"one two three four five six seven"
    assert (oracle.minhash(t, [0, len(t)], 5, 16, 0, 0) != oracle.minhash(t, [0, len(t)], 5, 16, 0, RF)).any()


def test_first_character_order_is_the_same_under_every_function():
    """Two shingles that differ only in their first character differ by c_1 - c_1' under every
    base (the first character has weight q^0), so the one with the smaller first character wins
    the minimum under every function unless the 32-bit truncation wraps (probability 2^-24).
    The affine family orders them either way, half of the functions each."""
    K = 256
    a, b = b"Aabcdefghijkl", b"Babcdefghijkl"                 # one byte 13-gram each
    off = [0, 13, 26]
    rf = oracle.minhash(a + b, off, 13, K, 0, RF | BYTES)
    assert (rf[0] < rf[1]).all() and ((rf[1] - rf[0]) == 1).all()
    aff = oracle.minhash(a + b, off, 13, K, 0, BYTES)
    frac = float((aff[0] < aff[1]).mean())
    assert 0.35 < frac < 0.65
    # consequence for the estimate, with single words as shingles: {Aword, Bword} against {Bword}
    # has Jaccard 1/2, but the family never lets the shared shingle be the minimum of the first
    # set, so no slot matches; the affine family matches about half of them
    x, y = b"Aword Bword", b"Bword"
    o2 = [0, len(x), len(x) + len(y)]
    r = oracle.minhash(x + y, o2, 1, K, 0, RF)
    assert (r[0] == r[1]).sum() == 0
    f = oracle.minhash(x + y, o2, 1, K, 0, 0)
    assert 0.35 < float((f[0] == f[1]).mean()) < 0.65


def test_last_character_carries_the_highest_power():
    """Orientation of Eq. 1: shingles that differ in their LAST character differ by
    (c - c') q^(k-1), which is spread over the range: their order varies with the function."""
    K = 256
    a, b = b"abcdefghijklA", b"abcdefghijklB"
    rf = oracle.minhash(a + b, [0, 13, 26], 13, K, 0, RF | BYTES)
    frac = float((rf[0] < rf[1]).mean())
    assert 0.35 < frac < 0.65


def test_estimates_jaccard_on_word_shingles():
    """On word shingles dominated pairs are rare (they need the same n-1 following words and a
    first word that differs in its first character only), and the slot-match rate estimates
    the Jaccard similarity like any min-hash family."""
    rng = np.random.default_rng(18)
    vocab = [bytes(rng.integers(97, 123, size=rng.integers(2, 9)).astype(np.uint8)) for _ in range(3000)]
    K, diffs = 64, []
    for _ in range(60):
        base = [vocab[i] for i in rng.integers(0, len(vocab), size=120)]
        other = list(base)
        for i in rng.choice(120, size=rng.integers(1, 20), replace=False):
            other[i] = vocab[rng.integers(0, len(vocab))]
        ta, tb = b" ".join(base), b" ".join(other)
        J = pm.jaccard(ta, tb, 5)
        sig = oracle.minhash(ta + tb, [0, len(ta), len(ta) + len(tb)], 5, K, 0, RF)
        diffs.append(float((sig[0] == sig[1]).mean()) - J)
    assert abs(np.mean(diffs)) < 0.02
    assert np.std(diffs) < 0.08
