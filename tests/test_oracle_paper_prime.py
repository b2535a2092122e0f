"""Pins for the oracle's paper-prime mode (flags bit 1).

Section 3.2 quotes p = 4,294,967 as the modulus of Eq. 1 in the paper's
experiments.  The mode evaluates Eq. 1 and the H hash functions modulo that
prime.  Expected values come from hand arithmetic, from Python big integers
(tests/pymirror), from Eq. 2's reuse identity, and from what a 22-bit range
implies: small documents still estimate the Jaccard similarity, documents
with millions of shingles exhaust the range and look alike.
"""
import random

import numpy as np
import pytest

import oracle
from tests import pymirror as pm

PP = 4294967
PAPER = oracle.FLAG_PAPER_PRIME
BYTES = oracle.FLAG_BYTE_SHINGLES

TEXTS = [
    b"", b" ", b"one", b"one two", b"  one   two  ", b"a b c d e", b"a b c d e f",
    b"a  b\tc\nd\re\x0bf\x0cg", b"x\x00y z\x00 \x00", b"\xc3\xa9t\xc3\xa9 na\xc3\xafve \xff\xfe \x80",
    b"w1 w2 w3 w4 w5 w6 w7 w8 w9 w10 w11 w12", b"z" * 300 + b" " + b"y" * 70 + b" q",
]


def test_the_constant_is_prime_and_fits_the_paper_s_bound():
    assert all(PP % d for d in range(2, int(PP ** 0.5) + 1))
    assert 257 * (PP - 1) < 2 ** 32          # h * q stays a 32-bit integer (Section 3.2)
    assert oracle.P_PAPER == PP == pm.P_PAPER


def test_eq1_hand_values():
    assert oracle.base_hash_pp(b"") == 0
    assert oracle.base_hash_pp(b"a") == 97
    assert oracle.base_hash_pp(b"ab") == 97 + 98 * 257                     # 25283, below p
    assert oracle.base_hash_pp(b"abc") == 97 + 98 * 257 + 99 * 66049 - PP  # 6564134 wraps once
    assert oracle.base_hash_pp(b"\x00\x00\x01") == 66049
    assert oracle.base_hash_pp(b"\xff" * 4) == (255 * (1 + 257 + 257 ** 2 + 257 ** 3)) % PP


def test_eq1_big_integers():
    rng = random.Random(5)
    for _ in range(300):
        s = bytes(rng.randrange(256) for _ in range(rng.randrange(0, 90)))
        assert oracle.base_hash_pp(s) == pm.eq1(s, 257, PP)


def test_eq2_reuse_identity():
    # h(t) = ((h(s) - c_1) / q + c_{k+1} q^(k-1)) mod p with the division as a modular inverse
    rng = random.Random(6)
    inv = pow(257, -1, PP)
    for k in (1, 2, 5, 13, 40):
        s = bytes(rng.randrange(256) for _ in range(k + 30))
        h = oracle.base_hash_pp(s[:k])
        for i in range(30):
            h = ((h - s[i]) * inv + s[i + k] * pow(257, k - 1, PP)) % PP
            assert h == oracle.base_hash_pp(s[i + 1:i + 1 + k])


@pytest.mark.parametrize("seed", [0, 1, 12345, (1 << 61) - 2, (1 << 64) - 1])
def test_coefficients_closed_form(seed):
    a, b = oracle.coeffs(seed, 40, paper_prime=True)
    wa, wb = pm.coeffs_pp(seed, 40)
    assert a.tolist() == wa and b.tolist() == wb
    assert all(1 <= x < PP for x in wa) and all(0 <= x < PP for x in wb)
    a61, b61 = oracle.coeffs(seed, 40)
    assert a.tolist() == [int(x) % (PP - 1) + 1 for x in a61]
    assert b.tolist() == [int(x) % PP for x in b61]


@pytest.mark.parametrize("n", [1, 3, 5, 13])
@pytest.mark.parametrize("byte_mode", [False, True])
def test_shingle_hashes_match_enumeration(n, byte_mode):
    for t in TEXTS:
        want = [pm.eq1(s, 257, PP) for s in pm.shingle_strings(t, n, byte_mode)]
        got = oracle.doc_shingles(t, n, byte_mode, paper_prime=True).tolist()
        assert got == want, (t, n, byte_mode)


@pytest.mark.parametrize("byte_mode", [False, True])
@pytest.mark.parametrize("seed", [0, 99])
def test_signatures_match_enumeration(byte_mode, seed):
    n, K = (13 if byte_mode else 5), 24
    data = b"".join(TEXTS)
    off = np.cumsum([0] + [len(t) for t in TEXTS]).astype(np.uint64)
    got = oracle.minhash(data, off, n, K, seed, PAPER | (BYTES if byte_mode else 0))
    for d, t in enumerate(TEXTS):
        assert got[d].tolist() == pm.signature_pp(t, n, K, seed, byte_mode), (d, t)


def test_values_are_residues_and_empty_is_all_ones():
    data = b"alpha beta gamma delta epsilon zeta eta theta" + b"  "
    sig = oracle.minhash(data, [0, 45, 47], 5, 64, 7, PAPER)
    assert (sig[0] < PP).all()
    assert (sig[1] == 0xFFFFFFFF).all()


def test_set_semantics_and_prefix_property():
    rng = np.random.default_rng(3)
    x = rng.integers(0, PP, size=200, dtype=np.uint64)
    s = oracle.minhash_shingles(x, 48, 11, paper_prime=True)
    assert (oracle.minhash_shingles(rng.permutation(np.concatenate([x, x[:50]])), 48, 11, True) == s).all()
    assert (oracle.minhash_shingles(x, 16, 11, True) == s[:16]).all()
    # the functions see x only through its residue
    assert (oracle.minhash_shingles(x + np.uint64(PP), 48, 11, True) == s).all()
    # a permutation of the residues: distinct inputs give distinct values per function
    a, b = pm.coeffs_pp(11, 4)
    for k in range(4):
        vals = {(a[k] * int(v) + b[k]) % PP for v in range(0, PP, 4099)}
        assert len(vals) == len(range(0, PP, 4099))


def test_flag_bits_are_checked():
    with pytest.raises(oracle.OracleError):
        oracle.minhash(b"a b", [0, 3], 5, 4, 0, 8)
    # the two modes are different functions of the same text
    t = b"one two three four five six seven"
    assert (oracle.minhash(t, [0, len(t)], 5, 16, 0, 0) != oracle.minhash(t, [0, len(t)], 5, 16, 0, PAPER)).any()


def _random_doc(rng, vocab, n_words):
    return b" ".join(vocab[i] for i in rng.integers(0, len(vocab), size=n_words))


def test_small_documents_still_estimate_jaccard():
    # a few hundred shingles out of 4.3 M residues: chance collisions are rare, so the slot-match
    # rate stays an unbiased estimate of the Jaccard similarity (Section 2.2) to within sampling noise
    rng = np.random.default_rng(17)
    vocab = [bytes(rng.integers(97, 123, size=rng.integers(2, 9)).astype(np.uint8)) for _ in range(3000)]
    K, diffs = 128, []
    for _ in range(120):
        base = [vocab[i] for i in rng.integers(0, len(vocab), size=150)]
        other = list(base)
        for i in rng.choice(150, size=rng.integers(1, 25), replace=False):
            other[i] = vocab[rng.integers(0, len(vocab))]
        ta, tb = b" ".join(base), b" ".join(other)
        J = pm.jaccard(ta, tb, 5)
        sig = oracle.minhash(ta + tb, [0, len(ta), len(ta) + len(tb)], 5, K, 0, PAPER)
        diffs.append(float((sig[0] == sig[1]).mean()) - J)
    assert abs(np.mean(diffs)) < 0.015
    assert np.std(diffs) < 0.06


def test_long_documents_exhaust_the_range():
    # n distinct shingles drawn from p residues leave a minimum of about p / n: with n near p the
    # minimum of every function is 0 or a handful, so unrelated long documents agree on a large
    # share of the slots (expected sum_v P(min = v)^2, about (1 - e^-c) / (1 + e^-c) for n = c p),
    # which the 61-bit modulus never does
    rng = np.random.default_rng(23)
    K, n = 64, 3_000_000                      # c = n / p = 0.70 -> expected match rate 0.34
    a = rng.integers(0, 256, size=n + 12, dtype=np.uint8).tobytes()
    b = rng.integers(0, 256, size=n + 12, dtype=np.uint8).tobytes()
    off = [0, len(a), len(a) + len(b)]
    sp = oracle.minhash(a + b, off, 13, K, 0, PAPER | BYTES)
    s61 = oracle.minhash(a + b, off, 13, K, 0, BYTES)
    c = n / PP
    expect = (1 - np.exp(-c)) / (1 + np.exp(-c))
    rate = float((sp[0] == sp[1]).mean())
    assert abs(rate - expect) < 4 * np.sqrt(expect * (1 - expect) / K)
    assert sp.max() < 40                       # every minimum is tiny
    assert (s61[0] == s61[1]).sum() <= 2       # 32-bit minima of 3 M draws: n / 2^33 per slot
