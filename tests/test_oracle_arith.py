"""Pins for the oracle's modular arithmetic, Eq. 1 hash and coefficient family.

Nothing here compares the oracle with itself: the expected values are Python
big-integer arithmetic, hand-derived closed forms (tests/golden) and the
paper's own identities (Section 3.2, Eq. 1 and Eq. 2).
"""
import os
import random

import numpy as np
import pytest

import oracle
from tests import pymirror as pm

P = pm.P
GOLD = os.path.join(os.path.dirname(__file__), "golden")

EDGE = [0, 1, 2, 255, 256, 257, (1 << 32) - 1, 1 << 32, (1 << 32) + 1, 1 << 60,
        (1 << 60) + 1, P - 2, P - 1]


def test_mulmod_against_bigint_edges_and_random():
    rng = random.Random(1)
    ops = [(a, b) for a in EDGE for b in EDGE]
    ops += [(rng.randrange(P), rng.randrange(P)) for _ in range(20000)]
    ops += [(rng.randrange(1 << 32), rng.randrange(P)) for _ in range(2000)]
    for a, b in ops:
        assert oracle.mulmod(a, b) == a * b % P


def test_addmod_against_bigint():
    rng = random.Random(2)
    ops = [(a, b) for a in EDGE for b in EDGE]
    ops += [(rng.randrange(P), rng.randrange(P)) for _ in range(5000)]
    for a, b in ops:
        assert oracle.addmod(a, b) == (a + b) % P


def test_mersenne_identity():
    # 2^61 = 1 (mod p): 2^60 * 2 wraps to 1, and (p-1)^2 = 1
    assert oracle.mulmod(1 << 60, 2) == 1
    assert oracle.mulmod(P - 1, P - 1) == 1
    assert oracle.mulmod(1 << 31, 1 << 30) == 1


def test_powmod_against_pow():
    for g in (2, 257, pm.GA, pm.GB, pm.QB, P - 1):
        for e in (0, 1, 2, 3, 61, 122, 511, 512):
            assert oracle.powmod(g, e) == pow(g, e, P)


def _golden_eq1():
    rows = []
    with open(os.path.join(GOLD, "eq1_closed_forms.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            hx, val = line.split()
            rows.append((bytes.fromhex(hx), int(val)))
    return rows


def test_base_hash_closed_forms():
    rows = _golden_eq1()
    assert len(rows) >= 6
    for s, val in rows:
        assert oracle.base_hash(s) == val


def test_base_hash_small_cases():
    assert oracle.base_hash(b"") == 0
    for c in (0, 1, 97, 255):
        assert oracle.base_hash(bytes([c])) == c
    # first character sits at q^0: reversing a two-byte string changes the value
    assert oracle.base_hash(b"ab") == 97 + 98 * 257
    assert oracle.base_hash(b"ba") == 98 + 97 * 257
    # a trailing zero byte adds 0 * q^len
    assert oracle.base_hash(b"xyz\x00") == oracle.base_hash(b"xyz")


def test_base_hash_against_bigint_random():
    rng = random.Random(3)
    for _ in range(300):
        n = rng.randrange(0, 80)
        s = bytes(rng.randrange(256) for _ in range(n))
        assert oracle.base_hash(s) == pm.eq1(s)


def test_eq2_rolling_identity():
    """Eq. 2: the next window's hash from the previous one (division by q = inverse mod p)."""
    rng = random.Random(4)
    qinv = pow(pm.Q, -1, P)
    assert qinv * pm.Q % P == 1
    for k in (1, 2, 5, 13, 40):
        text = bytes(rng.randrange(256) for _ in range(k + 60))
        h = oracle.base_hash(text[:k])
        for i in range(60):
            nxt = ((h - text[i]) * qinv + text[i + k] * pow(pm.Q, k - 1, P)) % P
            assert oracle.base_hash(text[i + 1:i + 1 + k]) == nxt
            h = nxt


def test_base_hash_concatenation_rule():
    # x(s || t) = x(s) + q^|s| x(t): the polynomial structure of Eq. 1
    rng = random.Random(5)
    for _ in range(100):
        s = bytes(rng.randrange(256) for _ in range(rng.randrange(0, 30)))
        t = bytes(rng.randrange(256) for _ in range(rng.randrange(0, 30)))
        want = (oracle.base_hash(s) + pow(pm.Q, len(s), P) * oracle.base_hash(t)) % P
        assert oracle.base_hash(s + t) == want


def test_base_hash_collision_rate_is_tiny():
    # Appendix B: collisions of distinct inputs ~ 1/p; 20k distinct strings -> none expected
    rng = random.Random(6)
    seen = {}
    for _ in range(20000):
        s = bytes(rng.randrange(97, 123) for _ in range(rng.randrange(8, 40)))
        h = oracle.base_hash(s)
        assert seen.setdefault(h, s) == s
    vals = np.array(list(seen.keys()), dtype=np.float64) / P
    # uniformity (Appendix B): mean 1/2, variance 1/12 within sampling error
    assert abs(vals.mean() - 0.5) < 0.01
    assert abs(vals.var() - 1 / 12) < 0.005


def test_coeffs_closed_form_and_constants():
    a, b = oracle.coeffs(0, 8)
    assert int(a[0]) == pm.GA and int(b[0]) == pm.GB          # seed 0 -> s0 = 1
    assert int(a[1]) == 1656610497311288960 == pm.GA * pm.GA % P
    assert int(b[1]) == 2131494254484603902 == pm.GB * pm.GB % P
    for seed in (0, 1, 12345, P - 2, P - 1, P, (1 << 64) - 1):
        a, b = oracle.coeffs(seed, 64)
        pa, pb = pm.coeffs(seed, 64)
        assert [int(v) for v in a] == pa
        assert [int(v) for v in b] == pb
        assert all(0 < int(v) < P for v in a) and all(0 < int(v) < P for v in b)


def test_coeffs_prefix_property_and_distinctness():
    a512, b512 = oracle.coeffs(7, 512)
    for K in (1, 64, 100, 128, 256):
        a, b = oracle.coeffs(7, K)
        assert np.array_equal(a, a512[:K]) and np.array_equal(b, b512[:K])
    assert len(set(a512.tolist())) == 512 and len(set(b512.tolist())) == 512


def test_coeffs_rejects_bad_K():
    with pytest.raises(oracle.OracleError):
        oracle.coeffs(0, 0)
