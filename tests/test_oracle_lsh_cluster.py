"""Pins for the oracle's band keys and clusters (Section 2.3, Appendix A.2; Section 2.2
"Constructing a union graph" / "Generating the final list of duplicates")."""
import os
import random

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import connected_components

import oracle
from tests import pymirror as pm
from tests.test_oracle_minhash import _planted_pairs

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_keys_closed_form_small():
    rng = np.random.default_rng(1)
    for (K, b, r) in [(128, 16, 8), (128, 8, 16), (256, 32, 8), (64, 64, 1), (40, 3, 7), (8, 1, 8)]:
        sig = rng.integers(0, 1 << 32, size=(6, K), dtype=np.uint64).astype(np.uint32)
        sig[0, :] = 0xFFFFFFFF
        sig[1, :] = 0
        keys = oracle.lsh_keys(sig, b, r)
        assert keys.shape == (6, b)
        for d in range(6):
            assert keys[d].tolist() == pm.band_keys(sig[d].tolist(), b, r)
        assert (keys < np.uint64(pm.P)).all()


def test_keys_r1_is_identity_and_uses_leading_columns():
    rng = np.random.default_rng(2)
    sig = rng.integers(0, 1 << 32, size=(10, 32), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(oracle.lsh_keys(sig, 32, 1), sig.astype(np.uint64))
    # only the first b*r columns matter
    sig2 = sig.copy()
    sig2[:, 24:] ^= 0x5A5A5A5A
    assert np.array_equal(oracle.lsh_keys(sig, 3, 8), oracle.lsh_keys(sig2, 3, 8))
    # hand value: (1, 2) in one band -> 1 + 2 Q
    one = np.array([[1, 2]], dtype=np.uint32)
    assert int(oracle.lsh_keys(one, 1, 2)[0, 0]) == (1 + 2 * pm.QB) % pm.P


def test_keys_equal_band_equal_key_unequal_band_unequal_key():
    rng = np.random.default_rng(3)
    sig = rng.integers(0, 1 << 32, size=(2000, 16), dtype=np.uint64).astype(np.uint32)
    sig[1000:, :8] = sig[:1000, :8]                 # band 0 copied, band 1 not
    keys = oracle.lsh_keys(sig, 2, 8)
    assert np.array_equal(keys[1000:, 0], keys[:1000, 0])
    assert not (keys[1000:, 1] == keys[:1000, 1]).any()
    # a single differing row changes the key, whichever row it is
    for i in range(8):
        s2 = sig[:50].copy()
        s2[:, i] += 1
        assert not (oracle.lsh_keys(s2, 2, 8)[:, 0] == keys[:50, 0]).any()
    assert len(set(keys[:1000, 0].tolist())) == 1000


def test_keys_argument_validation():
    sig = np.zeros((2, 16), dtype=np.uint32)
    for b, r in [(0, 8), (2, 0), (3, 8), (17, 1)]:
        with pytest.raises(oracle.OracleError):
            oracle.lsh_keys(sig, b, r)


def _scurve_rows():
    rows = []
    with open(os.path.join(GOLD, "lsh_scurve.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            b, r, s, p = line.split()
            rows.append((int(b), int(r), float(s), float(p)))
    return rows


@pytest.mark.parametrize("b,r", [(16, 8), (8, 16), (32, 4)])
def test_scurve_collision_probability_on_synthetic_signatures(b, r):
    """Signatures whose slots agree independently with probability s share a band key
    with probability 1-(1-s^r)^b; the tabulated points are hit within 4 sigma."""
    rng = np.random.default_rng(b * 100 + r)
    n = 4000
    for (gb, gr, s, p) in _scurve_rows() + [(32, 4, 0.5, 1 - (1 - 0.5 ** 4) ** 32)]:
        if (gb, gr) != (b, r):
            continue
        A = rng.integers(0, 1 << 32, size=(n, b * r), dtype=np.uint64).astype(np.uint32)
        B = rng.integers(0, 1 << 32, size=(n, b * r), dtype=np.uint64).astype(np.uint32)
        agree = rng.random((n, b * r)) < s
        B[agree] = A[agree]
        hit = (oracle.lsh_keys(A, b, r) == oracle.lsh_keys(B, b, r)).any(axis=1).mean()
        sd = max(np.sqrt(p * (1 - p) / n), 1e-3)
        assert abs(hit - p) < 4 * sd, (s, hit, p)


def test_scurve_on_planted_document_pairs():
    """End to end over text: planted pairs with exact Jaccard s_i become candidates at the
    rate sum_i 1-(1-s_i^r)^b predicts (Section 2.3 candidate rule)."""
    K, n, b, r = 128, 3, 16, 8
    pairs = _planted_pairs(1500, 0.0, 0.22, seed=33)
    J = np.array([pm.jaccard(x, y, n) for x, y in pairs])
    blob = b"".join(x + y for x, y in pairs)
    off = np.cumsum([0] + [l for x, y in pairs for l in (len(x), len(y))]).astype(np.uint64)
    keys = oracle.lsh_keys(oracle.minhash(blob, off, n, K), b, r)
    hit = (keys[0::2] == keys[1::2]).any(axis=1)
    p = 1 - (1 - J ** r) ** b
    for lo, hi in [(0.0, 0.6), (0.6, 0.75), (0.75, 0.9), (0.9, 1.01), (0.0, 1.01)]:
        m = (J >= lo) & (J < hi)
        assert m.sum() >= 40, (lo, hi, m.sum())
        sd = np.sqrt((p[m] * (1 - p[m])).sum()) + 1.0
        assert abs(hit[m].sum() - p[m].sum()) < 4 * sd, (lo, hi, hit[m].sum(), p[m].sum())
    # and the clusters join exactly the pairs that share a key (pairs are mutually unrelated)
    cid = oracle.cluster(keys)
    joined = cid[0::2] == cid[1::2]
    assert (joined >= hit).all()
    assert (joined & ~hit).sum() <= 2          # an indirect path through other documents is rare


def _components_bruteforce(keys):
    n, b = keys.shape
    rows, cols = [], []
    for j in range(b):
        col = keys[:, j]
        for u in range(n):
            same = np.nonzero(col[u + 1:] == col[u])[0]
            rows += [u] * len(same)
            cols += (same + u + 1).tolist()
    g = sp.coo_matrix((np.ones(len(rows)), (rows, cols)), shape=(n, n))
    _, lab = connected_components(g, directed=False)
    low = np.full(lab.max() + 1, n, dtype=np.int64)
    np.minimum.at(low, lab, np.arange(n))
    return low[lab]


@pytest.mark.parametrize("n,b,span,seed", [(1, 1, 1, 0), (2, 1, 1, 1), (60, 4, 40, 2), (300, 16, 400, 3),
                                           (500, 3, 100, 4), (400, 8, 10 ** 9, 5), (257, 2, 3, 6)])
def test_cluster_matches_bruteforce_components(n, b, span, seed):
    rng = np.random.default_rng(seed)
    keys = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    got = oracle.cluster(keys)
    assert np.array_equal(got, _components_bruteforce(keys))
    if n <= 60:
        assert got.tolist() == pm.clusters(keys.tolist())


def test_cluster_special_cases():
    n = 50
    ident = np.arange(n * 4, dtype=np.uint64).reshape(n, 4)
    assert np.array_equal(oracle.cluster(ident), np.arange(n))           # all keys distinct
    one = ident.copy()
    one[:, 2] = 7
    assert (oracle.cluster(one) == 0).all()                               # one band all equal
    # chain through different bands: 0~1 in band 0, 1~2 in band 1
    k = np.array([[1, 10], [1, 20], [2, 20], [3, 30]], dtype=np.uint64)
    assert oracle.cluster(k).tolist() == [0, 0, 0, 3]
    # the same value in different bands does not link
    k = np.array([[5, 6], [6, 5]], dtype=np.uint64)
    assert oracle.cluster(k).tolist() == [0, 1]
    # representative is the lowest index of the component, wherever the link is found
    k = np.array([[9], [4], [9], [4], [9]], dtype=np.uint64)
    assert oracle.cluster(k).tolist() == [0, 1, 0, 1, 0]
    # large key values (just below p) are fine
    k = np.array([[pm.P - 1], [pm.P - 1], [pm.P - 2]], dtype=np.uint64)
    assert oracle.cluster(k).tolist() == [0, 0, 2]
    assert oracle.cluster(np.zeros((0, 4), dtype=np.uint64)).shape == (0,)
    with pytest.raises(oracle.OracleError):
        oracle.cluster(np.zeros((3, 0), dtype=np.uint64))


def test_cluster_idempotent_and_permutation_equivariant():
    rng = np.random.default_rng(9)
    keys = rng.integers(0, 150, size=(400, 6), dtype=np.uint64)
    cid = oracle.cluster(keys)
    assert np.array_equal(cid[cid], cid)                # labels are fixed points
    assert (cid <= np.arange(400)).all()
    perm = rng.permutation(400)
    cid_p = oracle.cluster(keys[perm])
    # same partition after relabelling: two docs share a cluster before iff after
    inv = np.empty(400, dtype=np.int64)
    inv[perm] = np.arange(400)
    same_before = cid[:, None] == cid[None, :]
    same_after = cid_p[inv][:, None] == cid_p[inv][None, :]
    assert np.array_equal(same_before, same_after)


def test_exact_copies_and_shingleless_docs_always_cocluster():
    text = b"the cat sat on the mat and looked at the dog"
    other = b"completely different words appear in this other document here"
    blob = text + other + text + b"  " + b""
    off = np.cumsum([0, len(text), len(other), len(text), 2, 0]).astype(np.uint64)
    sig = oracle.minhash(blob, off, 5, 128)
    cid = oracle.cluster(oracle.lsh_keys(sig, 16, 8))
    assert cid.tolist() == [0, 1, 0, 3, 3]              # copies join; the two empty docs join
