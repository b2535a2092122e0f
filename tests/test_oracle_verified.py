"""Pins for the oracle's verified clusters (Section 2.3 last step, Section 3.3: a candidate pair
is a duplicate iff the number of equal signature entries is at least theta * H)."""
import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import connected_components

import oracle


def _verified_bruteforce(keys, sig, min_match):
    """All n^2 pairs: candidate iff some band key agrees; duplicate iff enough entries agree."""
    n = keys.shape[0]
    cand = np.zeros((n, n), dtype=bool)
    for j in range(keys.shape[1]):
        cand |= keys[:, j][:, None] == keys[:, j][None, :]
    same = (sig[:, None, :] == sig[None, :, :]).sum(axis=2)
    adj = cand & (same >= min_match)
    np.fill_diagonal(adj, False)
    _, lab = connected_components(sp.csr_matrix(adj), directed=False)
    low = np.full(lab.max() + 1, n, dtype=np.int64)
    np.minimum.at(low, lab, np.arange(n))
    return low[lab]


def _random_case(seed, n, K, b, span, groups):
    """Signatures drawn around a few prototypes so that match counts spread over 0..K; keys
    random in a small range so that buckets of several documents form."""
    rng = np.random.default_rng(seed)
    proto = rng.integers(0, 1 << 32, size=(groups, K), dtype=np.uint64).astype(np.uint32)
    pick = rng.integers(0, groups, size=n)
    sig = proto[pick].copy()
    flip = rng.random((n, K)) < rng.random((n, 1)) * 0.6
    sig[flip] = rng.integers(0, 1 << 32, size=int(flip.sum()), dtype=np.uint64).astype(np.uint32)
    keys = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    return keys, sig


@pytest.mark.parametrize("seed,n,K,b,span,groups", [(0, 1, 8, 1, 1, 1), (1, 2, 8, 1, 1, 1),
                                                    (2, 80, 16, 3, 12, 4), (3, 200, 32, 4, 30, 6),
                                                    (4, 150, 128, 16, 60, 5), (5, 120, 7, 2, 3, 2)])
def test_verified_matches_bruteforce(seed, n, K, b, span, groups):
    keys, sig = _random_case(seed, n, K, b, span, groups)
    for mm in sorted({0, 1, K // 4, K // 2, (4 * K + 4) // 5, K, K + 1}):
        got = oracle.cluster_verified(keys, sig, mm)
        assert np.array_equal(got, _verified_bruteforce(keys, sig, mm)), mm


def test_threshold_zero_is_plain_bucket_grouping_and_above_K_is_identity():
    keys, sig = _random_case(7, 300, 32, 5, 40, 5)
    assert np.array_equal(oracle.cluster_verified(keys, sig, 0), oracle.cluster(keys))
    assert np.array_equal(oracle.cluster_verified(keys, sig, 33), np.arange(300))


def test_threshold_boundary_is_inclusive():
    """A pair with exactly m equal entries is a duplicate for min_match = m and not for m + 1
    ("at least theta * H", Section 3.3)."""
    K = 20
    rng = np.random.default_rng(9)
    base = rng.integers(0, 1 << 32, size=K, dtype=np.uint64).astype(np.uint32)
    for m in (0, 1, 7, 19, 20):
        other = base.copy()
        other[m:] ^= np.uint32(1)                     # exactly m leading entries agree
        sig = np.stack([base, other])
        keys = np.array([[5, 1], [5, 2]], dtype=np.uint64)   # same bucket in band 0 only
        assert oracle.cluster_verified(keys, sig, m).tolist() == [0, 0]
        assert oracle.cluster_verified(keys, sig, m + 1).tolist() == [0, 1]
        # no shared bucket: never a candidate, however similar
        keys2 = np.array([[5, 1], [6, 2]], dtype=np.uint64)
        assert oracle.cluster_verified(keys2, sig, 0).tolist() == [0, 1]


def test_all_pairs_inside_a_bucket_not_only_the_first_document():
    """Documents 1 and 2 are duplicates of each other but not of document 0, the first of their
    bucket: an anchor-only comparison would miss the pair, the exhaustive one must not
    (Section 3.1: all pairs, O(D^2))."""
    K = 16
    a = np.arange(K, dtype=np.uint32)
    b = a + np.uint32(1000)
    sig = np.stack([a, b, b.copy()])
    keys = np.array([[9], [9], [9]], dtype=np.uint64)
    assert oracle.cluster_verified(keys, sig, K).tolist() == [0, 1, 1]


def test_transitive_through_different_bands_and_lowest_index():
    K = 8
    s = np.zeros((4, K), dtype=np.uint32)
    s[1, :2] = 1            # 0~1 agree on 6, 1~2 agree on 6, 0~2 agree on 4
    s[2, :2] = 1
    s[2, 2:4] = 2
    s[3] = 77
    keys = np.array([[1, 10], [1, 20], [2, 20], [3, 30]], dtype=np.uint64)
    assert oracle.cluster_verified(keys, s, 6).tolist() == [0, 0, 0, 3]
    assert oracle.cluster_verified(keys, s, 7).tolist() == [0, 1, 2, 3]
    perm = np.array([3, 2, 1, 0])
    assert oracle.cluster_verified(keys[perm], s[perm], 6).tolist() == [0, 1, 1, 1]


def test_monotone_in_the_threshold():
    keys, sig = _random_case(11, 400, 24, 6, 50, 6)
    prev = oracle.cluster_verified(keys, sig, 0)
    for mm in range(1, 26):
        cur = oracle.cluster_verified(keys, sig, mm)
        # a higher threshold only removes edges: every new cluster lies inside an old one
        assert np.array_equal(prev[cur], prev[np.arange(400)][cur]) and (prev[cur] == prev).all()
        prev = cur
    assert np.array_equal(prev, np.arange(400))


def test_min_match_is_the_ceiling_of_theta_times_K():
    assert oracle.min_match_for(0.8, 128) == 103      # 102.4 -> 103
    assert oracle.min_match_for(0.8, 125) == 100      # exactly 100: stays 100
    assert oracle.min_match_for(0.5, 3) == 2
    assert oracle.min_match_for(1.0, 64) == 64
    assert oracle.min_match_for(0.0, 64) == 0
    assert oracle.min_match_for(0.7, 10) == 7         # 0.7 * 10 is not exact in binary floating point


def test_on_documents_verified_clusters_refine_bucket_clusters():
    from paper_2501_01046_amd import corpus
    r = corpus.config(2).scaled(1500)
    data, off = corpus.generate(r)
    sig = oracle.minhash(data, off, 5, 128)
    keys = oracle.lsh_keys(sig, 16, 8)
    plain = oracle.cluster(keys)
    ver = oracle.cluster_verified(keys, sig, oracle.min_match_for(0.8, 128))
    assert (plain[ver] == plain).all()                # refinement
    assert (ver != np.arange(ver.size)).sum() <= (plain != np.arange(plain.size)).sum()
    # every member of a verified cluster agrees with some other member on >= 103 entries
    for d in np.nonzero(ver != np.arange(ver.size))[0][:200]:
        mates = np.nonzero(ver == ver[d])[0]
        best = max(int((sig[d] == sig[m]).sum()) for m in mates if m != d)
        assert best >= 103


def test_argument_validation():
    keys = np.zeros((2, 1), dtype=np.uint64)
    sig = np.zeros((2, 4), dtype=np.uint32)
    with pytest.raises(oracle.OracleError):
        oracle.cluster_verified(keys, sig, -1)
    assert oracle.cluster_verified(keys[:0], sig[:0], 1).size == 0


# ---- dense bucket ids (Section 3.2: sum of the band's values modulo the number of buckets) ----

def test_dense_keys_closed_form_and_range():
    rng = np.random.default_rng(21)
    for (K, b, r, nb) in [(128, 16, 8, 4000), (64, 64, 1, 7), (40, 3, 7, 1), (256, 32, 8, 12649),
                          (16, 1, 16, (1 << 40) + 5)]:
        sig = rng.integers(0, 1 << 32, size=(9, K), dtype=np.uint64).astype(np.uint32)
        sig[0] = 0xFFFFFFFF                       # the sum must not wrap at 32 or 64 bits
        sig[1] = 0
        keys = oracle.lsh_dense_keys(sig, b, r, nb)
        assert keys.shape == (9, b) and (keys < np.uint64(nb)).all()
        for d in range(9):
            for j in range(b):
                want = sum(int(v) for v in sig[d, j * r:(j + 1) * r]) % nb
                assert int(keys[d, j]) == want
    # hand values: band (1, 2, 3) -> 6 mod 4 = 2; all-ones band of 8 -> 8 (2^32 - 1) mod 1000
    assert int(oracle.lsh_dense_keys(np.array([[1, 2, 3]], np.uint32), 1, 3, 4)[0, 0]) == 2
    assert int(oracle.lsh_dense_keys(np.full((1, 8), 0xFFFFFFFF, np.uint32), 1, 8, 1000)[0, 0]) \
        == (8 * 0xFFFFFFFF) % 1000 == 360


def test_dense_keys_depend_on_the_band_as_a_multiset_and_only_on_leading_columns():
    rng = np.random.default_rng(22)
    sig = rng.integers(0, 1 << 32, size=(50, 32), dtype=np.uint64).astype(np.uint32)
    keys = oracle.lsh_dense_keys(sig, 3, 8, 977)
    perm = sig.copy()
    perm[:, :8] = sig[:, 7::-1]                   # a sum does not see the order inside a band
    assert np.array_equal(oracle.lsh_dense_keys(perm, 3, 8, 977), keys)
    tail = sig.copy()
    tail[:, 24:] ^= 0x1234
    assert np.array_equal(oracle.lsh_dense_keys(tail, 3, 8, 977), keys)
    # equal bands give equal buckets; r = 1 is the value modulo the count
    assert np.array_equal(oracle.lsh_dense_keys(sig, 32, 1, 1013), sig.astype(np.uint64) % np.uint64(1013))


def test_dense_buckets_are_balanced_and_coarse():
    """Random signatures spread evenly over the buckets (the paper's bucket-balance analysis):
    with N = 40000 and 4 sqrt(N) = 800 buckets the mean bucket holds 50 documents."""
    rng = np.random.default_rng(23)
    n = 40_000
    nb = oracle.dense_bucket_count(n)
    assert nb == 800 and oracle.dense_bucket_count(1_000_000) == 4000
    assert oracle.dense_bucket_count(32_800_000, k=2) == 11454       # floor(2 sqrt(N))
    sig = rng.integers(0, 1 << 32, size=(n, 8), dtype=np.uint64).astype(np.uint32)
    keys = oracle.lsh_dense_keys(sig, 1, 8, nb)[:, 0]
    counts = np.bincount(keys.astype(np.int64), minlength=nb)
    assert counts.sum() == n and abs(counts.mean() - 50) < 1e-9
    assert counts.std() < 2 * np.sqrt(50) and counts.max() < 50 + 6 * np.sqrt(50)


def test_dense_buckets_with_verification_find_the_planted_duplicates():
    """Coarse buckets propose many candidate pairs; the count-match test keeps the real ones."""
    rng = np.random.default_rng(24)
    n, K, b, r = 3000, 64, 8, 8
    sig = rng.integers(0, 1 << 32, size=(n, K), dtype=np.uint64).astype(np.uint32)
    src = rng.choice(n // 2, size=200, replace=False)
    dup = n // 2 + np.arange(200)
    sig[dup] = sig[src]
    noisy = rng.random((200, K)) < 0.1            # about 90 % of the entries still agree
    sig[dup] = np.where(noisy, rng.integers(0, 1 << 32, size=(200, K), dtype=np.uint64).astype(np.uint32), sig[dup])
    keys = oracle.lsh_dense_keys(sig, b, r, oracle.dense_bucket_count(n))
    cid = oracle.cluster_verified(keys, sig, oracle.min_match_for(0.8, K))
    same_band = (sig[dup].reshape(200, b, r) == sig[src].reshape(200, b, r)).all(axis=2).any(axis=1)
    enough = (sig[dup] == sig[src]).sum(axis=1) >= oracle.min_match_for(0.8, K)
    found = cid[dup] == cid[src]
    assert (found >= (same_band & enough)).all()  # an untouched band + enough agreement: found
    assert found.sum() >= 150
    others = np.setdiff1d(np.arange(n), np.concatenate([src, dup]))
    assert (cid[others] == others).all()          # random documents never verify
    assert np.array_equal(cid, _verified_bruteforce(keys, sig, oracle.min_match_for(0.8, K)))
