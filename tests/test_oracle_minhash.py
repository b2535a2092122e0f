"""Pins for the oracle's shingling and signatures (Section 2.2).

Expected values come from brute-force enumeration in Python (tests/pymirror),
from invariants the definitions imply, and from the statistics of MinHash: the
slot-match rate is an unbiased estimate of the Jaccard similarity
(Section 2.2, "Duplicate pair generation"; Appendix A.1, Eq. 4).
"""
import random

import numpy as np
import pytest

import oracle
from paper_2501_01046_amd import corpus
from tests import pymirror as pm

TEXTS = [
    b"", b" ", b"\t\n\r\x0b\x0c ", b"one", b"one two", b"  one   two  ", b"a b c d e",
    b"a b c d e f", b"a  b\tc\nd\re\x0bf\x0cg", b" lead and trail ", b"x\x00y z\x00 \x00",
    b"\xc3\xa9t\xc3\xa9 na\xc3\xafve caf\xc3\xa9 \xff\xfe \x80", b"\x1f not\x1fspace \x0e\x08",
    b"w1 w2 w3 w4 w5 w6 w7 w8 w9 w10 w11 w12", b"\xa0nbsp\xa0is\xa0not\xa0space",
]


@pytest.mark.parametrize("n", [1, 2, 3, 5, 13])
@pytest.mark.parametrize("byte_mode", [False, True])
def test_shingle_hashes_match_enumeration(n, byte_mode):
    for t in TEXTS:
        want = [pm.eq1(s) for s in pm.shingle_strings(t, n, byte_mode)]
        got = oracle.doc_shingles(t, n, byte_mode).tolist()
        assert got == want, (t, n, byte_mode)


def test_shingle_counts():
    assert oracle.doc_shingles(b"a b c d e", 5).size == 1
    assert oracle.doc_shingles(b"a b c d e f g", 5).size == 3
    assert oracle.doc_shingles(b"a b", 5).size == 1          # fewer tokens than n: one shingle
    assert oracle.doc_shingles(b"   ", 5).size == 0
    assert oracle.doc_shingles(b"abcdef", 3, True).size == 4
    assert oracle.doc_shingles(b"ab", 3, True).size == 1
    assert oracle.doc_shingles(b"", 3, True).size == 0
    # the short-document shingle is the tokens joined by single spaces
    assert oracle.doc_shingles(b" a \t b ", 5)[0] == pm.eq1(b"a b")


def test_whitespace_run_invariance_word_mode():
    a = b"alpha beta gamma delta epsilon zeta eta"
    b = b"\n alpha\t\tbeta  gamma\r\ndelta \x0b epsilon\x0czeta   eta \n"
    assert np.array_equal(oracle.doc_shingles(a, 5), oracle.doc_shingles(b, 5))
    off = np.array([0, len(a), len(a) + len(b)], dtype=np.uint64)
    sig = oracle.minhash(a + b, off, 5, 64)
    assert np.array_equal(sig[0], sig[1])


def _tiny_corpus(seed, n_docs, ws=1, **kw):
    r = corpus.Recipe("tiny", seed=seed, n_docs=n_docs, vocab=200, len_median=12, len_sigma=0.9,
                      len_lo=0, len_hi=60, near_frac=0.3, exact_frac=0.1, edit_lo=0.05,
                      edit_hi=0.3, ws_variety=ws, **kw)
    return corpus.generate(r, threads=2)


@pytest.mark.parametrize("n,byte_mode,K", [(5, False, 16), (3, False, 8), (13, True, 8), (1, True, 4)])
def test_signatures_match_bruteforce_on_tiny_corpus(n, byte_mode, K):
    data, off = _tiny_corpus(11, 40, utf8_pct=20)
    sig = oracle.minhash(data, off, n, K, seed=5, flags=int(byte_mode))
    raw = data.tobytes()
    for d in range(40):
        t = raw[int(off[d]):int(off[d + 1])]
        assert sig[d].tolist() == pm.signature(t, n, K, 5, byte_mode), d


def test_empty_and_shingleless_documents():
    data = b"hello world foo" + b"   \n"
    off = np.array([0, 0, 15, 19, 19], dtype=np.uint64)     # empty, text, whitespace only, empty
    sig = oracle.minhash(data, off, 5, 32)
    assert (sig[0] == 0xFFFFFFFF).all() and (sig[2] == 0xFFFFFFFF).all() and (sig[3] == 0xFFFFFFFF).all()
    assert (sig[1] != 0xFFFFFFFF).any()
    assert sig[1].tolist() == pm.signature(b"hello world foo", 5, 32)
    # zero documents is a no-op
    assert oracle.minhash(b"", np.array([0], dtype=np.uint64), 5, 8).shape == (0, 8)


def test_identical_documents_identical_signatures_and_position_independence():
    data, off = _tiny_corpus(12, 30, ws=0)
    raw = data.tobytes()
    docs = [raw[int(off[d]):int(off[d + 1])] for d in range(30)]
    sig = oracle.minhash(data, off, 5, 64, seed=9)
    # shuffle the documents, duplicate some, re-run: each keeps its signature
    order = list(range(30)) + [3, 3, 17]
    random.Random(0).shuffle(order)
    blob = b"".join(docs[i] for i in order)
    off2 = np.cumsum([0] + [len(docs[i]) for i in order]).astype(np.uint64)
    sig2 = oracle.minhash(blob, off2, 5, 64, seed=9)
    for pos, i in enumerate(order):
        assert np.array_equal(sig2[pos], sig[i])
    # chunk invariance: a sub-range with chunk-relative offsets
    sub = oracle.minhash(raw[int(off[10]):int(off[20])], off[10:21] - off[10], 5, 64, seed=9)
    assert np.array_equal(sub, sig[10:20])
    # offsets that do not start at 0
    pad = b"zzz " + raw
    assert np.array_equal(oracle.minhash(pad, off + np.uint64(4), 5, 64, seed=9), sig)


def test_signature_independent_of_shingle_order_and_repetition():
    rng = np.random.default_rng(0)
    x = rng.integers(0, pm.P, size=300, dtype=np.uint64)
    base = oracle.minhash_shingles(x, 128, seed=3)
    assert np.array_equal(oracle.minhash_shingles(rng.permutation(x), 128, seed=3), base)
    rep = np.concatenate([x, x[::3], x[:7]])
    assert np.array_equal(oracle.minhash_shingles(rng.permutation(rep), 128, seed=3), base)
    # the minimum over a union is the element-wise minimum of the parts
    part = np.minimum(oracle.minhash_shingles(x[:100], 128, seed=3),
                      oracle.minhash_shingles(x[100:], 128, seed=3))
    assert np.array_equal(part, base)
    # one shingle: the signature is h_k itself, from big integers
    a, b = pm.coeffs(3, 128)
    one = oracle.minhash_shingles(x[:1], 128, seed=3)
    assert one.tolist() == [((a[k] * int(x[0]) + b[k]) % pm.P) % (1 << 32) for k in range(128)]


def test_K_prefix_and_seed_dependence():
    data, off = _tiny_corpus(13, 20)
    s256 = oracle.minhash(data, off, 5, 256, seed=1)
    for K in (1, 64, 100, 128):
        assert np.array_equal(oracle.minhash(data, off, 5, K, seed=1), s256[:, :K])
    assert not np.array_equal(oracle.minhash(data, off, 5, 64, seed=2), s256[:, :64])


def test_truncation_happens_before_the_minimum():
    # two shingle values whose 61-bit hashes order one way and low 32 bits the other
    a, b = pm.coeffs(0, 1)
    rng = random.Random(8)
    while True:
        x1, x2 = rng.randrange(pm.P), rng.randrange(pm.P)
        h1, h2 = (a[0] * x1 + b[0]) % pm.P, (a[0] * x2 + b[0]) % pm.P
        if h1 < h2 and (h1 & 0xFFFFFFFF) > (h2 & 0xFFFFFFFF):
            break
    sig = oracle.minhash_shingles(np.array([x1, x2], dtype=np.uint64), 1, seed=0)
    assert int(sig[0]) == h2 & 0xFFFFFFFF


def test_argument_validation():
    off = np.array([0, 3], dtype=np.uint64)
    for kw in (dict(shingle_n=0, K=8), dict(shingle_n=5, K=0), dict(shingle_n=5, K=8, flags=8), dict(shingle_n=5, K=8, flags=6)):
        with pytest.raises(oracle.OracleError):
            oracle.minhash(b"abc", off, **kw)
    with pytest.raises(oracle.OracleError):
        oracle.minhash(b"abc", np.array([3, 0], dtype=np.uint64), 5, 8)


def _planted_pairs(n_pairs, rate_lo, rate_hi, seed):
    """(text_a, text_b) pairs: fresh documents and edited copies of them."""
    r = corpus.Recipe("pairs", seed=seed, n_docs=2 * n_pairs, vocab=5000, len_median=120,
                      len_sigma=0.5, len_lo=40, len_hi=400, near_frac=0.0)
    c = corpus.Corpus(r)
    rng = np.random.default_rng(seed)
    pairs = []
    for i in range(n_pairs):
        ids = c.word_ids(i).tolist()
        rate = rng.uniform(rate_lo, rate_hi)
        out = []
        for w in ids:
            u = rng.random()
            if u < rate:
                op = rng.integers(3)
                if op == 0:
                    out.append(int(rng.integers(5000)))
                elif op == 1:
                    out += [int(rng.integers(5000)), w]
            else:
                out.append(w)
        ta = b" ".join(c.word(w) for w in ids)
        tb = b" ".join(c.word(w) for w in out)
        pairs.append((ta, tb))
    return pairs


def test_slot_match_rate_is_unbiased_for_jaccard():
    K, n = 128, 3
    pairs = _planted_pairs(1200, 0.0, 0.25, seed=21)
    J = np.array([pm.jaccard(a, b, n) for a, b in pairs])
    blob = b"".join(a + b for a, b in pairs)
    lens = [l for a, b in pairs for l in (len(a), len(b))]
    off = np.cumsum([0] + lens).astype(np.uint64)
    sig = oracle.minhash(blob, off, n, K, seed=0)
    match = (sig[0::2] == sig[1::2]).mean(axis=1)
    assert J.min() < 0.35 and J.max() > 0.95          # the sample spans the range
    err = match - J
    sd_mean = np.sqrt((J * (1 - J) / K).mean() / len(pairs))
    assert abs(err.mean()) < 4 * sd_mean + 0.004
    # per-pair spread is binomial: Var(match) = J(1-J)/K
    z2 = (err ** 2).sum() / (J * (1 - J) / K).sum()
    assert 0.8 < z2 < 1.25
    # binned: no bin is biased
    for lo, hi in [(0.0, 0.5), (0.5, 0.7), (0.7, 0.85), (0.85, 1.01)]:
        m = (J >= lo) & (J < hi)
        if m.sum() >= 50:
            sd = np.sqrt((J[m] * (1 - J[m]) / K).mean() / m.sum())
            assert abs(err[m].mean()) < 4 * sd + 0.006, (lo, hi)


def test_unrelated_documents_share_almost_no_slots():
    data, off = corpus.generate(corpus.Recipe("u", seed=5, n_docs=200, near_frac=0.0,
                                              len_median=80, len_hi=300))
    sig = oracle.minhash(data, off, 5, 128)
    same = (sig[:100] == sig[100:]).mean()
    assert same < 0.01


@pytest.mark.parametrize("flags", [0, oracle.FLAG_BYTE_SHINGLES, oracle.FLAG_PAPER_PRIME,
                                   oracle.FLAG_ROLLING_FAMILY])
def test_sharded_wrapper_equals_the_single_call(flags):
    """minhash_sharded (the reference of most GPU comparisons) is the plain oracle cut into
    document ranges: same signatures for any worker count, with empty documents, offsets that
    do not start at 0, and fewer documents than two per worker."""
    data, off = _tiny_corpus(31, 700)
    # empty documents: repeat some offsets; a leading gap: the first document starts at byte 37
    off = np.concatenate([off[:200], off[199:200], off[199:400], off[399:400], off[399:]])
    lead = np.frombuffer(b"unused lead-in bytes, not a document ", dtype=np.uint8)
    data = np.concatenate([lead, data])
    off = (off + np.uint64(lead.size)).astype(np.uint64)
    n = 13 if flags & oracle.FLAG_BYTE_SHINGLES else 3
    want = oracle.minhash(data, off, n, 24, 5, flags)
    assert (want[200] == 0xFFFFFFFF).all()                   # the planted empty document
    for procs in (1, 2, 3, 8):
        got = oracle.minhash_sharded(data, off, n, 24, 5, flags, procs=procs)
        assert np.array_equal(got, want), procs
    # fewer documents than 2 * procs: the wrapper must fall back to one call
    few = off[:6]
    assert np.array_equal(oracle.minhash_sharded(data, few, n, 24, 5, flags, procs=8),
                          oracle.minhash(data, few, n, 24, 5, flags))
    # exactly 2 * procs documents, and a worker count that does not divide the document count
    assert np.array_equal(oracle.minhash_sharded(data, off[:17], n, 24, 5, flags, procs=8),
                          oracle.minhash(data, off[:17], n, 24, 5, flags))
    assert np.array_equal(oracle.minhash_sharded(data, off[:101], n, 24, 5, flags, procs=7),
                          oracle.minhash(data, off[:101], n, 24, 5, flags))
