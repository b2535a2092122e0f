"""GPU parity of the paper-prime mode (SEDD_FLAG_PAPER_PRIME: Section 3.2's p = 4,294,967 as the
modulus of Eq. 1 and of the K hash functions) against the CPU oracle, bit for bit, through the
C-ABI."""
import os

import numpy as np
import pytest

import oracle
from paper_2501_01046_amd import corpus
from tests.test_gpu_parity import _edge_corpus, _fuzz_docs, _pack, _piece_edge_docs, dev, host, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
NPROC = min(16, os.cpu_count() or 1)
PP = 4294967
PAPER = 2
BYTES = 1


@pytest.fixture(scope="module")
def sedd():
    import paper_2501_01046_amd as m
    m.lib()
    assert m.FLAG_PAPER_PRIME == PAPER == oracle.FLAG_PAPER_PRIME
    yield m
    m.debug_set_chunk_bytes(0)


@pytest.mark.parametrize("seed,K", [(0, 1), (0, 128), (7, 100), ((1 << 64) - 1, 512), ((1 << 61) - 2, 64)])
def test_coeffs(sedd, seed, K):
    say("paper-prime coeffs", seed, K)
    a, b = sedd.debug_coeffs(seed, K, paper_prime=True)
    wa, wb = oracle.coeffs(seed, K, paper_prime=True)
    assert np.array_equal(host(a), wa) and np.array_equal(host(b), wb)


def _oracle_x(docs, n, byte_mode):
    parts = [oracle.doc_shingles(d, n, byte_mode, paper_prime=True) for d in docs]
    soff = np.cumsum([0] + [p.size for p in parts]).astype(np.uint64)
    return (np.concatenate(parts) if parts else np.zeros(0, np.uint64)), soff


@pytest.mark.parametrize("byte_mode", [False, True])
@pytest.mark.parametrize("n", [1, 2, 5, 7, 13, 64])
def test_shingle_hashes_edge_cases(sedd, byte_mode, n):
    say("paper-prime shingle_hashes edge", byte_mode, n)
    docs = _edge_corpus()
    # tokens of 254..257 and 300 bytes sit on both sides of the record format's length escape
    docs += [b"q " + b"k" * l + b" r s t u v" for l in (63, 64, 254, 255, 256, 257, 300)]
    data, off = _pack(docs, 3)
    wx, woff = _oracle_x(docs, n, byte_mode)
    x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), n, PAPER | int(byte_mode))
    assert np.array_equal(host(soff), woff)
    assert np.array_equal(host(x), wx)


@pytest.mark.parametrize("chunk", [0, 1 << 12, 70_000])
@pytest.mark.parametrize("byte_mode", [False, True])
def test_shingle_hashes_generated_corpus_and_chunking(sedd, chunk, byte_mode):
    say("paper-prime shingle_hashes corpus", chunk, byte_mode)
    r = corpus.Recipe("t", seed=31, n_docs=600, vocab=3000, len_median=150, len_sigma=1.0,
                      len_lo=0, len_hi=3000, near_frac=0.2, exact_frac=0.05, ws_variety=1,
                      utf8_pct=10)
    data, off = corpus.generate(r)
    raw = data.tobytes()
    docs = [raw[int(off[d]):int(off[d + 1])] for d in range(r.n_docs)]
    n = 13 if byte_mode else 5
    wx, woff = _oracle_x(docs, n, byte_mode)
    sedd.debug_set_chunk_bytes(chunk)
    try:
        x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), n, PAPER | int(byte_mode))
    finally:
        sedd.debug_set_chunk_bytes(0)
    assert np.array_equal(host(soff), woff)
    assert np.array_equal(host(x), wx)


def _from_x_case(sedd, parts, K, seed):
    x = np.concatenate(parts) if parts else np.zeros(0, np.uint64)
    off = np.cumsum([0] + [p.size for p in parts]).astype(np.uint64)
    got = host(sedd.debug_minhash_from_x(dev(x), dev(off), K, seed, paper_prime=True))
    for d, p in enumerate(parts):
        assert np.array_equal(got[d], oracle.minhash_shingles(p, K, seed, paper_prime=True)), (K, seed, d)


def test_minhash_from_x_random_and_edge_values(sedd):
    say("paper-prime minhash from x")
    rng = np.random.default_rng(5)
    lens = [0, 1, 2, 3, 4, 5, 7, 8, 9, 159, 160, 161, 319, 320, 321, 639, 640, 641, 5000, 0, 3]
    parts = [rng.integers(0, PP, size=l, dtype=np.uint64) for l in lens]
    parts.append(np.array([0, 1, 2, PP - 2, PP - 1, 1 << 22, (1 << 22) - 1, 4194304, 2147483], dtype=np.uint64))
    parts.append(np.array([PP, PP + 1, (1 << 61) - 2, (1 << 64) - 1, 1 << 32], dtype=np.uint64))  # reduced first
    for K, seed in [(128, 0), (64, 3), (256, 9), (100, 1), (1, 2), (32, 4), (33, 5), (1000, 6)]:
        _from_x_case(sedd, parts, K, seed)


def test_minhash_values_next_to_the_modulus(sedd):
    """Shingle values chosen so that (a x + b) mod p lands on chosen targets next to 0 and next to
    p: the kernel's quotient estimate is off by one just below p, where it must fall back to the
    plain reduction whenever such a value could be the minimum."""
    say("paper-prime near-modulus values")
    K, seed = 128, 0
    a, b = oracle.coeffs(seed, K, paper_prime=True)
    top = [PP - 1, PP - 2, PP - 3, PP - 10, PP - 100, PP - 1000, PP - 4000, PP - 4294, PP - 4295,
           PP - 4296, PP - 4399, PP - 4400, PP - 4401, PP - 5000, PP - 9000]
    low = [0, 1, 2, 3, 100]
    parts = []
    for k in (0, 1, 31, 32, 63, 64, 127):
        inv = pow(int(a[k]), -1, PP)
        xs_top = [((t - int(b[k])) * inv) % PP for t in top]
        xs_low = [((t - int(b[k])) * inv) % PP for t in low]
        for t, xv in zip(top, xs_top):
            assert (int(a[k]) * xv + int(b[k])) % PP == t
        # documents whose minimum for function k is one of the top values: alone, in pairs, all
        for xv in xs_top:
            parts.append(np.array([xv], dtype=np.uint64))
        parts.append(np.array(xs_top, dtype=np.uint64))
        parts.append(np.array(xs_top[:2], dtype=np.uint64))
        parts.append(np.array(xs_top + xs_low, dtype=np.uint64))
        parts.append(np.concatenate([np.array(xs_top * 30, dtype=np.uint64)]))      # 450: two tiles
        filler = np.random.default_rng(k).integers(0, PP, size=300, dtype=np.uint64)
        parts.append(np.concatenate([np.array(xs_top + xs_low, dtype=np.uint64), filler]))
    _from_x_case(sedd, parts, K, seed)
    _from_x_case(sedd, parts, 256, seed)        # the whole-wave layout (more than 128 functions)


def test_every_residue_through_one_function(sedd):
    """All p residues as the shingles of 2,000 documents of consecutive values, 8 functions:
    every value the quotient estimate can meet passes through the kernel once per function."""
    say("paper-prime all residues")
    K, seed, step = 8, 11, 2148
    a, b = oracle.coeffs(seed, K, paper_prime=True)
    x = np.arange(PP, dtype=np.uint64)
    bounds = np.arange(0, PP + step, step, dtype=np.uint64)
    bounds[-1] = PP
    got = host(sedd.debug_minhash_from_x(dev(x), dev(bounds), K, seed, paper_prime=True))
    for k in range(K):
        h = (x * a[k] + b[k]) % np.uint64(PP)                    # below 2^46: exact in uint64
        want = np.minimum.reduceat(h, bounds[:-1].astype(np.int64))
        assert np.array_equal(got[:, k], want.astype(np.uint32)), k


def _check_minhash(sedd, data, off, n, K, seed, flags, procs=1):
    want = oracle.minhash_sharded(data, off, n, K, seed, flags, procs=procs)
    got = host(sedd.sedd_minhash(dev(data), dev(off), n, K, seed, flags))
    assert got.shape == want.shape
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} documents differ, first {bad[:5]}"
    return want


@pytest.mark.parametrize("K", [1, 31, 64, 65, 128, 200, 256, 512, 1000])
def test_minhash_K_sweep(sedd, K):
    say("paper-prime minhash K", K)
    data, off = corpus.generate(corpus.config(1).scaled(300))
    _check_minhash(sedd, data, off, 5, K, seed=K, flags=PAPER)


@pytest.mark.parametrize("n,flags", [(1, 0), (3, 0), (5, 0), (9, 0), (1, 1), (5, 1), (13, 1), (64, 1)])
def test_minhash_edge_documents(sedd, n, flags):
    say("paper-prime minhash edge", n, flags)
    data, off = _pack(_edge_corpus(), 5)
    _check_minhash(sedd, data, off, n, 128, seed=99, flags=flags | PAPER)


@pytest.mark.parametrize("chunk", [1 << 12, 50_000, 0])
def test_minhash_chunk_invariance(sedd, chunk):
    say("paper-prime minhash chunk", chunk)
    r = corpus.config(1).scaled(400, ws_variety=1)
    data, off = corpus.generate(r)
    sedd.debug_set_chunk_bytes(chunk)
    try:
        _check_minhash(sedd, data, off, 5, 128, 0, PAPER, procs=NPROC)
    finally:
        sedd.debug_set_chunk_bytes(0)


def test_minhash_long_documents_split_into_tiles(sedd):
    say("paper-prime minhash long docs")
    r = corpus.Recipe("long", seed=4, n_docs=40, len_median=3000, len_sigma=1.0, len_lo=1,
                      len_hi=40000, near_frac=0.2, utf8_pct=5)
    data, off = corpus.generate(r)
    _check_minhash(sedd, data, off, 5, 128, 1, PAPER, procs=NPROC)
    _check_minhash(sedd, data[: int(off[12])], off[:13], 13, 128, 1, PAPER | BYTES, procs=NPROC)


@pytest.mark.parametrize("piece", [1024, 5120, 1 << 20])
def test_stream_kernel_piece_size_invariance(sedd, piece):
    """Word shingles of this mode run through the streaming kernel too: shingle hashes in order and
    signatures against the oracle however the text is cut between wavefronts."""
    say("paper-prime stream piece", piece)
    sedd.debug_set_piece_bytes(piece)
    try:
        for lead in (0, 1019):
            docs = _piece_edge_docs() + _fuzz_docs(piece + lead, 60)
            data, off = _pack(docs, lead)
            d_data, d_off = dev(data), dev(off)
            for n in (1, 5, 64):
                wx, woff = _oracle_x(docs, n, False)
                x, soff = sedd.debug_shingle_hashes(d_data, d_off, n, PAPER)
                assert np.array_equal(host(soff), woff), (lead, n)
                assert np.array_equal(host(x), wx), (lead, n)
            for n, K in ((5, 128), (3, 256), (1, 40), (64, 32)):
                want = oracle.minhash(data, off, n, K, 3, PAPER)
                got = host(sedd.sedd_minhash(d_data, d_off, n, K, 3, PAPER))
                bad = np.nonzero((got != want).any(axis=1))[0]
                assert bad.size == 0, (lead, n, K, bad[:5])
    finally:
        sedd.debug_set_piece_bytes(0)


@pytest.mark.parametrize("max_len", [8, 9, 16, 17, 40])
def test_stream_kernel_token_length_tiers(sedd, max_len):
    """Longest word exactly at and next to the limits of the three token-hash paths, all byte
    values inside the words."""
    say("paper-prime stream token lengths up to", max_len)
    rng = np.random.default_rng(100 + max_len)
    pool = np.array([c for c in range(256) if c not in (9, 10, 11, 12, 13, 32)], dtype=np.uint8)
    docs = []
    for _ in range(120):
        lens = rng.integers(1, max_len + 1, size=int(rng.integers(1, 400)))
        lens[rng.integers(0, lens.size)] = max_len
        docs.append(b" ".join(bytes(rng.choice(pool, size=int(l))) for l in lens))
    data, off = _pack(docs, lead=max_len % 16)
    wx, woff = _oracle_x(docs, 3, False)
    x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), 3, PAPER)
    assert np.array_equal(host(soff), woff) and np.array_equal(host(x), wx)
    _check_minhash(sedd, data, off, 5, 64, seed=max_len, flags=PAPER, procs=NPROC)


@pytest.mark.parametrize("n,K", [(1, 64), (2, 256), (1, 1000)])
def test_stream_kernel_rounds_of_one_or_two_shingles(sedd, n, K):
    """The hash loop's quotient estimate is exact only below p' minus a margin; a round whose
    minimum lies above is redone exactly.  That needs rounds of very few shingles: tens of
    thousands of documents of one to three short words, about one (document, function) pair in a
    thousand within the margin."""
    say("paper-prime stream tiny documents", n, K)
    rng = np.random.default_rng(n * 1000 + K)
    n_docs = 30_000 if K <= 256 else 8_000
    docs = []
    for _ in range(n_docs):
        words = [bytes(rng.integers(97, 123, size=int(rng.integers(1, 10)), dtype=np.uint8))
                 for _ in range(int(rng.integers(1, 4)))]
        docs.append(b" ".join(words))
    data, off = _pack(docs, 0)
    want = _check_minhash(sedd, data, off, n, K, seed=5, flags=PAPER, procs=NPROC)
    near = int((want >= PP - 4400).sum())
    assert near >= 20, near          # the case did occur: minima inside the margin


def test_modes_alternate_on_the_same_scratch(sedd):
    say("paper-prime alternating modes")
    data, off = corpus.generate(corpus.config(1).scaled(700))
    w61 = oracle.minhash_sharded(data, off, 5, 128, 0, 0, procs=NPROC)
    wpp = oracle.minhash_sharded(data, off, 5, 128, 0, PAPER, procs=NPROC)
    d_data, d_off = dev(data), dev(off)
    for _ in range(2):
        assert np.array_equal(host(sedd.sedd_minhash(d_data, d_off, 5, 128, 0, PAPER)), wpp)
        assert np.array_equal(host(sedd.sedd_minhash(d_data, d_off, 5, 128, 0, 0)), w61)
    assert (wpp[wpp != 0xFFFFFFFF] < PP).all()


def _full_path(sedd, recipe, procs):
    data, off = corpus.generate(recipe)
    flags = int(recipe.byte_mode) | PAPER
    wsig = oracle.minhash_sharded(data, off, recipe.shingle_n, recipe.K, 0, flags, procs=procs)
    wkeys = oracle.lsh_keys(wsig, recipe.b, recipe.r)
    wcid = oracle.cluster(wkeys)
    sig = sedd.sedd_minhash(dev(data), dev(off), recipe.shingle_n, recipe.K, 0, flags)
    keys = sedd.sedd_lsh_keys(sig, recipe.b, recipe.r)
    cid = sedd.sedd_cluster(keys)
    assert np.array_equal(host(sig), wsig)
    assert np.array_equal(host(keys), wkeys)
    assert np.array_equal(host(cid), wcid)
    mm = oracle.min_match_for(0.8, recipe.K)
    assert np.array_equal(host(sedd.sedd_cluster_verified(keys, sig, mm)),
                          oracle.cluster_verified(wkeys, wsig, mm))
    return wsig, wcid


def test_config1_whole_path(sedd):
    say("paper-prime config 1 whole path")
    _, cid = _full_path(sedd, corpus.config(1), NPROC)
    dups = int((cid != np.arange(cid.size)).sum())
    assert 100 <= dups <= 600          # small documents: about the clusters of the 61-bit mode


def test_config3_and_config5_shapes_small(sedd):
    say("paper-prime config 3 / 5 shapes (scaled)")
    _full_path(sedd, corpus.config(3).scaled(3000), NPROC)
    _full_path(sedd, corpus.config(5).scaled(1500, K=512, b=64, r=4, shingle_n=3), NPROC)


def test_config4_shape_small_and_range_exhaustion(sedd):
    """Byte 13-grams with documents of up to 2 MB: the 22-bit range is exhausted, the minima of
    long documents collapse towards 0 and unrelated long documents share bands."""
    say("paper-prime config 4 shape (scaled)")
    r = corpus.config(4).scaled(600, long_lo=200_000, long_hi=400_000)
    wsig, _ = _full_path(sedd, r, NPROC)
    data, off = corpus.generate(r)
    lens = np.diff(off.astype(np.int64))
    longest = np.argsort(lens)[-2:]
    assert lens[longest].min() > 1_000_000
    assert wsig[longest].max() < 64
