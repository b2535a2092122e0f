"""GPU parity of the rolling-family mode (SEDD_FLAG_ROLLING_FAMILY: every hash function is Eq. 1
of Section 3.2 to a base of its own) against the CPU oracle, bit for bit, through the C-ABI."""
import os

import numpy as np
import pytest

import oracle
from paper_2501_01046_amd import corpus
from tests.test_gpu_parity import _edge_corpus, _pack, dev, host, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
NPROC = min(16, os.cpu_count() or 1)
RF = 4
BYTES = 1


@pytest.fixture(scope="module")
def sedd():
    import paper_2501_01046_amd as m
    m.lib()
    assert m.FLAG_ROLLING_FAMILY == RF == oracle.FLAG_ROLLING_FAMILY
    yield m
    m.debug_set_chunk_bytes(0)


@pytest.mark.parametrize("seed,K", [(0, 1), (0, 128), (7, 100), ((1 << 64) - 1, 512)])
def test_bases(sedd, seed, K):
    say("rolling-family bases", seed, K)
    assert np.array_equal(host(sedd.debug_bases(seed, K)), oracle.bases(seed, K))


def _check_minhash(sedd, data, off, n, K, seed, flags, procs=1):
    want = oracle.minhash_sharded(data, off, n, K, seed, flags, procs=procs)
    got = host(sedd.sedd_minhash(dev(data), dev(off), n, K, seed, flags))
    assert got.shape == want.shape
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} documents differ, first {bad[:5]}"
    return want


def _small_edge_corpus():
    """The shared edge documents with the very long ones shortened (the oracle hashes every
    shingle once per function here)."""
    rng = np.random.default_rng(8)
    docs = [d for d in _edge_corpus() if len(d) <= 6000]
    docs.append(bytes(rng.integers(97, 123, size=700, dtype=np.uint8)))          # one long token
    docs.append(b"q " + b"k" * 63 + b" r " + b"k" * 64 + b" s " + b"k" * 65 + b" t u v w")
    docs.append(b"q " + b"m" * 254 + b" r " + b"m" * 255 + b" s " + b"m" * 256 + b" t u v w")
    docs.append(b" ".join(bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8))
                          for l in rng.integers(1, 12, size=900)))               # several tiles
    docs.append(bytes(rng.integers(0, 256, size=3000, dtype=np.uint8)))
    return docs


@pytest.mark.parametrize("n,flags", [(1, 0), (2, 0), (3, 0), (5, 0), (6, 0), (9, 0),
                                     (1, 1), (5, 1), (13, 1), (64, 1)])
def test_minhash_edge_documents(sedd, n, flags):
    say("rolling-family minhash edge", n, flags)
    data, off = _pack(_small_edge_corpus(), 5)
    _check_minhash(sedd, data, off, n, 24, seed=99, flags=flags | RF, procs=NPROC)


@pytest.mark.parametrize("K", [1, 63, 64, 65, 128, 200])
def test_minhash_K_sweep(sedd, K):
    say("rolling-family minhash K", K)
    data, off = corpus.generate(corpus.config(1).scaled(60))
    _check_minhash(sedd, data, off, 5, K, seed=K, flags=RF, procs=NPROC)


@pytest.mark.parametrize("chunk", [1 << 12, 50_000, 0])
def test_minhash_chunk_invariance(sedd, chunk):
    say("rolling-family minhash chunk", chunk)
    r = corpus.config(1).scaled(150, ws_variety=1)
    data, off = corpus.generate(r)
    sedd.debug_set_chunk_bytes(chunk)
    try:
        _check_minhash(sedd, data, off, 5, 32, 0, RF, procs=NPROC)
        _check_minhash(sedd, data, off, 13, 32, 0, RF | BYTES, procs=NPROC)
    finally:
        sedd.debug_set_chunk_bytes(0)


def test_minhash_long_documents_split_into_tiles(sedd):
    say("rolling-family minhash long docs")
    r = corpus.Recipe("long", seed=4, n_docs=12, len_median=1500, len_sigma=1.0, len_lo=1,
                      len_hi=8000, near_frac=0.2, utf8_pct=5)
    data, off = corpus.generate(r)
    _check_minhash(sedd, data, off, 5, 128, 1, RF, procs=NPROC)
    _check_minhash(sedd, data[: int(off[6])], off[:7], 13, 128, 1, RF | BYTES, procs=NPROC)


def test_flag_combinations(sedd):
    say("rolling-family flags")
    data, off = _pack([b"a b c d e f g"], 0)
    for flags in (6, 7, 8):
        with pytest.raises(sedd.SeddError) as e:
            sedd.sedd_minhash(dev(data), dev(off), 5, 8, 0, flags)
        assert e.value.code == -1
    with pytest.raises(sedd.SeddError):
        sedd.debug_shingle_hashes(dev(data), dev(off), 5, RF)


def test_modes_alternate_on_the_same_scratch(sedd):
    say("rolling-family alternating modes")
    data, off = corpus.generate(corpus.config(1).scaled(120))
    w61 = oracle.minhash_sharded(data, off, 5, 64, 0, 0, procs=NPROC)
    wrf = oracle.minhash_sharded(data, off, 5, 64, 0, RF, procs=NPROC)
    wpp = oracle.minhash_sharded(data, off, 5, 64, 0, 2, procs=NPROC)
    d_data, d_off = dev(data), dev(off)
    for _ in range(2):
        assert np.array_equal(host(sedd.sedd_minhash(d_data, d_off, 5, 64, 0, RF)), wrf)
        assert np.array_equal(host(sedd.sedd_minhash(d_data, d_off, 5, 64, 0, 0)), w61)
        assert np.array_equal(host(sedd.sedd_minhash(d_data, d_off, 5, 64, 0, 2)), wpp)


def _full_path(sedd, recipe, procs):
    data, off = corpus.generate(recipe)
    flags = int(recipe.byte_mode) | RF
    wsig = oracle.minhash_sharded(data, off, recipe.shingle_n, recipe.K, 0, flags, procs=procs)
    wkeys = oracle.lsh_keys(wsig, recipe.b, recipe.r)
    wcid = oracle.cluster(wkeys)
    sig = sedd.sedd_minhash(dev(data), dev(off), recipe.shingle_n, recipe.K, 0, flags)
    keys = sedd.sedd_lsh_keys(sig, recipe.b, recipe.r)
    cid = sedd.sedd_cluster(keys)
    assert np.array_equal(host(sig), wsig)
    assert np.array_equal(host(keys), wkeys)
    assert np.array_equal(host(cid), wcid)
    return wcid


def test_config1_shape_whole_path(sedd):
    say("rolling-family config 1 shape (scaled)")
    cid = _full_path(sedd, corpus.config(1).scaled(1500), NPROC)
    assert int((cid != np.arange(cid.size)).sum()) >= 20


def test_config4_shape_small(sedd):
    say("rolling-family config 4 shape (scaled)")
    _full_path(sedd, corpus.config(4).scaled(300, long_lo=3_000, long_hi=8_000), NPROC)
