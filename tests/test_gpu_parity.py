"""GPU parity: every result of the HIP library against the CPU oracle, bit for bit.

All of these go through the C-ABI (ctypes) via the thin binding.  Signatures, band keys and
cluster ids are integers with a unique correct value, so the bar is exact equality.
"""
import os
import time

import numpy as np
import pytest

import oracle
from paper_2501_01046_amd import corpus

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
NPROC = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def sedd():
    import paper_2501_01046_amd as m
    m.lib()
    yield m
    m.debug_set_chunk_bytes(0)


def dev(a):
    a = np.ascontiguousarray(a)
    if not a.flags.writeable:
        a = a.copy()
    return torch.from_numpy(a).cuda()


def host(t):
    return t.cpu().numpy()


def say(*a):
    print(*a, flush=True)


# ---- stage level ---------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 5, 64, 1023, 1024, 1025, 4097, (1 << 20) + 3, 3_000_001])
def test_scan_u32(sedd, n):
    say("scan", n)
    rng = np.random.default_rng(n)
    v = rng.integers(0, 1000, size=n, dtype=np.uint32)
    got = host(sedd.debug_scan_u32(dev(v)))
    want = np.concatenate([[0], np.cumsum(v[:-1], dtype=np.uint64)]).astype(np.uint32)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("seed,K", [(0, 128), (1, 1), (12345, 512), ((1 << 64) - 1, 300), ((1 << 61) - 2, 64)])
def test_coeffs(sedd, seed, K):
    say("coeffs", seed, K)
    a, b = sedd.debug_coeffs(seed, K)
    wa, wb = oracle.coeffs(seed, K)
    assert np.array_equal(host(a), wa) and np.array_equal(host(b), wb)


EDGE_TEXTS = [
    b"", b" ", b"\t\n\r\x0b\x0c ", b"one", b"one two", b"  one   two  ", b"a b c d e",
    b"a b c d e f", b"a  b\tc\nd\re\x0bf\x0cg", b" lead and trail ", b"x\x00y z\x00 \x00",
    b"\xc3\xa9t\xc3\xa9 na\xc3\xafve caf\xc3\xa9 \xff\xfe \x80", b"\x1f not\x1fspace \x0e\x08", b"",
    b"w1 w2 w3 w4 w5 w6 w7 w8 w9 w10 w11 w12", b"\xa0nbsp\xa0is\xa0not\xa0space", b"a", b"b", b"c",
    b"ab", b"cd", b" ", b"tail",
]


def _edge_corpus():
    rng = np.random.default_rng(7)
    docs = list(EDGE_TEXTS)
    # a token longer than a 4 KiB tile, a document spanning several tiles, abutting tokens
    docs.append(bytes(rng.integers(97, 123, size=9000, dtype=np.uint8)))
    docs.append(b" ".join(bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8))
                          for l in rng.integers(1, 12, size=3000)))
    docs.append(b"x" * 4096)
    docs.append(b"y" * 4095 + b" " + b"z" * 10)
    docs.append(b" " * 5000)
    docs.append((b"ab " * 3000) + b"\n")
    docs.append(bytes(rng.integers(0, 256, size=20000, dtype=np.uint8)))
    return docs


def _pack(docs, lead=0):
    blob = b"\x20" * lead + b"".join(docs)
    off = np.cumsum([lead] + [len(d) for d in docs]).astype(np.uint64)
    return np.frombuffer(blob, dtype=np.uint8), off


def _oracle_x(docs, n, byte_mode):
    parts = [oracle.doc_shingles(d, n, byte_mode) for d in docs]
    soff = np.cumsum([0] + [p.size for p in parts]).astype(np.uint64)
    return (np.concatenate(parts) if parts else np.zeros(0, np.uint64)), soff


@pytest.mark.parametrize("byte_mode", [False, True])
@pytest.mark.parametrize("n", [1, 2, 5, 13])
@pytest.mark.parametrize("lead", [0, 3])
def test_shingle_hashes_edge_cases(sedd, byte_mode, n, lead):
    say("shingle_hashes edge", byte_mode, n, lead)
    docs = _edge_corpus()
    data, off = _pack(docs, lead)
    wx, woff = _oracle_x(docs, n, byte_mode)
    x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), n, int(byte_mode))
    assert np.array_equal(host(soff), woff)
    assert np.array_equal(host(x), wx)


@pytest.mark.parametrize("chunk", [0, 1 << 12, 70_000])
@pytest.mark.parametrize("byte_mode", [False, True])
def test_shingle_hashes_generated_corpus_and_chunking(sedd, chunk, byte_mode):
    say("shingle_hashes corpus", chunk, byte_mode)
    r = corpus.Recipe("t", seed=3, n_docs=600, vocab=3000, len_median=150, len_sigma=1.0,
                      len_lo=0, len_hi=3000, near_frac=0.2, exact_frac=0.05, ws_variety=1,
                      utf8_pct=10)
    data, off = corpus.generate(r)
    raw = data.tobytes()
    docs = [raw[int(off[d]):int(off[d + 1])] for d in range(r.n_docs)]
    n = 13 if byte_mode else 5
    wx, woff = _oracle_x(docs, n, byte_mode)
    sedd.debug_set_chunk_bytes(chunk)
    try:
        x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), n, int(byte_mode))
    finally:
        sedd.debug_set_chunk_bytes(0)
    assert np.array_equal(host(soff), woff)
    assert np.array_equal(host(x), wx)


def test_unaligned_text_pointer(sedd):
    say("unaligned pointer")
    docs = _edge_corpus()
    data, off = _pack(docs, 0)
    wx, woff = _oracle_x(docs, 5, False)
    for shift in (1, 7, 15):
        buf = torch.zeros(data.size + 32, dtype=torch.uint8, device="cuda")
        view = buf[shift:shift + data.size]
        view.copy_(dev(data))
        assert view.data_ptr() % 16 == shift
        x, soff = sedd.debug_shingle_hashes(view, dev(off), 5, 0)
        assert np.array_equal(host(soff), woff) and np.array_equal(host(x), wx)


# ---- signatures ----------------------------------------------------------------------------

def _check_minhash(sedd, data, off, n, K, seed, flags, procs=1):
    want = oracle.minhash_sharded(data, off, n, K, seed, flags, procs=procs)
    got = host(sedd.sedd_minhash(dev(data), dev(off), n, K, seed, flags))
    assert got.shape == want.shape
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} documents differ, first {bad[:5]}"
    return want


@pytest.mark.parametrize("K", [1, 63, 64, 65, 100, 128, 200, 256, 300, 512, 1000])
def test_minhash_K_sweep(sedd, K):
    say("minhash K", K)
    data, off = corpus.generate(corpus.config(1).scaled(300))
    _check_minhash(sedd, data, off, 5, K, seed=K, flags=0)


@pytest.mark.parametrize("n,flags", [(1, 0), (3, 0), (5, 0), (9, 0), (1, 1), (5, 1), (13, 1), (64, 1)])
def test_minhash_edge_documents(sedd, n, flags):
    say("minhash edge", n, flags)
    data, off = _pack(_edge_corpus(), 5)
    _check_minhash(sedd, data, off, n, 128, seed=99, flags=flags)


@pytest.mark.parametrize("chunk", [1 << 12, 50_000, 0])
def test_minhash_chunk_invariance(sedd, chunk):
    say("minhash chunk", chunk)
    r = corpus.config(1).scaled(400, ws_variety=1)
    data, off = corpus.generate(r)
    sedd.debug_set_chunk_bytes(chunk)
    try:
        _check_minhash(sedd, data, off, 5, 128, 0, 0, procs=NPROC)
    finally:
        sedd.debug_set_chunk_bytes(0)


def test_minhash_long_documents_split_into_tiles(sedd):
    say("minhash long docs")
    r = corpus.Recipe("long", seed=4, n_docs=40, len_median=3000, len_sigma=1.0, len_lo=1,
                      len_hi=40000, near_frac=0.2, utf8_pct=5)
    data, off = corpus.generate(r)
    _check_minhash(sedd, data, off, 5, 128, 1, 0, procs=NPROC)
    _check_minhash(sedd, data[: int(off[12])], off[:13], 13, 128, 1, 1, procs=NPROC)


def test_minhash_zero_docs_and_repeat_determinism(sedd):
    say("minhash zero/repeat")
    out = sedd.sedd_minhash(torch.zeros(0, dtype=torch.uint8, device="cuda"),
                            dev(np.zeros(1, np.uint64)), 5, 128)
    assert tuple(out.shape) == (0, 128)
    data, off = corpus.generate(corpus.config(1).scaled(500))
    a = host(sedd.sedd_minhash(dev(data), dev(off), 5, 128))
    b = host(sedd.sedd_minhash(dev(data), dev(off), 5, 128))
    assert np.array_equal(a, b)


def test_minhash_rejects_decreasing_offsets(sedd):
    say("minhash bad offsets")
    data = dev(np.zeros(64, np.uint8))
    off = dev(np.array([0, 40, 20, 64], dtype=np.uint64))
    out = torch.full((3, 8), 7, dtype=torch.int32, device="cuda").view(torch.uint32)
    with pytest.raises(sedd.SeddError) as e:
        sedd.sedd_minhash(data, off, 5, 8, out=out)
    assert e.value.code == -1
    assert (out.view(torch.int32) == 7).all().item()          # nothing written


def test_minhash_from_x_random_and_structured(sedd):
    say("minhash from x")
    rng = np.random.default_rng(5)
    P = (1 << 61) - 1
    lens = [0, 1, 2, 1023, 1024, 1025, 5000, 0, 3]
    parts = [rng.integers(0, P, size=l, dtype=np.uint64) for l in lens]
    # limb edge values: all-ones / zero limbs, values around 2^31 and 2^60
    edge = np.array([0, 1, 2, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, (1 << 32) - 1, 1 << 32,
                     (1 << 60) - 1, 1 << 60, P - 2, P - 1, 0x1FFFFFFF80000000, 0x7FFFFFFF,
                     0x1FFFFFFFFFFFFFFE, 0x1555555555555555, 0x0AAAAAAAAAAAAAAA], dtype=np.uint64)
    parts.append(edge)
    x = np.concatenate(parts)
    off = np.cumsum([0] + [p.size for p in parts]).astype(np.uint64)
    for K, seed in [(128, 0), (64, 3), (256, 9), (100, 1)]:
        got = host(sedd.debug_minhash_from_x(dev(x), dev(off), K, seed))
        for d, p in enumerate(parts):
            assert np.array_equal(got[d], oracle.minhash_shingles(p, K, seed)), (K, seed, d)


def test_minhash_exact_path_for_values_next_to_the_modulus(sedd):
    """Shingle values chosen so that (a_k x + b_k) mod p lands within a few units of 0 or p:
    the kernel's fast evaluation cannot decide those and must take its exact path."""
    say("minhash near-modulus values")
    P = (1 << 61) - 1
    K, seed = 128, 0
    a, b = oracle.coeffs(seed, K)
    targets = [0, 1, 2, 5, 7, P - 1, P - 2, P - 5, P - (1 << 32), P - (1 << 32) - 1,
               P - (1 << 33), (1 << 32) - 1, 1 << 32]
    docs = []
    for k in (0, 1, 63, 64, 127):
        inv = pow(int(a[k]), -1, P)
        xs = [((t - int(b[k])) * inv) % P for t in targets]
        for t, xv in zip(targets, xs):
            assert (int(a[k]) * xv + int(b[k])) % P == t
        filler = np.random.default_rng(k).integers(0, P, size=200, dtype=np.uint64)
        docs.append(np.concatenate([np.array(xs, dtype=np.uint64), filler]))
        docs.append(np.array(xs[:3], dtype=np.uint64))
    x = np.concatenate(docs)
    off = np.cumsum([0] + [d.size for d in docs]).astype(np.uint64)
    before = sedd.debug_stats()[sedd.STAT_SLOW_TILES]
    got = host(sedd.debug_minhash_from_x(dev(x), dev(off), K, seed))
    after = sedd.debug_stats()[sedd.STAT_SLOW_TILES]
    for d, p in enumerate(docs):
        assert np.array_equal(got[d], oracle.minhash_shingles(p, K, seed)), d
    assert after > before, "the exact path was never taken"


# ---- band keys -----------------------------------------------------------------------------

@pytest.mark.parametrize("K,b,r", [(128, 16, 8), (128, 8, 16), (256, 32, 8), (256, 64, 4), (64, 64, 1),
                                   (40, 3, 7), (8, 1, 8), (512, 16, 8)])
def test_lsh_keys_parity(sedd, K, b, r):
    say("keys", K, b, r)
    rng = np.random.default_rng(K + b)
    sig = rng.integers(0, 1 << 32, size=(3001, K), dtype=np.uint64).astype(np.uint32)
    sig[0] = 0xFFFFFFFF
    sig[1] = 0
    got = host(sedd.sedd_lsh_keys(dev(sig), b, r))
    assert np.array_equal(got, oracle.lsh_keys(sig, b, r))


# ---- sort and clusters ---------------------------------------------------------------------

@pytest.mark.parametrize("n,b,span", [(1, 1, 10), (5, 3, 4), (4096, 2, 1 << 61), (4097, 4, 1000),
                                      (100_000, 16, (1 << 61) - 1), (33_333, 5, 1 << 20)])
def test_sort_bands(sedd, n, b, span):
    say("sort", n, b, span)
    rng = np.random.default_rng(n + b)
    keys = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    ks, ds = sedd.debug_sort_bands(dev(keys))
    ks, ds = host(ks), host(ds)
    for j in range(b):
        order = np.argsort(keys[:, j], kind="stable")
        assert np.array_equal(ds[j], order.astype(np.uint32)), j
        assert np.array_equal(ks[j], keys[order, j]), j


@pytest.mark.parametrize("n,b,span,seed", [(1, 1, 1, 0), (2, 1, 1, 1), (300, 16, 400, 3), (500, 3, 100, 4),
                                           (5000, 8, 1 << 61, 5), (20_000, 16, 30_000, 6),
                                           (100_000, 4, 150_000, 7), (50_000, 2, 3, 8),
                                           (70_000, 1, 1, 9)])
def test_cluster_random_keys(sedd, n, b, span, seed):
    say("cluster", n, b, span)
    rng = np.random.default_rng(seed)
    keys = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    got = host(sedd.sedd_cluster(dev(keys)))
    assert np.array_equal(got, oracle.cluster(keys))


@pytest.mark.parametrize("n,b", [(3000, 3), (70_000, 2)])
def test_cluster_keys_that_agree_in_their_low_bits(sedd, n, b):
    """Few distinct low words, several high words: records with different keys interleave
    inside every group of equal low bits, which is what the grouping sort leaves to the linker."""
    say("cluster low-bit collisions", n, b)
    rng = np.random.default_rng(n)
    lo = rng.integers(0, 40, size=(n, b), dtype=np.uint64)
    hi = rng.integers(0, 6, size=(n, b), dtype=np.uint64)
    keys = (hi << np.uint64(45)) | (lo << np.uint64(3)) | (hi & np.uint64(1))
    assert np.array_equal(host(sedd.sedd_cluster(dev(keys))), oracle.cluster(keys))
    # and spread out so that most keys are singletons but some collide only in the low 32 bits
    base = rng.integers(0, 1 << 32, size=(n, b), dtype=np.uint64)
    keys = base | (rng.integers(0, 3, size=(n, b), dtype=np.uint64) << np.uint64(50))
    keys[n // 2:] = keys[: n - n // 2] ^ (rng.integers(0, 2, size=(n - n // 2, b), dtype=np.uint64) << np.uint64(50))
    assert np.array_equal(host(sedd.sedd_cluster(dev(keys))), oracle.cluster(keys))


def test_cluster_long_chain_across_bands(sedd):
    say("cluster chain")
    # doc i shares band (i % 2) with doc i+1: one component threaded through two bands
    n = 30_000
    keys = np.zeros((n, 2), dtype=np.uint64)
    idx = np.arange(n, dtype=np.uint64)
    keys[:, 0] = (idx + 1) // 2 + 10 * n
    keys[:, 1] = idx // 2 + 20 * n
    want = oracle.cluster(keys)
    assert (want == 0).all()
    assert np.array_equal(host(sedd.sedd_cluster(dev(keys))), want)
    perm = np.random.default_rng(0).permutation(n)
    assert np.array_equal(host(sedd.sedd_cluster(dev(keys[perm]))), oracle.cluster(keys[perm]))


@pytest.mark.parametrize("kind", ["shifted", "seven_high_values", "uniform"])
def test_cluster_keys_with_constant_low_bits_at_200k(sedd, kind):
    """Keys whose low bits say nothing (d << 32: all distinct, all zero below bit 32; a few high
    values over a small low part: large groups of interleaved buckets).  The grouping sort
    cannot separate them; the calls must notice, sort by the whole key, and still finish in
    milliseconds with the oracle's clusters.  Uniform keys must not take that detour."""
    say("cluster constant low bits", kind)
    n, b = 200_000, 4
    rng = np.random.default_rng(7)
    d = np.arange(n, dtype=np.uint64)
    if kind == "shifted":
        keys = np.stack([(d << np.uint64(32)), ((d // np.uint64(3)) << np.uint64(32)),
                         ((d % np.uint64(50_000)) << np.uint64(29)), d << np.uint64(40)], axis=1)
    elif kind == "seven_high_values":
        c = rng.integers(0, 200, size=(n, b), dtype=np.uint64)
        keys = ((d % np.uint64(7))[:, None] << np.uint64(40)) | c
    else:
        keys = rng.integers(0, (1 << 61) - 1, size=(n, b), dtype=np.uint64)
        keys[n // 2:, 0] = keys[: n // 2, 0]                  # some real duplicates
    keys = np.ascontiguousarray(keys)
    want = oracle.cluster(keys)
    d_keys = dev(keys)
    sedd.sedd_cluster(d_keys)                                # first call pays the allocation
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    got = sedd.sedd_cluster(d_keys)
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0)
    regroup = sedd.debug_last_regroup()
    assert np.array_equal(host(got), want)
    say(f"  {kind}: {ms:.2f} ms, whole-key sort: {regroup}")
    if kind != "seven_high_values":                          # there the walks may all stay short
        assert regroup == (0 if kind == "uniform" else 1)
    assert ms < 200, f"sedd_cluster took {ms:.1f} ms on 200k x 4 records"
    # the verified call on the same keys: threshold 0 is plain bucket grouping, K + 1 links nothing
    sig = rng.integers(0, 1 << 32, size=(n, 8), dtype=np.uint64).astype(np.uint32)
    sig[n // 2:] = sig[: n // 2]
    d_sig = dev(sig)
    for mm in (0, 8, 9):
        t0 = time.perf_counter()
        vgot = sedd.sedd_cluster_verified(d_keys, d_sig, mm)
        torch.cuda.synchronize()
        vms = 1e3 * (time.perf_counter() - t0)
        vre = sedd.debug_last_regroup()
        assert np.array_equal(host(vgot), oracle.cluster_verified(keys, sig, mm)), mm
        assert vms < 2000, f"sedd_cluster_verified took {vms:.1f} ms"
    say(f"  {kind}: verified {vms:.2f} ms, whole-key sort: {vre}")
    assert vre == (0 if kind == "uniform" else 1)


def test_cluster_on_caller_workspaces_and_two_streams(sedd):
    """sedd_cluster_ws / sedd_cluster_verified_ws: same results as the arena calls, with a
    misaligned workspace, and two calls in flight on two streams with a workspace each."""
    say("cluster workspaces")
    rng = np.random.default_rng(12)
    cases = []
    for n, b, K in ((30_000, 8, 32), (50_000, 4, 16)):
        keys = rng.integers(0, n // 2, size=(n, b), dtype=np.uint64)
        proto = rng.integers(0, 1 << 32, size=(50, K), dtype=np.uint64).astype(np.uint32)
        sig = proto[rng.integers(0, 50, size=n)].copy()
        noise = rng.random((n, K)) < 0.15
        sig[noise] = rng.integers(0, 1 << 32, size=int(noise.sum()), dtype=np.uint64).astype(np.uint32)
        cases.append((keys, sig, K))
    arena_before = sedd.sedd_scratch_bytes()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for (keys, sig, K), st in zip(cases, streams):
        n, b = keys.shape
        need_c = sedd.sedd_cluster_workspace_bytes(n, b)
        need_v = sedd.sedd_cluster_workspace_bytes(n, b, K)
        ws_c = torch.empty(need_c + 3, dtype=torch.uint8, device="cuda")[3:]     # misaligned on purpose
        ws_v = torch.empty(need_v, dtype=torch.uint8, device="cuda")
        d_keys, d_sig = dev(keys), dev(sig)
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            c = sedd.sedd_cluster_ws(d_keys, ws_c[: need_c], stream=st)
            v = sedd.sedd_cluster_ws(d_keys, ws_v, sig=d_sig, min_match=K - 6, stream=st)
        outs.append((c, v, ws_c, ws_v, d_keys, d_sig))
    torch.cuda.synchronize()
    assert sedd.sedd_scratch_bytes() == arena_before            # the arena was not used
    for (keys, sig, K), (c, v, *_rest) in zip(cases, outs):
        assert np.array_equal(host(c), oracle.cluster(keys))
        assert np.array_equal(host(v), oracle.cluster_verified(keys, sig, K - 6))
    keys, sig, K = cases[0]
    small = torch.empty(1000, dtype=torch.uint8, device="cuda")
    with pytest.raises(sedd.SeddError) as e:
        sedd.sedd_cluster_ws(dev(keys), small)
    assert e.value.code == -4


def test_enomem_leaves_outputs_untouched_and_the_next_call_works(sedd):
    say("scratch cap -> ENOMEM")
    rng = np.random.default_rng(13)
    keys = rng.integers(0, 5000, size=(20_000, 4), dtype=np.uint64)
    d_keys = dev(keys)
    out = torch.full((20_000,), -5, dtype=torch.int64, device="cuda")
    sedd.debug_set_scratch_cap(4096)
    try:
        with pytest.raises(sedd.SeddError) as e:
            sedd.sedd_cluster(d_keys, out=out)
        assert e.value.code == -2
        torch.cuda.synchronize()
        assert bool((out == -5).all())
        data, off = corpus.generate(corpus.config(1).scaled(200))
        sig = torch.full((200, 16), 9, dtype=torch.int32, device="cuda").view(torch.uint32)
        with pytest.raises(sedd.SeddError) as e:
            sedd.sedd_minhash(dev(data), dev(off), 13, 16, 0, 1, out=sig)      # byte shingles: chunk scratch
        assert e.value.code == -2
        torch.cuda.synchronize()
        assert bool((sig.view(torch.int32) == 9).all())
    finally:
        sedd.debug_set_scratch_cap(0)
    assert np.array_equal(host(sedd.sedd_cluster(d_keys, out=out)), oracle.cluster(keys))


# ---- the whole path ------------------------------------------------------------------------

def _full_path(sedd, recipe, procs):
    data, off = corpus.generate(recipe)
    flags = int(recipe.byte_mode)
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


def test_config1_whole_path(sedd):
    say("config 1 whole path")
    cid = _full_path(sedd, corpus.config(1), NPROC)
    dups = int((cid != np.arange(cid.size)).sum())
    # 10 % planted near-duplicates at a 5 % word edit rate: Jaccard of 5-grams is about 0.6,
    # where the (16, 8) collision curve catches a bit under half of them
    assert 100 <= dups <= 500


def test_config3_shape_small(sedd):
    say("config 3 shape (scaled)")
    _full_path(sedd, corpus.config(3).scaled(3000), NPROC)


def test_config4_shape_small(sedd):
    say("config 4 shape (scaled)")
    r = corpus.config(4).scaled(1500, long_lo=20_000, long_hi=200_000)
    _full_path(sedd, r, NPROC)


@pytest.mark.parametrize("K,b,r,n", [(64, 8, 8, 3), (128, 8, 16, 5), (256, 32, 8, 3), (512, 64, 4, 5),
                                     (256, 64, 4, 3)])
def test_config5_sweep_points_small(sedd, K, b, r, n):
    say("config 5 point", K, b, r, n)
    _full_path(sedd, corpus.config(5).scaled(1500, K=K, b=b, r=r, shingle_n=n), NPROC)


# ---- full-size workload, in the launch configuration bench.py times -------------------------

def test_config2_full_size_whole_path(sedd):
    """1M documents, 2.6 GB of text: every signature, band key and cluster id against the
    oracle (run as NPROC processes over disjoint document ranges)."""
    say("config 2 at full size: generating")
    r = corpus.config(2)
    data, off = corpus.generate(r)
    say("config 2: oracle on", NPROC, "processes")
    wsig = oracle.minhash_sharded(data, off, r.shingle_n, r.K, 0, 0, procs=NPROC)
    wkeys = oracle.lsh_keys(wsig, r.b, r.r)
    wcid = oracle.cluster(wkeys)
    say("config 2: GPU")
    d_data, d_off = dev(data), dev(off)
    sig = sedd.sedd_minhash(d_data, d_off, r.shingle_n, r.K, 0, 0)
    keys = sedd.sedd_lsh_keys(sig, r.b, r.r)
    cid = sedd.sedd_cluster(keys)
    bad = np.nonzero((host(sig) != wsig).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} signatures differ, first {bad[:5]}"
    assert np.array_equal(host(keys), wkeys)
    assert np.array_equal(host(cid), wcid)
    say("config 2: verified clusters")
    mm = oracle.min_match_for(0.8, r.K)
    wv = oracle.cluster_verified(wkeys, wsig, mm)
    assert np.array_equal(host(sedd.sedd_cluster_verified(keys, sig, mm)), wv)
    say("config 2: verified duplicates", int((wv != np.arange(wv.size)).sum()))
    # second call on the same buffers: identical bytes (scratch reuse, atomics, exact path)
    sig2 = sedd.sedd_minhash(d_data, d_off, r.shingle_n, r.K, 0, 0)
    assert torch.equal(sig.view(torch.int32), sig2.view(torch.int32))
    dups = int((wcid != np.arange(wcid.size)).sum())
    say("config 2: duplicates found", dups)
    assert 20_000 <= dups <= 150_000


# ---- verified clusters (Section 3.3) ---------------------------------------------------------

def _proto_case(seed, n, K, b, span, groups, noise=0.6):
    """Signatures scattered around a few prototypes (match counts spread over 0..K) and keys
    from a small range (buckets of several documents, unrelated to the signatures)."""
    rng = np.random.default_rng(seed)
    proto = rng.integers(0, 1 << 32, size=(groups, K), dtype=np.uint64).astype(np.uint32)
    sig = proto[rng.integers(0, groups, size=n)].copy()
    flip = rng.random((n, K)) < rng.random((n, 1)) * noise
    sig[flip] = rng.integers(0, 1 << 32, size=int(flip.sum()), dtype=np.uint64).astype(np.uint32)
    keys = rng.integers(0, span, size=(n, b), dtype=np.uint64)
    return keys, sig


@pytest.mark.parametrize("seed,n,K,b,span,groups", [
    (0, 1, 8, 1, 1, 1), (1, 2, 8, 1, 1, 1), (2, 500, 16, 3, 60, 4), (3, 3000, 32, 4, 400, 6),
    (4, 2000, 128, 16, 700, 5), (5, 1500, 7, 2, 30, 2), (6, 4000, 130, 5, 500, 8),
    (7, 5000, 256, 32, 3000, 10)])
def test_cluster_verified_random_buckets(sedd, seed, n, K, b, span, groups):
    say("verified random", seed, n, K, b)
    keys, sig = _proto_case(seed, n, K, b, span, groups)
    d_keys, d_sig = dev(keys), dev(sig)
    for mm in sorted({0, 1, K // 2, oracle.min_match_for(0.8, K), K, K + 1}):
        got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
        assert np.array_equal(got, oracle.cluster_verified(keys, sig, mm)), mm
    assert np.array_equal(host(sedd.sedd_cluster_verified(d_keys, d_sig, 0)),
                          host(sedd.sedd_cluster(d_keys)))


def test_cluster_verified_large_buckets(sedd):
    """One bucket holding every document: identical signatures (no second step needed), two
    interleaved groups, and unrelated signatures (every record ends up compared with all)."""
    say("verified large buckets")
    rng = np.random.default_rng(1)
    n, K = 1200, 64
    keys = np.zeros((n, 2), dtype=np.uint64)
    keys[:, 1] = np.arange(n)
    same = np.tile(rng.integers(0, 1 << 32, size=K, dtype=np.uint64).astype(np.uint32), (n, 1))
    two = same.copy()
    two[1::2] = rng.integers(0, 1 << 32, size=K, dtype=np.uint64).astype(np.uint32)
    rand = rng.integers(0, 1 << 32, size=(n, K), dtype=np.uint64).astype(np.uint32)
    chain = np.zeros((n, K), dtype=np.uint32)
    for i in range(n):                      # document i agrees with i-1 on K-1 entries only
        chain[i] = np.arange(K) + 1000 * ((i + np.arange(K)) // K)
    for name, sig, mm in (("same", same, K), ("two", two, K), ("rand", rand, 1),
                          ("chain", chain, K - 1), ("chain", chain, K - 8)):
        want = oracle.cluster_verified(keys, sig, mm)
        got = host(sedd.sedd_cluster_verified(dev(keys), dev(sig), mm))
        assert np.array_equal(got, want), (name, mm)
    assert oracle.cluster_verified(keys, two, K).tolist()[:4] == [0, 1, 0, 1]


@pytest.mark.parametrize("K", [1, 31, 33, 100, 130, 300, 1000])
def test_cluster_verified_large_buckets_sketch_bound(sedd, K):
    """Buckets of hundreds of documents go through the sketch-bounded tile kernel: signature
    lengths around the 32-entry sketch words and beyond one staging pass, prototypes with noise
    (match counts spread over 0..K), and signatures whose lowest bits all agree, where the bound
    rules nothing out and every pair has to be counted."""
    say("verified sketch bound", K)
    rng = np.random.default_rng(K)
    n, b = 700, 3
    keys = rng.integers(0, 3, size=(n, b), dtype=np.uint64)             # buckets of ~230
    _, sig = _proto_case(K, n, K, b, 3, 6, noise=0.5)
    even = (sig & np.uint32(0xFFFFFFFE)).astype(np.uint32)               # all sketch bits zero
    odd_rows = sig.copy()
    odd_rows[::2] |= np.uint32(1)                                        # half the documents all-ones sketches
    odd_rows[1::2] &= np.uint32(0xFFFFFFFE)
    for name, sg in (("noise", sig), ("even", even), ("halves", odd_rows)):
        d_keys, d_sig = dev(keys), dev(sg)
        for mm in sorted({0, 1, max(1, K // 2), oracle.min_match_for(0.8, K), K, K + 1}):
            got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
            assert np.array_equal(got, oracle.cluster_verified(keys, sg, mm)), (name, mm)


@pytest.mark.parametrize("K,sizes", [
    (256, (65, 127, 128, 129, 191, 192, 193, 319, 320, 321, 639, 640, 641, 895, 896, 897, 1100, 1343, 1344, 1345)),
    (128, (255, 256, 257, 319, 320, 321, 1023, 1024, 1025, 1151, 1152, 1153, 1343, 1344, 1345)),
    (1000, (64, 65, 191, 192, 193, 383, 384, 385, 500, 895, 896, 897))])
def test_cluster_verified_bucket_sizes_at_the_limits_of_the_three_kernels(sedd, K, sizes):
    """Buckets of more than 64 documents are compared from LDS by one wavefront, from LDS by four,
    or tile by tile from memory, depending on how many records fit LDS next to the sketch words
    kept there, which in turn depends on the threshold: bucket sizes at and next to those limits
    for three signature lengths and the thresholds used below, with related documents spread over
    the tiles of every bucket."""
    say("verified bucket sizes", K, sizes)
    rng = np.random.default_rng(K)
    n = int(sum(sizes))
    band0 = np.repeat(np.arange(len(sizes), dtype=np.uint64), sizes)
    rng.shuffle(band0)
    keys = np.stack([band0 * np.uint64(1_000_003) + np.uint64(17),
                     rng.integers(0, n // 3, size=n, dtype=np.uint64)], axis=1)
    _, sig = _proto_case(K + 1, n, K, 2, 3, max(8, n // 40), noise=0.35)
    d_keys, d_sig = dev(keys), dev(sig)
    for mm in (oracle.min_match_for(0.8, K), oracle.min_match_for(0.95, K), K // 2, 1):
        got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
        want = oracle.cluster_verified(keys, sig, mm)
        assert np.array_equal(got, want), (mm, int((got != want).sum()))
        if mm == oracle.min_match_for(0.8, K):                 # the buckets do hold related documents
            assert n // 10 < int((want != np.arange(n)).sum()) < n


def test_cluster_verified_buckets_of_copies_with_strangers(sedd):
    """Buckets that are mostly copies of one document with unrelated documents mixed in (and one
    with two families of copies): the tiles that hold a stranger cannot be skipped, and nearly all
    of their pairs pass the sketch bound."""
    say("verified copies with strangers")
    rng = np.random.default_rng(77)
    K, sizes = 256, (800, 500, 130, 896)
    n = int(sum(sizes))
    band0 = np.repeat(np.arange(len(sizes), dtype=np.uint64), sizes)
    sig = rng.integers(0, 1 << 32, size=(n, K), dtype=np.uint64).astype(np.uint32)
    start = 0
    for gi, s in enumerate(sizes):
        idx = np.arange(start, start + s)
        copies = idx[rng.random(s) < 0.85]
        if gi == 1:                                    # two families
            half = copies.size // 2
            sig[copies[:half]] = sig[copies[0]]
            sig[copies[half:]] = sig[copies[half]]
        else:
            sig[copies] = sig[copies[0]]
        near = copies[rng.random(copies.size) < 0.1]   # some copies with a few entries changed
        for d in near:
            sig[d, rng.integers(0, K, size=20)] = rng.integers(0, 1 << 32, size=20, dtype=np.uint64).astype(np.uint32)
        start += s
    perm = rng.permutation(n)
    band0, sig = band0[perm], sig[perm]
    keys = np.stack([band0 + np.uint64(5), rng.integers(0, n, size=n, dtype=np.uint64)], axis=1)
    d_keys, d_sig = dev(keys), dev(sig)
    for mm in (oracle.min_match_for(0.8, K), K, 1):
        got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
        assert np.array_equal(got, oracle.cluster_verified(keys, sig, mm)), mm


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_fuzz_cluster_verified(sedd, seed):
    """Random mixes of bucket sizes (single documents up to buckets beyond what LDS holds), band
    counts, key magnitudes, signature lengths, noise levels and thresholds; sometimes all sketch
    bits equal, so that the bound rules nothing out."""
    say("fuzz verified", seed)
    rng = np.random.default_rng(seed)
    for case in range(14):
        K = int(rng.choice([1, 7, 32, 33, 64, 100, 128, 200, 256, 300, 512, 777, 1024]))
        b = int(rng.integers(1, 6))
        sizes = rng.choice([1, 2, 5, 40, 63, 64, 65, 100, 130, 200, 333, 500, 700, 900, 1300],
                           size=int(rng.integers(1, 8)))
        n = int(sizes.sum())
        band0 = np.repeat(np.arange(sizes.size, dtype=np.uint64), sizes)
        rng.shuffle(band0)
        keys = np.empty((n, b), dtype=np.uint64)
        keys[:, 0] = band0 * np.uint64(rng.choice([1, 1 << 20, 1 << 40, 999_983])) + np.uint64(3)
        for j in range(1, b):
            keys[:, j] = rng.integers(0, max(1, n // int(rng.choice([1, 3, 50]))), size=n, dtype=np.uint64)
        protos = max(1, n // int(rng.choice([5, 30, 200])))
        proto = rng.integers(0, 1 << 32, size=(protos, K), dtype=np.uint64).astype(np.uint32)
        sig = proto[rng.integers(0, protos, size=n)].copy()
        flip = rng.random((n, K)) < rng.random((n, 1)) * float(rng.choice([0.0, 0.2, 0.5]))
        sig[flip] = rng.integers(0, 1 << 32, size=int(flip.sum()), dtype=np.uint64).astype(np.uint32)
        if rng.random() < 0.3:
            sig &= np.uint32(0xFFFFFFFE)
        d_keys, d_sig = dev(keys), dev(sig)
        for mm in sorted({0, 1, K // 2, oracle.min_match_for(0.8, K), oracle.min_match_for(0.95, K), K, K + 1}):
            got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
            want = oracle.cluster_verified(keys, sig, mm)
            assert np.array_equal(got, want), (case, K, b, sizes.tolist(), mm)


@pytest.mark.parametrize("strangers,whole_key_sort", [(4, 0), (60, 1)])
def test_cluster_verified_large_buckets_with_strangers_in_their_group(sedd, strangers, whole_key_sort):
    """Large buckets whose sorted group also holds records of another key (equal below the sorted
    bits).  A few: too few to make the call sort by the whole key, so the large-group kernels
    meet pairs with different keys and must leave them alone.  Many: the call sorts by the whole
    key first.  The clusters are the oracle's either way."""
    say("verified strangers in large groups", strangers)
    rng = np.random.default_rng(41)
    n, K, b = 120_000, 64, 4
    sizes = (70, 200, 600, 3000)                       # one-wavefront, four-wavefront and tiled groups
    lo = rng.integers(0, 1 << 61, size=(n, b), dtype=np.uint64) & np.uint64((1 << 61) - 1)
    sig = rng.integers(0, 1 << 32, size=(n, K), dtype=np.uint64).astype(np.uint32)
    at = 0
    for band in range(b):
        for gi, s in enumerate(sizes):
            idx = np.arange(at, at + s)
            at += s
            key = np.uint64(1000 * band + gi + 1)
            lo[idx, band] = key
            fam = idx[rng.random(s) < 0.7]             # a family of near copies inside the bucket
            sig[fam] = sig[fam[0]]
            sig[fam[::3], :6] = rng.integers(0, 1 << 32, size=(fam[::3].size, 6), dtype=np.uint64).astype(np.uint32)
            # strangers: same low bits, another key; two of them copies of the family's document
            odd = idx[rng.choice(s, size=min(strangers, s // 3), replace=False)]
            lo[odd, band] = key | np.uint64(1 << 50)
            sig[odd[:2]] = sig[fam[0]]
    perm = rng.permutation(n)
    keys, sig = np.ascontiguousarray(lo[perm]), sig[perm]
    d_keys, d_sig = dev(keys), dev(sig)
    for mm in (oracle.min_match_for(0.8, K), K, 0):
        got = host(sedd.sedd_cluster_verified(d_keys, d_sig, mm))
        assert sedd.debug_last_regroup() == whole_key_sort   # 0: the strangers stayed in their groups
        assert np.array_equal(got, oracle.cluster_verified(keys, sig, mm)), mm


def test_cluster_verified_keys_that_agree_in_their_low_bits(sedd):
    """Buckets whose keys differ only above the sorted bits share one sorted group."""
    say("verified low-bit collisions")
    rng = np.random.default_rng(2)
    n, K, b = 4000, 32, 3
    lo = rng.integers(0, 50, size=(n, b), dtype=np.uint64)
    hi = rng.integers(0, 4, size=(n, b), dtype=np.uint64)
    keys = (hi << np.uint64(45)) | lo
    _, sig = _proto_case(3, n, K, b, 10, 5, noise=0.3)
    for mm in (0, 20, 26, 32):
        got = host(sedd.sedd_cluster_verified(dev(keys), dev(sig), mm))
        assert np.array_equal(got, oracle.cluster_verified(keys, sig, mm)), mm


@pytest.mark.parametrize("cfg,docs", [(1, 5000), (3, 3000), (4, 1500)])
def test_cluster_verified_on_corpora(sedd, cfg, docs):
    say("verified on corpus", cfg)
    r = corpus.config(cfg).scaled(docs) if cfg != 4 else \
        corpus.config(4).scaled(docs, long_lo=20_000, long_hi=100_000)
    data, off = corpus.generate(r)
    flags = int(r.byte_mode)
    wsig = oracle.minhash_sharded(data, off, r.shingle_n, r.K, 0, flags, procs=NPROC)
    wkeys = oracle.lsh_keys(wsig, r.b, r.r)
    sig = sedd.sedd_minhash(dev(data), dev(off), r.shingle_n, r.K, 0, flags)
    keys = sedd.sedd_lsh_keys(sig, r.b, r.r)
    for theta in (0.5, 0.8, 0.95):
        mm = sedd.min_match_for(theta, r.K)
        assert mm == oracle.min_match_for(theta, r.K)
        got = host(sedd.sedd_cluster_verified(keys, sig, mm))
        assert np.array_equal(got, oracle.cluster_verified(wkeys, wsig, mm)), theta


def test_all_pairs_reference_of_the_fidelity_figure_on_config1(sedd):
    """The fidelity figure (Section 4.3) compares LSH + verification with brute-force all-pairs
    comparison of the same signatures; the brute force is sedd_cluster_verified on one key
    column that is equal for every document.  Both sides against the oracle on workload 1."""
    say("fidelity reference on config 1")
    r = corpus.config(1)
    data, off = corpus.generate(r)
    wsig = oracle.minhash_sharded(data, off, r.shingle_n, r.K, 0, 0, procs=NPROC)
    sig = sedd.sedd_minhash(dev(data), dev(off), r.shingle_n, r.K)
    mm = sedd.min_match_for(0.8, r.K)
    ones = np.zeros((r.n_docs, 1), dtype=np.uint64)
    want_all = oracle.cluster_verified(ones, wsig, mm)
    got_all = host(sedd.sedd_cluster_verified(dev(ones), sig, mm))
    assert np.array_equal(got_all, want_all)
    want_lsh = oracle.cluster_verified(oracle.lsh_keys(wsig, r.b, r.r), wsig, mm)
    got_lsh = host(sedd.sedd_cluster_verified(sedd.sedd_lsh_keys(sig, r.b, r.r), sig, mm))
    assert np.array_equal(got_lsh, want_lsh)
    ident = np.arange(r.n_docs)
    a, b_ = set(np.nonzero(got_lsh != ident)[0]), set(np.nonzero(got_all != ident)[0])
    assert a <= b_ and len(b_) > 0            # LSH can only miss pairs, never add them
    say(f"  duplicates: LSH + verification {len(a)}, all pairs {len(b_)}, "
        f"set-Jaccard {len(a & b_) / len(a | b_):.4f}")


def test_cluster_verified_rejects_bad_arguments(sedd):
    keys = dev(np.zeros((4, 2), np.uint64))
    sig = dev(np.zeros((4, 8), np.uint32))
    with pytest.raises(sedd.SeddError):
        sedd.sedd_cluster_verified(keys, sig, -1)
    with pytest.raises(ValueError):
        sedd.sedd_cluster_verified(keys, sig[:3], 1)


# ---- dense buckets (Section 3.2) and the tiled count-match path -------------------------------

@pytest.mark.parametrize("K,b,r,nb", [(128, 16, 8, 4000), (64, 64, 1, 7), (40, 3, 7, 1),
                                      (256, 32, 8, 12649), (16, 1, 16, (1 << 40) + 5)])
def test_lsh_dense_keys_parity(sedd, K, b, r, nb):
    say("dense keys", K, b, r, nb)
    rng = np.random.default_rng(K + b)
    sig = rng.integers(0, 1 << 32, size=(3001, K), dtype=np.uint64).astype(np.uint32)
    sig[0] = 0xFFFFFFFF
    sig[1] = 0
    got = host(sedd.sedd_lsh_dense_keys(dev(sig), b, r, nb))
    assert np.array_equal(got, oracle.lsh_dense_keys(sig, b, r, nb))


def _planted_signatures(seed, n, K, n_dup, keep=0.9):
    rng = np.random.default_rng(seed)
    sig = rng.integers(0, 1 << 32, size=(n, K), dtype=np.uint64).astype(np.uint32)
    src = rng.choice(n // 2, size=n_dup, replace=False)
    dup = n // 2 + np.arange(n_dup)
    noisy = rng.random((n_dup, K)) >= keep
    sig[dup] = np.where(noisy, rng.integers(0, 1 << 32, size=(n_dup, K), dtype=np.uint64).astype(np.uint32),
                        sig[src])
    return sig


@pytest.mark.parametrize("n,K,b,r,k_buckets", [(6000, 64, 8, 8, 4), (40_000, 32, 4, 8, 1),
                                               (100_000, 64, 8, 8, 4), (30_000, 100, 5, 20, 2)])
def test_dense_buckets_then_verified_clusters(sedd, n, K, b, r, k_buckets):
    """The paper's own flow: coarse buckets of tens to hundreds of documents, all pairs inside
    a bucket compared on the full signatures."""
    say("dense + verified", n, K, b, r, k_buckets)
    sig = _planted_signatures(n, n, K, n // 20)
    nb = oracle.dense_bucket_count(n, k_buckets)
    wkeys = oracle.lsh_dense_keys(sig, b, r, nb)
    d_sig = dev(sig)
    keys = sedd.sedd_lsh_dense_keys(d_sig, b, r, nb)
    assert np.array_equal(host(keys), wkeys)
    for theta in (0.8, 0.5):
        mm = oracle.min_match_for(theta, K)
        got = host(sedd.sedd_cluster_verified(keys, d_sig, mm))
        want = oracle.cluster_verified(wkeys, sig, mm)
        assert np.array_equal(got, want), theta
    say("  buckets", nb, "mean size", n / nb, "duplicates", int((want != np.arange(n)).sum()))


def test_verified_clusters_mixed_small_and_large_groups(sedd):
    """Buckets of 1 to 400 documents in one call; signatures from a few prototypes so that many
    pairs verify, some chains form and some large groups are entirely alike."""
    say("verified mixed group sizes")
    rng = np.random.default_rng(5)
    sizes = np.concatenate([rng.integers(1, 8, size=300), rng.integers(60, 70, size=10),
                            rng.integers(100, 400, size=6), [65, 64, 63, 128, 129, 1]])
    n = int(sizes.sum())
    keys = np.zeros((n, 2), dtype=np.uint64)
    keys[:, 0] = np.repeat(np.arange(sizes.size), sizes) * 7919
    keys[:, 1] = rng.integers(0, n // 3, size=n)
    perm = rng.permutation(n)
    keys = keys[perm]
    K = 48
    proto = rng.integers(0, 1 << 32, size=(12, K), dtype=np.uint64).astype(np.uint32)
    sig = proto[rng.integers(0, 12, size=n)].copy()
    flip = rng.random((n, K)) < rng.random((n, 1)) * 0.5
    sig[flip] = rng.integers(0, 1 << 32, size=int(flip.sum()), dtype=np.uint64).astype(np.uint32)
    for mm in (0, 24, 39, 48):
        got = host(sedd.sedd_cluster_verified(dev(keys), dev(sig), mm))
        assert np.array_equal(got, oracle.cluster_verified(keys, sig, mm)), mm


# ---- seeded fuzz of tokenisation and shingling ------------------------------------------------

def _fuzz_docs(seed, n_docs):
    """Documents over a small alphabet rich in every whitespace byte, with lengths that put
    token and document boundaries at all offsets relative to the 16-byte segments and 1 KiB
    tiles the kernels work in; some long tokens, some empty and whitespace-only documents."""
    rng = np.random.default_rng(seed)
    alphabet = np.frombuffer(b"ab\xc3\xa9z0\x00\x7f\xff \t\n\r\x0b\x0c  ", dtype=np.uint8)
    docs = []
    for _ in range(n_docs):
        kind = rng.integers(0, 10)
        if kind == 0:
            docs.append(b"")
        elif kind == 1:
            docs.append(bytes(rng.choice(alphabet[-8:], size=int(rng.integers(1, 40)))))
        elif kind == 2:                                  # long tokens, up to 3 KiB
            parts = [bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8))
                     for l in rng.integers(1, 3000, size=int(rng.integers(1, 4)))]
            docs.append(b" ".join(parts))
        else:
            ln = int(rng.integers(1, 2500))
            docs.append(bytes(rng.choice(alphabet, size=ln)))
    return docs


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_fuzz_shingle_hashes_and_signatures(sedd, seed):
    say("fuzz", seed)
    docs = _fuzz_docs(seed, 400)
    data, off = _pack(docs, lead=seed % 16)
    d_data, d_off = dev(data), dev(off)
    for byte_mode, n in ((False, 1), (False, 3), (False, 5), (True, 1), (True, 4), (True, 13)):
        wx, woff = _oracle_x(docs, n, byte_mode)
        x, soff = sedd.debug_shingle_hashes(d_data, d_off, n, int(byte_mode))
        assert np.array_equal(host(soff), woff), (byte_mode, n)
        assert np.array_equal(host(x), wx), (byte_mode, n)
        want = oracle.minhash(data, off, n, 24, seed, int(byte_mode))
        got = host(sedd.sedd_minhash(d_data, d_off, n, 24, seed, int(byte_mode)))
        bad = np.nonzero((got != want).any(axis=1))[0]
        assert bad.size == 0, (byte_mode, n, bad[:5])


def _piece_edge_docs():
    """Documents built to put every special case of the streaming kernel on a boundary between
    two wavefronts' pieces of the text (pieces are multiples of 1 KiB): documents of fewer than n
    tokens that cross one or several pieces (a giant first token, giant whitespace runs before,
    between and after the tokens), tokens that straddle a boundary, a document whose last few
    tokens spill into the next piece, documents that end exactly on a boundary, empty documents
    on a boundary, whitespace-only documents longer than a piece."""
    rng = np.random.default_rng(17)

    def word(l):
        return bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8))
    docs = []
    docs.append(word(3000) + b" " + word(5) + b" " + word(7))              # 3 tokens, first is giant
    docs.append(b" " * 2500 + word(4) + b" " * 3000 + word(6) + b"\n" * 1500)   # 2 tokens, far apart
    docs.append(word(2) + b" " * 5000)                                      # 1 token then whitespace
    docs.append(b" " * 5000 + word(3))                                      # whitespace then 1 token
    docs.append(b" " * 7000)                                                # nothing, several pieces
    docs.append(b"")
    docs.append(word(1024))                                                 # exactly one tile, one token
    docs.append(b"")
    docs.append(b"")
    docs.append(b" ".join(word(l) for l in rng.integers(1, 9, size=900)))   # ordinary, crosses pieces
    docs.append(word(700) + b" " + word(700) + b" " + word(700) + b" " + word(700))  # 4 tokens < n = 5
    docs.append(word(700) + b" " + word(700) + b" " + word(700) + b" " + word(700) + b" " + word(2))
    docs.append(word(10) + b" " * 1013 + word(1) + b" " + word(2) + b" " + word(3) + b" " + word(4))
    for total in (1024, 2048, 1023, 1025):                                  # end on / next to a boundary
        body = b" ".join(word(l) for l in rng.integers(1, 9, size=400))
        docs.append(body[:total])
    docs.append(word(70_000))                                               # one token, dozens of pieces
    docs.append(word(5) + b" " + word(70_000) + b" " + word(5))
    return docs


@pytest.mark.parametrize("piece", [1024, 2048, 5120, 16384, 1 << 20])
def test_stream_kernel_piece_size_invariance(sedd, piece):
    """Results never depend on how the text is cut between wavefronts: shingle hashes in order
    and signatures against the oracle for pieces from one tile to more than the whole text,
    with different amounts of text in front of the first document."""
    say("stream piece", piece)
    sedd.debug_set_piece_bytes(piece)
    try:
        for lead in (0, 9, 1019):
            docs = _piece_edge_docs() + (_edge_corpus() if lead == 9 else []) + _fuzz_docs(piece + lead, 60)
            data, off = _pack(docs, lead)
            d_data, d_off = dev(data), dev(off)
            for n in (1, 2, 5, 7, 64):
                wx, woff = _oracle_x(docs, n, False)
                x, soff = sedd.debug_shingle_hashes(d_data, d_off, n, 0)
                assert np.array_equal(host(soff), woff), (lead, n)
                assert np.array_equal(host(x), wx), (lead, n)
            for n, K in ((5, 128), (3, 256), (1, 40), (9, 64), (64, 32)):
                want = oracle.minhash(data, off, n, K, 3, 0)
                got = host(sedd.sedd_minhash(d_data, d_off, n, K, 3, 0))
                bad = np.nonzero((got != want).any(axis=1))[0]
                assert bad.size == 0, (lead, n, K, bad[:5])
    finally:
        sedd.debug_set_piece_bytes(0)


@pytest.mark.parametrize("max_len", [8, 9, 12, 15, 16, 17, 40])
def test_stream_kernel_token_length_tiers(sedd, max_len):
    """The token hash has a path for rounds of tokens of at most 8 bytes, one for at most 16 and
    a general one: corpora whose longest word is exactly at and around those limits, with all
    byte values (UTF-8 letters, control characters) inside the words."""
    say("stream token lengths up to", max_len)
    rng = np.random.default_rng(max_len)
    pool = np.array([c for c in range(256) if c not in (9, 10, 11, 12, 13, 32)], dtype=np.uint8)
    docs = []
    for _ in range(120):
        lens = rng.integers(1, max_len + 1, size=int(rng.integers(1, 400)))
        lens[rng.integers(0, lens.size)] = max_len            # every document reaches the limit
        docs.append(b" ".join(bytes(rng.choice(pool, size=int(l))) for l in lens))
    data, off = _pack(docs, lead=max_len % 16)
    wx, woff = _oracle_x(docs, 3, False)
    x, soff = sedd.debug_shingle_hashes(dev(data), dev(off), 3, 0)
    assert np.array_equal(host(soff), woff) and np.array_equal(host(x), wx)
    _check_minhash(sedd, data, off, 5, 64, seed=max_len, flags=0, procs=NPROC)


@pytest.mark.parametrize("flags", [0, 2, 4])
def test_words_longer_than_tiles_and_pieces(sedd, flags):
    """Words (no whitespace inside) of about one 1 KiB tile, one 8 KiB piece of the streaming
    kernel, 70 KiB and 3 MB, alone in a document, at its start, in its middle and at its end: the
    wavefront that owns the word's first byte walks it to its end, the wavefronts whose pieces
    lie inside it own nothing.  Default, paper-prime and rolling-family mode."""
    say("words longer than tiles and pieces, flags", flags)
    rng = np.random.default_rng(64 + flags)

    def word(length):
        return bytes(rng.integers(33, 127, size=int(length), dtype=np.uint8))

    def filler(k):
        return b" ".join(word(l) for l in rng.integers(1, 12, size=k))

    docs = []
    for length in (1007, 1008, 1024, 1025, 8191, 8192, 8193, 70_001, 3_000_000):
        docs.append(word(length))
        docs.append(word(length) + b" " + filler(9))
        docs.append(filler(7) + b"\n" + word(length) + b"\t" + filler(300))
        docs.append(filler(40) + b" " + word(length))
        docs.append(word(length) + b" " + word(length + 1))
    data, off = _pack(docs, lead=3)
    for n, K in ((1, 8), (5, 40)):
        _check_minhash(sedd, data, off, n, K, seed=7, flags=flags, procs=NPROC)


def _token_with_hash(x, rng):
    """A whitespace-free byte string whose Eq. 1 value is x: random high digits, then the base-257
    expansion of what is left, retried until every digit is a usable byte."""
    P = (1 << 61) - 1
    ws = {0x09, 0x0A, 0x0B, 0x0C, 0x0D, 0x20}
    while True:
        high = [int(c) for c in rng.integers(0x21, 0x7F, size=4)]
        rest = (x - sum(c * pow(257, 8 + i, P) for i, c in enumerate(high))) % P
        low = []
        for _ in range(8):                       # 257^8 > p: eight digits always suffice
            low.append(rest % 257)
            rest //= 257
        if rest == 0 and all(c < 256 and c not in ws for c in low):
            tok = bytes(low + high)
            assert sum(c * pow(257, i, P) for i, c in enumerate(tok)) % P == x
            return tok


def test_stream_kernel_exact_path_for_values_next_to_the_modulus(sedd):
    """Text whose shingle hashes are solved so that (a_k x + b_k) mod p lands within a few units
    of 0 or p for some function: the streaming kernel's fast evaluation cannot decide those and
    must redo the round exactly.  One-token documents (their single shingle is the token) and
    the same tokens inside longer documents with n = 1."""
    say("stream near-modulus values")
    P = (1 << 61) - 1
    K, seed = 128, 0
    a, b = oracle.coeffs(seed, K)
    rng = np.random.default_rng(4)
    targets = [0, 1, 2, 5, P - 1, P - 2, P - 5, P - (1 << 32), P - (1 << 32) - 1, (1 << 32) - 1]
    toks = []
    for k in (0, 63, 64, 127):
        inv = pow(int(a[k]), -1, P)
        for t in targets:
            xv = ((t - int(b[k])) * inv) % P
            toks.append(_token_with_hash(xv, rng))
    filler = [bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8)) for l in rng.integers(1, 9, size=300)]
    docs = [t for t in toks] + [b" ".join(filler[:150] + toks[:20] + filler[150:]),
                                b" ".join(toks)]
    data, off = _pack(docs, 3)
    before = sedd.debug_stats()[sedd.STAT_SLOW_TILES]
    for n in (1, 5):
        want = oracle.minhash(data, off, n, K, seed, 0)
        got = host(sedd.sedd_minhash(dev(data), dev(off), n, K, seed, 0))
        bad = np.nonzero((got != want).any(axis=1))[0]
        assert bad.size == 0, (n, bad[:5])
    after = sedd.debug_stats()[sedd.STAT_SLOW_TILES]
    assert after > before, "the exact path was never taken"


@pytest.mark.parametrize("flags,n", [(0, 5), (1, 13), (2, 5), (4, 3)])
def test_minhash_from_host_memory_in_chunks(sedd, flags, n):
    """sedd_minhash_host_chunked: text and offsets in host memory (pinned and pageable), cut into
    many chunks, a chunk size below the longest document, offsets that do not start at 0, empty
    documents at chunk edges: signatures equal the oracle's and those of the resident call."""
    say("host chunked", flags, n)
    r = corpus.Recipe("h", seed=8, n_docs=900, vocab=2000, len_median=120, len_sigma=1.1, len_lo=0,
                      len_hi=6000, near_frac=0.2, ws_variety=1)
    data, off = corpus.generate(r)
    lead = np.frombuffer(b"not part of any document ", dtype=np.uint8)
    data = np.concatenate([lead, data])
    off = np.concatenate([off[:300], off[299:300], off[299:]]) + np.uint64(lead.size)   # one empty doc
    K = 48 if flags != 4 else 16
    want = oracle.minhash_sharded(data, off, n, K, 2, flags, procs=NPROC)
    resident = host(sedd.sedd_minhash(dev(data), dev(off), n, K, 2, flags))
    assert np.array_equal(resident, want)
    for pinned in (True, False):
        h_text = torch.from_numpy(data.copy())
        h_off = torch.from_numpy(off.astype(np.int64))
        if pinned:
            h_text, h_off = h_text.pin_memory(), h_off.pin_memory()
        for chunk in (0, 1 << 20, 40_000, 3_000):
            got = sedd.sedd_minhash_host_chunked(h_text, h_off, n, K, 2, flags, chunk_bytes=chunk)
            torch.cuda.synchronize()
            bad = np.nonzero((host(got) != want).any(axis=1))[0]
            assert bad.size == 0, (pinned, chunk, bad[:5])
    bad_off = torch.from_numpy(np.array([0, 50, 40, 60], dtype=np.int64))
    with pytest.raises(sedd.SeddError) as e:
        sedd.sedd_minhash_host_chunked(torch.from_numpy(data.copy()), bad_off, n, K)
    assert e.value.code == -1


def test_minhash_default_mode_from_four_threads_on_four_streams(sedd):
    """Word shingles with the affine family keep no mutable shared scratch: four threads, a stream
    each, different corpora, K and seeds (one thread in the paper-prime mode), several calls per
    thread in flight together; every result against the oracle.  More (K, seed) pairs than the
    coefficient cache holds are cycled through first, and again by one thread while the others
    are calling, so that sets are evicted while others are in use."""
    import threading
    say("minhash concurrent")
    for s_ in range(20):                                    # overflow the cache of coefficient sets
        data, off = corpus.generate(corpus.config(1).scaled(40))
        _check_minhash(sedd, data, off, 5, 8, seed=1000 + s_, flags=0)
    jobs = []
    for t in range(4):
        r = corpus.config(1).scaled(2500 + 400 * t, seed=50 + t)
        data, off = corpus.generate(r)
        K, seed, n, flags = (64, 128, 200, 256)[t], 7 * t, (5, 3, 5, 2)[t], (0, 0, 2, 0)[t]
        jobs.append((data, off, n, K, seed, flags,
                     oracle.minhash_sharded(data, off, n, K, seed, flags, procs=NPROC)))
    small, small_off = corpus.generate(corpus.config(1).scaled(40))
    small_want = [oracle.minhash(small, small_off, 5, 8, 3000 + s_, 0) for s_ in range(24)]
    errors = []

    def work(t):
        try:
            data, off, n, K, seed, flags, want = jobs[t]
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                d_data, d_off = dev(data), dev(off)
                d_small, d_small_off = dev(small), dev(small_off)
                for rep in range(6):
                    got = sedd.sedd_minhash(d_data, d_off, n, K, seed, flags, stream=st)
                    st.synchronize()
                    if not np.array_equal(host(got), want):
                        errors.append((t, rep))
                    if t == 0:                              # fresh seeds: the cache overflows meanwhile
                        for s_ in range(4 * rep, 4 * rep + 4):
                            g = sedd.sedd_minhash(d_small, d_small_off, 5, 8, 3000 + s_, 0, stream=st)
                            st.synchronize()
                            if not np.array_equal(host(g), small_want[s_]):
                                errors.append((t, rep, "seed", s_))
        except Exception as e:                              # surfaced in the main thread
            errors.append((t, repr(e)))
    threads = [threading.Thread(target=work, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors


def test_minhash_rejects_offsets_beyond_the_text(sedd):
    """The binding passes the size of the text: offsets that point past it are refused before
    any kernel follows them."""
    say("minhash offsets past the text")
    data = dev(np.full(64, 97, np.uint8))
    out = torch.full((2, 8), 7, dtype=torch.int32, device="cuda").view(torch.uint32)
    for flags in (0, 1, 2, 4):
        with pytest.raises(sedd.SeddError) as e:
            sedd.sedd_minhash(data, dev(np.array([0, 40, 65], dtype=np.uint64)), 5, 8, 0, flags, out=out)
        assert e.value.code == -1
    assert (out.view(torch.int32) == 7).all().item()
    sedd.sedd_minhash(data, dev(np.array([0, 40, 64], dtype=np.uint64)), 5, 8, out=out)


@pytest.mark.parametrize("seed", [21, 22])
def test_fuzz_signatures_in_the_other_hash_modes(sedd, seed):
    """The same adversarial tokenisation inputs through the paper-prime and rolling-family modes."""
    say("fuzz modes", seed)
    docs = _fuzz_docs(seed, 250)
    data, off = _pack(docs, lead=seed % 16)
    d_data, d_off = dev(data), dev(off)
    for mode in (sedd.FLAG_PAPER_PRIME, sedd.FLAG_ROLLING_FAMILY):
        for byte_mode, n in ((False, 1), (False, 5), (False, 7), (True, 1), (True, 13)):
            flags = mode | int(byte_mode)
            want = oracle.minhash_sharded(data, off, n, 16, seed, flags, procs=NPROC)
            got = host(sedd.sedd_minhash(d_data, d_off, n, 16, seed, flags))
            bad = np.nonzero((got != want).any(axis=1))[0]
            assert bad.size == 0, (mode, byte_mode, n, bad[:5])


# ---- the largest parameters the calls accept ---------------------------------------------------

def test_largest_K_bands_and_shingle_length(sedd):
    """K = 4096 hash functions, 4096 bands of one row (and 1 band of 4096 rows), 64-token and
    64-byte shingles: the limits stated in the header."""
    say("maximum parameters")
    data, off = corpus.generate(corpus.config(1).scaled(60))
    K = 4096
    for flags, n in ((0, 5), (0, 64), (1, 64), (2, 5), (3, 64), (4, 5), (5, 64)):
        want = oracle.minhash_sharded(data, off, n, K, 3, flags, procs=NPROC)
        sig = sedd.sedd_minhash(dev(data), dev(off), n, K, 3, flags)
        assert np.array_equal(host(sig), want), (flags, n)
        if flags == 0 and n == 5:
            for b, r in ((4096, 1), (1, 4096), (512, 8)):
                wkeys = oracle.lsh_keys(want, b, r)
                keys = sedd.sedd_lsh_keys(sig, b, r)
                assert np.array_equal(host(keys), wkeys), (b, r)
                assert np.array_equal(host(sedd.sedd_cluster(keys)), oracle.cluster(wkeys)), (b, r)
                for mm in (1, 3000, 4096):
                    assert np.array_equal(host(sedd.sedd_cluster_verified(keys, sig, mm)),
                                          oracle.cluster_verified(wkeys, want, mm)), (b, r, mm)
            nb = 3
            wd = oracle.lsh_dense_keys(want, 16, 256, nb)
            dk = sedd.sedd_lsh_dense_keys(sig, 16, 256, nb)
            assert np.array_equal(host(dk), wd)
            assert np.array_equal(host(sedd.sedd_cluster_verified(dk, sig, 2000)),
                                  oracle.cluster_verified(wd, want, 2000))
