"""GPU parity at the full sizes of workloads 3, 4 and 5, in the launch configuration bench.py
times (workload 3 streamed through sedd_minhash in 2 GB pieces).

The CPU oracle cannot process these corpora whole in test time, so:
  * signatures and band keys are compared bit for bit on a sample the oracle computes: at least
    1 % of the documents of workloads 3 and 5 and 10 % of workload 4 (random runs of consecutive
    documents, a contiguous prefix, every document within 50 of an edge of a streamed 2 GB piece
    or of a chunk boundary of the chunked paths, the longest documents, random single documents,
    exact copies and their sources);
  * on the contiguous prefix (200k documents; 20k of workload 4, long documents included) the
    oracle runs the whole path on its own signatures and keys, and the GPU's cluster ids and
    verified cluster ids of the same prefix must equal the oracle's;
  * cluster ids are also checked over ALL documents against the defining property: they must equal
    the minimum-index labelling of the connected components of the graph "same key in the same
    band", recomputed here from the band keys with library sorts and scipy (no code shared with
    the HIP path or the oracle);
  * verified cluster ids (Section 3.3) are checked over ALL documents the same way: every pair
    of documents inside a bucket is enumerated with torch, its equal signature entries counted,
    and the components of the pairs at or above the threshold recomputed with scipy;
  * for workload 5 the signatures of every K of the sweep must be the leading columns of the
    K = 512 signatures (prefix property of the hash family), so one sampled comparison at K = 512
    covers all of them.
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
STREAM_CHUNK_BYTES = 2 << 30
_PROGRESS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")


def say(*a):
    """Progress line on stdout and, where the folder exists, in a file a watcher can see."""
    line = " ".join(str(x) for x in a)
    print(line, flush=True)
    if os.path.isdir(_PROGRESS):
        with open(os.path.join(_PROGRESS, "gpu_tests_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {line}\n")


@pytest.fixture(scope="module")
def sedd():
    import paper_2501_01046_amd as m
    m.lib()
    yield m
    m.sedd_release_scratch()


CHUNK_BYTES_WORDS = 256 << 20     # chunk size of sedd_minhash's chunked paths (rolling family on words;
CHUNK_BYTES_BYTES = 1 << 30       # byte shingles); the streaming kernel has no chunks
CHUNK_DOCS = 1 << 22


class Sampler:
    """Collects, while the corpus streams by, the bytes of the documents the oracle will redo."""

    def __init__(self, n_docs, seed, n_runs, run_len, prefix, n_single, n_longest_per_piece,
                 byte_mode):
        rng = np.random.default_rng(seed)
        self.ranges = [(0, min(prefix, n_docs))] if prefix else []
        for s0 in rng.integers(0, max(1, n_docs - run_len), size=n_runs):
            self.ranges.append((int(s0), int(min(n_docs, s0 + run_len))))
        self.single = np.unique(rng.integers(0, n_docs, size=n_single))
        self.n_longest = n_longest_per_piece
        self.chunk_bytes = CHUNK_BYTES_BYTES if byte_mode else CHUNK_BYTES_WORDS
        self.docs = {}                     # doc id -> bytes
        self.edge_docs = 0

    def take(self, d0, d1, data, off):
        """Called once per streamed piece: documents [d0, d1) with piece-relative offsets."""
        nd = d1 - d0
        want = set()
        for a, b in self.ranges:
            want.update(range(max(a, d0), min(b, d1)))
        lo, hi = np.searchsorted(self.single, [d0, d1])
        want.update(int(x) for x in self.single[lo:hi])
        # edges: of the piece, and of the chunks sedd_minhash cuts it into (first document at or
        # beyond every multiple of the chunk size in bytes, and every CHUNK_DOCS documents)
        edges = {0, nd}
        k = 1
        while k * self.chunk_bytes <= int(off[-1]):
            edges.add(int(np.searchsorted(off, np.uint64(int(off[0]) + k * self.chunk_bytes), side="left")))
            k += 1
        edges.update(range(CHUNK_DOCS, nd, CHUNK_DOCS))
        before = len(want)
        for e in edges:
            want.update(range(d0 + max(0, e - 50), d0 + min(nd, e + 50)))
        self.edge_docs += len(want) - before
        lens = np.diff(off.astype(np.int64))
        want.update(int(d0 + x) for x in np.argsort(lens)[::-1][: self.n_longest])
        want.update(int(d0 + x) for x in np.argsort(lens)[:2])
        for d in want:
            if d not in self.docs:
                i = d - d0
                self.docs[d] = data[int(off[i]):int(off[i + 1])].copy()

    def add(self, gen, d):
        if d not in self.docs:
            data, off = gen.generate(int(d), int(d) + 1, threads=1)
            self.docs[int(d)] = data

    def corpus(self):
        """(ids sorted, concatenated bytes, offsets) of everything collected."""
        ids = np.array(sorted(self.docs), dtype=np.int64)
        lens = np.array([self.docs[int(d)].size for d in ids], dtype=np.uint64)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
        data = np.concatenate([self.docs[int(d)] for d in ids]) if ids.size else np.zeros(0, np.uint8)
        return ids, data, off


def _stream_minhash(sedd, gen, recipe, n, K, flags, chunk_bytes, sampler=None):
    """sedd_minhash over the whole corpus, piece by piece (pieces of about chunk_bytes).
    Returns the device signatures, the piece boundaries and the per-document byte lengths."""
    n_docs = recipe.n_docs
    sig = torch.empty((n_docs, K), dtype=torch.uint32, device="cuda")
    lengths = np.zeros(n_docs, dtype=np.uint64)
    docs_per = max(1000, int(chunk_bytes / (recipe.len_median * 2.0 * 6.5)))
    bounds = []
    d0, total = 0, 0
    while d0 < n_docs:
        d1 = min(n_docs, d0 + docs_per)
        data, off = gen.generate(d0, d1)
        while data.size > chunk_bytes and d1 - d0 > 1:
            d1 = d0 + (d1 - d0) * 3 // 4
            data, off = gen.generate(d0, d1)
        lengths[d0:d1] = np.diff(off)
        t_data, t_off = torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda()
        sedd.sedd_minhash(t_data, t_off, n, K, 0, flags, out=sig[d0:d1])
        if sampler is not None:
            sampler.take(d0, d1, data, off)
        torch.cuda.synchronize()
        del t_data, t_off
        bounds.append((d0, d1))
        total += int(data.size)
        say(f"  piece docs [{d0}, {d1}) {data.size / 1e9:.2f} GB")
        d0 = d1
    return sig, bounds, lengths, total


def _oracle_on_collected(sampler, n, K, flags, procs=None):
    ids, data, off = sampler.corpus()
    return ids, oracle.minhash_sharded(data, off, n, K, 0, flags, procs=procs or NPROC)


def _check_prefix_whole_path(sedd, sig, ids, want_sig, prefix, K, b, r, label, theta=0.8):
    """Documents [0, prefix): the oracle's whole path on its own signatures against the GPU's
    band keys, clusters and verified clusters of the same prefix."""
    assert np.array_equal(ids[:prefix], np.arange(prefix)), "the prefix was not collected whole"
    o_sig = np.ascontiguousarray(want_sig[:prefix, :K])
    o_keys = oracle.lsh_keys(o_sig, b, r)
    o_cid = oracle.cluster(o_keys)
    mm = oracle.min_match_for(theta, K)
    o_vcid = oracle.cluster_verified(o_keys, o_sig, mm)
    g_sig = sig[:prefix]
    g_keys = sedd.sedd_lsh_keys(g_sig, b, r)
    g_cid = sedd.sedd_cluster(g_keys)
    g_vcid = sedd.sedd_cluster_verified(g_keys, g_sig, sedd.min_match_for(theta, K))
    torch.cuda.synchronize()
    assert np.array_equal(g_keys.cpu().numpy(), o_keys), f"{label}: prefix band keys differ"
    assert np.array_equal(g_cid.cpu().numpy(), o_cid), f"{label}: prefix cluster ids differ"
    assert np.array_equal(g_vcid.cpu().numpy(), o_vcid), f"{label}: prefix verified cluster ids differ"
    say(f"  {label}: oracle whole path on the first {prefix} documents ok "
        f"({int((o_cid != np.arange(prefix)).sum())} duplicates, "
        f"{int((o_vcid != np.arange(prefix)).sum())} verified at >= {mm})")


def _sample_docs(gen, recipe, bounds, lengths, n_random, n_longest, n_copies, seed):
    rng = np.random.default_rng(seed)
    n_docs = recipe.n_docs
    picks = set(int(x) for x in rng.choice(n_docs, size=min(n_random, n_docs), replace=False))
    for d0, d1 in bounds:
        picks.update((d0, d1 - 1))
    picks.update(int(x) for x in np.argsort(lengths)[::-1][:n_longest])
    picks.update(int(x) for x in np.argsort(lengths)[:3])
    copies = []
    if recipe.exact_frac > 0:
        for d in rng.choice(n_docs, size=min(n_docs, 40 * n_copies), replace=False):
            kind, src, _ = gen.meta(int(d))
            if kind == 2:
                copies.append((int(d), int(src)))
                picks.update((int(d), int(src)))
                if len(copies) >= n_copies:
                    break
    return np.array(sorted(picks), dtype=np.int64), copies


def _oracle_on_sample(gen, ids, n, K, flags):
    """The oracle's signatures of the sampled documents (each regenerated from its id)."""
    parts, lens = [], []
    for d in ids:
        data, off = gen.generate(int(d), int(d) + 1, threads=1)
        parts.append(data)
        lens.append(int(off[1]))
    data = np.concatenate(parts) if parts else np.zeros(0, np.uint8)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    return oracle.minhash_sharded(data, off, n, K, 0, flags, procs=NPROC)


def _components_min_label(keys_dev, n_docs, b):
    """cluster ids implied by the band keys: connected components of "same key in the same
    band", labelled by their smallest member.  torch sorts + scipy, independent of libsedd."""
    from scipy.sparse import coo_matrix
    from scipy.sparse.csgraph import connected_components
    k_signed = keys_dev.view(torch.int64)            # keys < 2^61: order is preserved
    src, dst = [], []
    for j in range(b):
        vals, order = torch.sort(k_signed[:, j])
        same = vals[1:] == vals[:-1]
        idx = torch.nonzero(same).flatten()
        src.append(order[idx].cpu().numpy())
        dst.append(order[idx + 1].cpu().numpy())
        del vals, order, same, idx
    src = np.concatenate(src)
    dst = np.concatenate(dst)
    g = coo_matrix((np.ones(src.size, dtype=np.int8), (src, dst)), shape=(n_docs, n_docs))
    _, lab = connected_components(g, directed=False)
    _, first = np.unique(lab, return_index=True)      # first occurrence = smallest member
    return first[lab].astype(np.int64), int(src.size)


def _verified_components_min_label(keys_dev, sig_dev, n_docs, b, min_match, max_bucket=2048):
    """cluster ids implied by keys and signatures under the count-match threshold: all pairs of
    every bucket, match counts by torch, components by scipy.  Independent of libsedd."""
    from scipy.sparse import coo_matrix
    from scipy.sparse.csgraph import connected_components
    k_signed = keys_dev.view(torch.int64)
    s32 = sig_dev.view(torch.int32)
    packed = []
    for j in range(b):
        vals, order = torch.sort(k_signed[:, j])
        d = 1
        while True:
            same = vals[d:] == vals[:-d]
            idx = torch.nonzero(same).flatten()
            if idx.numel() == 0:
                break
            assert d < max_bucket, "a bucket is too large for the exhaustive check"
            u, v = order[idx], order[idx + d]
            packed.append((torch.minimum(u, v) << 32) | torch.maximum(u, v))
            d += 1
        del vals, order
    if packed:
        pairs = torch.unique(torch.cat(packed))
    else:
        pairs = torch.zeros(0, dtype=torch.int64, device=keys_dev.device)
    u, v = pairs >> 32, pairs & 0xFFFFFFFF
    keep = []
    step = 1 << 20
    for i in range(0, pairs.numel(), step):
        m = (s32[u[i:i + step]] == s32[v[i:i + step]]).sum(dim=1)
        keep.append(m >= min_match)
    keep = torch.cat(keep) if keep else torch.zeros(0, dtype=torch.bool, device=keys_dev.device)
    src, dst = u[keep].cpu().numpy(), v[keep].cpu().numpy()
    g = coo_matrix((np.ones(src.size, dtype=np.int8), (src, dst)), shape=(n_docs, n_docs))
    _, lab = connected_components(g, directed=False)
    _, first = np.unique(lab, return_index=True)
    return first[lab].astype(np.int64), int(pairs.numel()), int(src.size)


def _check_verified(sedd, sig, keys, K, b, label, theta=0.8):
    n_docs = sig.shape[0]
    mm = sedd.min_match_for(theta, K)
    cid = sedd.sedd_cluster_verified(keys, sig, mm)
    torch.cuda.synchronize()
    want, n_pairs, n_edges = _verified_components_min_label(keys, sig, n_docs, b, mm)
    got = cid.cpu().numpy()
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"{label}: {bad.size} verified cluster ids differ, first {bad[:5]}"
    dups = int((got != np.arange(n_docs)).sum())
    say(f"  {label}: verified clusters (>= {mm} of {K}) ok on all {n_docs} "
        f"({n_pairs} candidate pairs, {n_edges} verified, {dups} duplicates)")
    return got


def _check_keys_and_clusters(sedd, sig, ids, want_sig, K, b, r, copies, label, verified=False):
    n_docs = sig.shape[0]
    keys = sedd.sedd_lsh_keys(sig, b, r)
    cid = sedd.sedd_cluster(keys)
    torch.cuda.synchronize()
    want_keys = oracle.lsh_keys(np.ascontiguousarray(want_sig[:, :K]), b, r)
    t_ids = torch.from_numpy(ids).cuda()
    got_keys = keys.view(torch.int64)[t_ids].cpu().numpy().view(np.uint64)
    assert np.array_equal(got_keys, want_keys), f"{label}: sampled band keys differ"
    want_cid, n_edges = _components_min_label(keys, n_docs, b)
    got_cid = cid.cpu().numpy()
    bad = np.nonzero(got_cid != want_cid)[0]
    assert bad.size == 0, f"{label}: {bad.size} cluster ids differ, first {bad[:5]}"
    for d, s in copies:
        assert got_cid[d] == got_cid[s], f"{label}: exact copy {d} of {s} not co-clustered"
    dups = int((got_cid != np.arange(n_docs)).sum())
    say(f"  {label}: keys ok on {ids.size} sampled docs, clusters ok on all {n_docs} "
        f"({n_edges} equal-key neighbours, {dups} duplicates)")
    if verified:
        vcid = _check_verified(sedd, sig, keys, K, b, label)
        assert (got_cid[vcid] == got_cid).all(), f"{label}: verified clusters do not refine"
        for d, s in copies:
            assert vcid[d] == vcid[s], f"{label}: exact copy {d} of {s} not co-clustered (verified)"
    del keys, cid
    return dups


def _check_sampled_signatures(sig, ids, want_sig, K, label):
    got = sig.view(torch.int32)[torch.from_numpy(ids).cuda()].cpu().numpy().view(np.uint32)
    bad = np.nonzero((got != want_sig[:, :K]).any(axis=1))[0]
    assert bad.size == 0, f"{label}: {bad.size} sampled signatures differ, first docs {ids[bad[:5]]}"


def _copies(gen, recipe, n_copies, seed):
    rng = np.random.default_rng(seed)
    copies = []
    if recipe.exact_frac > 0:
        for d in rng.choice(recipe.n_docs, size=min(recipe.n_docs, 40 * n_copies), replace=False):
            kind, src, _ = gen.meta(int(d))
            if kind == 2:
                copies.append((int(d), int(src)))
                if len(copies) >= n_copies:
                    break
    return copies


def test_config3_full_size_streamed(sedd):
    """10M documents, about 62 GB of text, K=256, 32x8 bands, streamed in 2 GB pieces."""
    r = corpus.config(3)
    gen = corpus.Corpus(r)
    say("config 3 at full size: streaming", r.n_docs, "documents")
    prefix = 200_000
    smp = Sampler(r.n_docs, seed=3, n_runs=100, run_len=1000, prefix=prefix, n_single=1500,
                  n_longest_per_piece=1, byte_mode=False)
    sig, bounds, lengths, total = _stream_minhash(sedd, gen, r, r.shingle_n, r.K, 0,
                                                  STREAM_CHUNK_BYTES, sampler=smp)
    copies = _copies(gen, r, 50, seed=3)
    for d, s in copies:
        smp.add(gen, d)
        smp.add(gen, s)
    say(f"  {total / 1e9:.1f} GB in {len(bounds)} pieces; oracle on {len(smp.docs)} documents "
        f"({smp.edge_docs} of them next to piece and chunk edges)")
    assert len(smp.docs) >= r.n_docs // 100
    ids, want = _oracle_on_collected(smp, r.shingle_n, r.K, 0)
    _check_sampled_signatures(sig, ids, want, r.K, "config 3")
    for d, s in copies:                                   # exact copies: identical signatures
        assert torch.equal(sig[d].view(torch.int32), sig[s].view(torch.int32))
    say(f"  signatures ok on {ids.size} documents = {100.0 * ids.size / r.n_docs:.2f} % "
        f"({len(copies)} exact copies)")
    _check_prefix_whole_path(sedd, sig, ids, want, prefix, r.K, r.b, r.r, "config 3")
    dups = _check_keys_and_clusters(sedd, sig, ids, want, r.K, r.b, r.r, copies, "config 3",
                                    verified=True)
    assert dups >= int(0.03 * r.n_docs * 0.9)             # at least the exact copies


def test_config4_full_size_long_documents(sedd):
    """200k documents, 1 % of them 1-14 MB: byte 13-grams, split-document minimum."""
    r = corpus.config(4)
    gen = corpus.Corpus(r)
    say("config 4 at full size:", r.n_docs, "documents")
    prefix = 20_000                                      # 10 %, with its ~200 long documents
    smp = Sampler(r.n_docs, seed=4, n_runs=4, run_len=250, prefix=prefix, n_single=1200,
                  n_longest_per_piece=1, byte_mode=True)
    sig, bounds, lengths, total = _stream_minhash(sedd, gen, r, r.shingle_n, r.K, 1, 1 << 62,
                                                  sampler=smp)
    n_long = int(sum(1 for d in smp.docs if lengths[d] > 1_000_000))
    say(f"  {total / 1e9:.1f} GB; longest document {int(lengths.max())} bytes; oracle on "
        f"{len(smp.docs)} documents ({n_long} of 1 MB or more, {smp.edge_docs} next to chunk edges)")
    assert n_long >= 20 and len(smp.docs) >= r.n_docs // 10
    ids, want = _oracle_on_collected(smp, r.shingle_n, r.K, 1)
    _check_sampled_signatures(sig, ids, want, r.K, "config 4")
    say(f"  signatures ok on {ids.size} documents = {100.0 * ids.size / r.n_docs:.2f} %")
    _check_prefix_whole_path(sedd, sig, ids, want, prefix, r.K, r.b, r.r, "config 4")
    _check_keys_and_clusters(sedd, sig, ids, want, r.K, r.b, r.r, [], "config 4",
                             verified=True)


def test_one_document_above_one_gigabyte(sedd):
    """A single document of 1.2 GB between small ones, in one call: positions inside a document
    beyond 2^30, about 150,000 wavefronts merging their minima into one signature row, and the
    documents after it found by their offsets beyond 2^30."""
    say("one document of 1.2 GB")
    rng = np.random.default_rng(9)
    words = [bytes(rng.integers(97, 123, size=int(l), dtype=np.uint8)) for l in rng.integers(1, 10, size=160_000)]
    block = (b" ".join(words) + b"\n")
    reps = (1_200_000_000 // len(block)) + 1
    small = [b" ".join(words[i:i + 40]) for i in range(0, 4000, 40)]
    docs = small[:50] + [block * reps] + small[50:]
    data = np.frombuffer(b"".join(docs), dtype=np.uint8)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.uint64)
    assert int(off[51] - off[50]) > (1 << 30)
    K, n = 8, 5
    t0 = time.time()
    want = oracle.minhash_sharded(data, off, n, K, 1, 0, procs=NPROC)
    say(f"  oracle {time.time() - t0:.1f} s")
    d_data, d_off = torch.from_numpy(data.copy()).cuda(), torch.from_numpy(off).cuda()
    got = sedd.sedd_minhash(d_data, d_off, n, K, 1, 0).cpu().numpy()
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"documents {bad[:5]} differ"
    del d_data, data
    # byte shingles (the chunked path): one document of 160 MB with chunks of 64 MB, so that the
    # document is longer than a chunk
    docs = small[:50] + [block * (160_000_000 // len(block) + 1)] + small[50:]
    data = np.frombuffer(b"".join(docs), dtype=np.uint8)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.uint64)
    want_b = oracle.minhash_sharded(data, off, 13, K, 1, 1, procs=NPROC)
    sedd.debug_set_chunk_bytes(64 << 20)
    try:
        got_b = sedd.sedd_minhash(torch.from_numpy(data.copy()).cuda(), torch.from_numpy(off).cuda(),
                                  13, K, 1, 1).cpu().numpy()
    finally:
        sedd.debug_set_chunk_bytes(0)
    assert np.array_equal(got_b, want_b)


def test_more_than_two_to_the_32_signature_entries(sedd):
    """9M short documents at K = 512: the signature matrix has 4.6e9 entries (18.4 GB), so every
    index d * K beyond document 8,388,608 needs more than 32 bits.  Signatures, band keys and
    dense keys of sampled documents (many of them beyond that point) against the oracle; the
    verified clusters, which compare whole signature rows, against the planted exact copies."""
    say("more than 2^32 signature entries")
    rng = np.random.default_rng(23)
    n_docs, K, n, L = 9_000_000, 512, 2, 14
    rows = rng.integers(97, 123, size=(n_docs, L), dtype=np.uint8)
    rows[:, 3] = 0x20
    rows[:, 7] = 0x20
    ids = np.arange(n_docs)
    for j in range(5):                                  # the document's index, so that no two are alike
        rows[:, 8 + j] = 97 + (ids // 26 ** j) % 26
    rows[::7, 3] = 0x61                                 # some documents of two tokens
    rows[::11, 3] = 0x61
    rows[::11, 7] = 0x61                                # and of one (fewer tokens than n)
    # exact copies: document dst repeats src < dst; most of them in the upper range of indices
    edge = (1 << 32) // K
    src = np.concatenate([rng.integers(0, n_docs // 2, size=300), rng.integers(edge, n_docs - 10, size=300)])
    dst = np.concatenate([rng.integers(edge, n_docs, size=300), np.zeros(300, dtype=np.int64)])
    dst[300:] = src[300:] + rng.integers(1, 10, size=300)
    keep = np.unique(dst, return_index=True)[1]
    src, dst = src[keep], dst[keep]
    ok = ~np.isin(src, dst)                             # no chains: a source is never a copy itself
    src, dst = src[ok], dst[ok]
    rows[dst] = rows[src]
    lens = np.full(n_docs, L, dtype=np.uint64)
    empty = np.setdiff1d(np.arange(5, n_docs, 999_983), np.concatenate([src, dst]))
    lens[empty] = 0
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    data = np.ascontiguousarray(rows[lens > 0]).reshape(-1)
    d_data, d_off = torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda()
    sig = sedd.sedd_minhash(d_data, d_off, n, K)
    torch.cuda.synchronize()
    assert sig.numel() > (1 << 32)
    sample = np.unique(np.concatenate([
        np.arange(0, 100), np.arange(n_docs - 100, n_docs), np.arange(edge - 100, edge + 100),
        rng.integers(0, n_docs, size=1500), rng.integers(edge, n_docs, size=1500), src, dst, empty]))
    s_lens = lens[sample]
    s_off = np.concatenate([[0], np.cumsum(s_lens)]).astype(np.uint64)
    s_data = np.ascontiguousarray(rows[sample][s_lens > 0]).reshape(-1)
    want_sig = oracle.minhash(s_data, s_off, n, K)
    idx = torch.from_numpy(sample).cuda()
    got_sig = sig.view(torch.int32)[idx].cpu().numpy().view(np.uint32)   # (no uint32 gather in torch)
    bad = np.nonzero((got_sig != want_sig).any(axis=1))[0]
    assert bad.size == 0, f"signatures of documents {sample[bad][:5]} differ"
    say(f"  signatures of {sample.size} sampled documents ok ({int((sample >= edge).sum())} beyond 2^32 / K)")
    for b, r in ((64, 8), (4, 8)):
        keys = sedd.sedd_lsh_keys(sig, b, r)
        got_keys = keys.view(torch.int64)[idx].cpu().numpy().view(np.uint64)
        assert np.array_equal(got_keys, oracle.lsh_keys(want_sig, b, r)), (b, r)
        del keys
    nb = sedd.dense_bucket_count(n_docs)
    dkeys = sedd.sedd_lsh_dense_keys(sig, 16, 8, nb)
    got_dkeys = dkeys.view(torch.int64)[idx].cpu().numpy().view(np.uint64)
    assert np.array_equal(got_dkeys, oracle.lsh_dense_keys(want_sig, 16, 8, nb))
    del dkeys
    # verified clusters at min_match = K: exactly the planted copies (and the empty documents,
    # whose signatures are all 0xFFFFFFFF, with the first of them)
    keys = sedd.sedd_lsh_keys(sig, 4, 8)
    cid = sedd.sedd_cluster_verified(keys, sig, K).cpu().numpy()
    want = np.arange(n_docs, dtype=np.int64)
    want[dst] = src
    want[empty] = empty[0]
    diff = np.nonzero(cid != want)[0]
    assert diff.size == 0, f"verified cluster ids differ at {diff[:5]}: {cid[diff[:5]]} vs {want[diff[:5]]}"
    say(f"  verified clusters: {dst.size} planted copies and {empty.size} empty documents found, nothing else")


def test_cluster_close_to_two_to_the_32_records(sedd):
    """67M documents in 64 bands: 4.288e9 (key, document) records, just below the 2^32 the calls
    accept, so record indices in the upper bands pass 2^31.  Every key holds its document's index
    in its high bits (no two documents agree by accident) over 34 random low bits (the sorted
    bits stay random); copies are planted band by band, most of them in the last bands and the
    last documents.  sedd_cluster and sedd_cluster_verified must find exactly the planted pairs."""
    say("cluster close to 2^32 records")
    n, b, K = 67_000_000, 64, 8
    assert n * b < (1 << 32) and n * b > (1 << 32) - (1 << 24)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    keys = torch.empty((n, b), dtype=torch.int64, device="cuda")
    step = 1 << 22
    for i in range(0, n, step):
        part = keys[i:i + step]
        part.random_(0, 1 << 34, generator=gen)
        part += (torch.arange(i, min(n, i + step), device="cuda", dtype=torch.int64) << 34)[:, None]
    sig = torch.empty((n, K), dtype=torch.int32, device="cuda")
    sig.random_(0, (1 << 31) - 1, generator=gen)
    rng = np.random.default_rng(6)
    m = 4000
    src = np.concatenate([rng.integers(0, n - 2000, size=m // 2), rng.integers(n - 200_000, n - 2000, size=m // 2)])
    dst = src + rng.integers(1, 1000, size=m)
    keep = np.unique(dst, return_index=True)[1]
    src, dst = src[keep], dst[keep]
    ok = ~np.isin(src, dst)
    src, dst = src[ok], dst[ok]
    band = np.where(rng.random(src.size) < 0.5, rng.integers(b - 3, b, size=src.size), rng.integers(0, b, size=src.size))
    t_src, t_dst, t_band = (torch.from_numpy(a).cuda() for a in (src, dst, band))
    keys[t_dst, t_band] = keys[t_src, t_band]
    half = src.size // 2                                 # half of the copies also repeat the signature
    sig[t_dst[:half]] = sig[t_src[:half]]
    torch.cuda.synchronize()
    want = torch.arange(n, dtype=torch.int64, device="cuda")
    want[t_dst] = t_src
    cid = sedd.sedd_cluster(keys.view(torch.uint64))
    diff = torch.nonzero(cid != want).flatten()
    assert diff.numel() == 0, f"cluster ids differ at {diff[:5].tolist()}"
    say(f"  sedd_cluster: {src.size} planted pairs found, nothing else")
    del cid
    want_v = torch.arange(n, dtype=torch.int64, device="cuda")
    want_v[t_dst[:half]] = t_src[:half]
    vcid = sedd.sedd_cluster_verified(keys.view(torch.uint64), sig.view(torch.uint32), K)
    diff = torch.nonzero(vcid != want_v).flatten()
    assert diff.numel() == 0, f"verified cluster ids differ at {diff[:5].tolist()}"
    say(f"  sedd_cluster_verified: the {half} pairs with equal signatures found, nothing else")
    del keys, sig, vcid
    sedd.sedd_release_scratch()


def test_one_call_on_more_than_four_gigabytes_of_words(sedd):
    """850k documents of the 10M-document recipe, 5 GB of text, handed to sedd_minhash in ONE call
    (the workload itself uses 2 GB pieces): byte positions inside the call pass 2^32.  Sampled
    documents, and every document within 50 of the 2^32 position, against the oracle."""
    r = corpus.config(3).scaled(850_000)
    gen = corpus.Corpus(r)
    K = 64
    say("one call on 5 GB of words:", r.n_docs, "documents")
    smp = Sampler(r.n_docs, seed=8, n_runs=8, run_len=250, prefix=0, n_single=1500,
                  n_longest_per_piece=2, byte_mode=False)
    sig, bounds, lengths, total = _stream_minhash(sedd, gen, r, r.shingle_n, K, 0, 1 << 62, sampler=smp)
    assert len(bounds) == 1 and total > (1 << 32) + (1 << 28)
    at = int(np.searchsorted(np.cumsum(lengths), 1 << 32))
    for d in range(at - 50, at + 50):
        smp.add(gen, d)
    for d in range(r.n_docs - 50, r.n_docs):
        smp.add(gen, d)
    ids, want = _oracle_on_collected(smp, r.shingle_n, K, 0)
    _check_sampled_signatures(sig, ids, want, K, "5 GB call")
    say(f"  {total / 1e9:.2f} GB in one call; signatures ok on {ids.size} documents "
        f"({int((ids > at).sum())} of them beyond byte 2^32)")


def test_config2_full_size_paper_prime(sedd):
    """The medium workload with the paper's own modulus (SEDD_FLAG_PAPER_PRIME)."""
    r = corpus.config(2)
    gen = corpus.Corpus(r)
    say("config 2 at full size, paper-prime mode:", r.n_docs, "documents")
    sig, bounds, lengths, total = _stream_minhash(sedd, gen, r, r.shingle_n, r.K, 2, 1 << 62)
    ids, copies = _sample_docs(gen, r, bounds, lengths, n_random=4000, n_longest=6, n_copies=0,
                               seed=22)
    # and documents at regular distances through the corpus
    edge = [d for c in range(1, 10) for d in range(c * 98_000, c * 98_000 + 2_500, 25)]
    ids = np.array(sorted(set(ids.tolist()) | set(edge)), dtype=np.int64)
    want = _oracle_on_sample(gen, ids, r.shingle_n, r.K, 2)
    _check_sampled_signatures(sig, ids, want, r.K, "config 2 paper prime")
    vals = sig.view(torch.int32)
    assert int(vals.max().item()) < 4294967 and int(vals.min().item()) >= -1
    say(f"  signatures ok on {ids.size} sampled docs")
    _check_keys_and_clusters(sedd, sig, ids, want, r.K, r.b, r.r, copies, "config 2 paper prime",
                             verified=True)


def test_config4_full_size_paper_prime(sedd):
    """Long documents with the paper's own modulus: the 22-bit range is exhausted, which the
    results must reproduce exactly (minima of a few units, large chance buckets)."""
    r = corpus.config(4)
    gen = corpus.Corpus(r)
    say("config 4 at full size, paper-prime mode:", r.n_docs, "documents")
    sig, bounds, lengths, total = _stream_minhash(sedd, gen, r, r.shingle_n, r.K, 3, 1 << 62)
    ids, copies = _sample_docs(gen, r, bounds, lengths, n_random=1200, n_longest=1, n_copies=0,
                               seed=44)
    long_ids = np.nonzero(lengths > 1_000_000)[0]
    extra = long_ids[np.argsort(lengths[long_ids])[:3]]
    ids = np.array(sorted(set(ids.tolist()) | set(int(x) for x in extra)), dtype=np.int64)
    want = _oracle_on_sample(gen, ids, r.shingle_n, r.K, 3)
    _check_sampled_signatures(sig, ids, want, r.K, "config 4 paper prime")
    say(f"  signatures ok on {ids.size} sampled docs")
    _check_keys_and_clusters(sedd, sig, ids, want, r.K, r.b, r.r, copies, "config 4 paper prime")
    t_long = torch.from_numpy(long_ids).cuda()
    assert int(sig.view(torch.int32)[t_long].max().item()) < 256    # every minimum collapsed


def test_config5_full_size_sweep(sedd):
    """2M documents; K in {64,128,256,512} x (b,r) in {(8,16),(16,8),(32,8),(64,4)} x n in {3,5}."""
    r = corpus.config(5)
    gen = corpus.Corpus(r)
    say("config 5 at full size:", r.n_docs, "documents")
    data, off = gen.generate()
    t_data, t_off = torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda()
    prefix = 200_000
    smp = Sampler(r.n_docs, seed=5, n_runs=20, run_len=1000, prefix=prefix, n_single=1500,
                  n_longest_per_piece=4, byte_mode=False)
    smp.take(0, r.n_docs, data, off)
    say(f"  oracle on {len(smp.docs)} documents ({smp.edge_docs} of them next to chunk edges)")
    assert len(smp.docs) >= r.n_docs // 100
    for n in (3, 5):
        ids, want = _oracle_on_collected(smp, n, 512, 0)
        sig512 = sedd.sedd_minhash(t_data, t_off, n, 512)
        _check_sampled_signatures(sig512, ids, want, 512, f"config 5 n={n} K=512")
        say(f"  n={n}: K=512 signatures ok on {ids.size} documents = "
            f"{100.0 * ids.size / r.n_docs:.2f} %")
        for K in (64, 128, 256, 512):
            if K == 512:
                sig = sig512
            else:
                sig = sedd.sedd_minhash(t_data, t_off, n, K)
                assert torch.equal(sig.view(torch.int32), sig512[:, :K].contiguous().view(torch.int32)), \
                    f"n={n} K={K}: not the leading columns of the K=512 signatures"
            for b, rr in ((8, 16), (16, 8), (32, 8), (64, 4)):
                if b * rr > K:
                    continue
                if (K, b) in ((64, 8), (128, 16), (256, 32), (512, 64)):
                    _check_prefix_whole_path(sedd, sig, ids, want, prefix, K, b, rr,
                                             f"config 5 n={n} K={K} b={b} r={rr}")
                _check_keys_and_clusters(sedd, sig, ids, want, K, b, rr, [],
                                         f"config 5 n={n} K={K} b={b} r={rr}",
                                         verified=(K, b) in ((128, 16), (256, 64), (512, 8)))
            if K != 512:
                del sig
        del sig512


def test_dense_buckets_on_documents(sedd):
    """The paper's candidate generation on real signatures: 300k documents of the medium
    workload, 4 sqrt(N) = 2190 buckets of about 137 documents per band, every pair of a bucket
    compared (the tiled count-match path).  Keys against the oracle on sampled documents,
    cluster ids of all documents against the all-pairs recomputation."""
    r = corpus.config(2).scaled(300_000)
    gen = corpus.Corpus(r)
    say("dense buckets on", r.n_docs, "documents of config 2")
    data, off = gen.generate()
    sig = sedd.sedd_minhash(torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(),
                            r.shingle_n, r.K)
    nb = sedd.dense_bucket_count(r.n_docs)
    assert nb == oracle.dense_bucket_count(r.n_docs) == 2190
    keys = sedd.sedd_lsh_dense_keys(sig, r.b, r.r, nb)
    ids, _ = _sample_docs(gen, r, [(0, r.n_docs)], np.diff(off), n_random=1000, n_longest=2,
                          n_copies=0, seed=6)
    want_sig = _oracle_on_sample(gen, ids, r.shingle_n, r.K, 0)
    _check_sampled_signatures(sig, ids, want_sig, r.K, "dense")
    got_keys = keys.view(torch.int64)[torch.from_numpy(ids).cuda()].cpu().numpy().view(np.uint64)
    assert np.array_equal(got_keys, oracle.lsh_dense_keys(want_sig, r.b, r.r, nb))
    mm = sedd.min_match_for(0.8, r.K)
    cid = sedd.sedd_cluster_verified(keys, sig, mm)
    torch.cuda.synchronize()
    want, n_pairs, n_edges = _verified_components_min_label(keys, sig, r.n_docs, r.b, mm,
                                                            max_bucket=1024)
    got = cid.cpu().numpy()
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"{bad.size} cluster ids differ, first {bad[:5]}"
    # the sparse 61-bit keys find the same verified pairs wherever a whole band agrees; dense
    # buckets can only add pairs to those
    sparse = sedd.sedd_cluster_verified(sedd.sedd_lsh_keys(sig, r.b, r.r), sig, mm).cpu().numpy()
    assert (got[sparse] == got).all()
    say(f"  {n_pairs} candidate pairs, {n_edges} verified, "
        f"{int((got != np.arange(r.n_docs)).sum())} duplicates "
        f"({int((sparse != np.arange(r.n_docs)).sum())} with sparse keys)")
