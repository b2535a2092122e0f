#!/usr/bin/env python3
"""Benchmark of the MinHash-LSH hot path on one MI355X.

A step is one pass of the whole path (sedd_minhash -> sedd_lsh_keys -> sedd_cluster) over one
batch of synthetic input that is already resident in HBM.  The default workload is the largest
one that fits a single GPU: 10M web-text-shaped documents (about 62 GB of text), 5-word shingles,
K=256, 32 bands of 8 rows, the text handed to sedd_minhash in pieces of 2 GB.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--docs N]
                    [--sweep] [--no-cpu-baseline] [--no-host-leg] [--no-extras] [--no-per-config]

--config 2 is the medium workload (1M documents, K=128, 16x8); --config 5 --sweep runs the
K x (b, r) x n grid and adds the planted-pair S-curve fit per setting.
After the timed steps the same buffers serve a few untimed measurements reported beside the
headline: verified clusters, the dense-bucket flow with its bucket-balance statistics, the fidelity
of LSH + verification against brute-force all-pairs comparison, (workloads of at most 2M
documents) the two alternative hash-function modes, the path fed from pinned host memory (the
PCIe-inclusive rate), and a short run of the other workloads (`per_config`).
The CPU oracle is timed on a bounded sample of the same corpus and reported beside the GPU
figure as `cpu_baseline`; it is a reported baseline, not the target.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Algorithmic work of the dominant kernel, in 32-bit integer VALU lane-operations:
#   per (shingle, hash function): one 61-bit multiply-add mod 2^61-1, truncation, minimum
#     = 8 operations in the best sequence known here (six 32x32+64 multiply-adds, one 3-input
#       add, one minimum);
#   per shingle: its Eq. 1 base hash from n token records (word mode) = n-1 modular
#     multiply-adds of 8 operations, or n byte steps of 4 operations (byte mode).
OPS_PER_PAIR = 8
OPS_PER_BASE_STEP_WORD = 8
OPS_PER_BASE_STEP_BYTE = 4
# The paper-prime mode (modulus 4,294,967): per (shingle, function) one 32x32+64 multiply-add,
# two 24-bit multiply-adds and half a three-input minimum; per Eq. 1 step one product reduced
# through a quotient estimate (10 operations), two of them per byte window (reuse form).
OPS_PER_PAIR_PP = 3.5
OPS_PER_BASE_STEP_PP = 10
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one 32-bit integer lane-operation per lane per clock
PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
STREAM_CHUNK_BYTES = 2 << 30
DEFAULT_CONFIG = 3


def ops_per_shingle(recipe, K):
    if recipe.byte_mode:
        base = recipe.shingle_n * OPS_PER_BASE_STEP_BYTE
    else:
        base = (recipe.shingle_n - 1) * OPS_PER_BASE_STEP_WORD
    return K * OPS_PER_PAIR + base


def ops_per_shingle_pp(recipe, K):
    base = (2 if recipe.byte_mode else recipe.shingle_n - 1) * OPS_PER_BASE_STEP_PP
    return K * OPS_PER_PAIR_PP + base


def measured_traffic(workload):
    """HBM bytes one launch of the dominant kernel moves on `workload`, as recorded in the
    rocprofv3 --pmc summary under profiles/ (a line `traffic_bytes_per_launch: <number>`).
    None when no summary of that workload is there."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return (float(m.group(1)), os.path.relpath(path, ROOT)) if m else (None, None)
    except OSError:
        return None, None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def load_corpus(torch, corpus, recipe, stream_chunk=None, keep_host_docs=0):
    """Generate the corpus and place it in HBM.  Returns a list of (text, offsets, d0, d1)
    device pieces (one piece unless stream_chunk is given), total bytes, and host arrays of
    the first documents (at least keep_host_docs of them, for the oracle sample)."""
    gen = corpus.Corpus(recipe)
    pieces = []
    total = 0
    if stream_chunk is None:
        data, off = gen.generate()
        pieces.append((torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(), 0, recipe.n_docs))
        return pieces, int(data.size), (data, off)
    host_parts = []
    # documents per generation batch sized from the recipe's mean length (about 6 bytes a word)
    mean_words = recipe.len_median * 2.0
    docs_per = max(1000, int(stream_chunk / (mean_words * 6.5)))
    d0 = 0
    while d0 < recipe.n_docs:
        d1 = min(recipe.n_docs, d0 + docs_per)
        data, off = gen.generate(d0, d1)
        while data.size > stream_chunk and d1 - d0 > 1:      # keep each piece within the chunk size
            d1 = d0 + (d1 - d0) * 3 // 4
            data, off = gen.generate(d0, d1)
        if d0 < max(1, keep_host_docs):
            host_parts.append((data, off))
        pieces.append((torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(), d0, d1))
        total += int(data.size)
        d0 = d1
    import numpy as np
    h_data = np.concatenate([p[0] for p in host_parts])
    offs, base = [np.zeros(1, np.uint64)], 0
    for _, o in host_parts:
        offs.append(o[1:] + np.uint64(base))
        base += int(o[-1])
    return pieces, total, (h_data, np.concatenate(offs))


def jaccard_of_pair(oracle, a: bytes, b: bytes, n: int, byte_mode: bool) -> float:
    sa = set(oracle.doc_shingles(a, n, byte_mode).tolist())
    sb = set(oracle.doc_shingles(b, n, byte_mode).tolist())
    if not sa and not sb:
        return 1.0
    return len(sa & sb) / len(sa | sb)


class Workload:
    """One corpus resident in HBM and the timed path over it."""

    def __init__(self, torch, sedd, corpus, recipe, streamed, keep_host_docs=0):
        self.torch, self.sedd, self.recipe = torch, sedd, recipe
        self.flags = sedd.FLAG_BYTE_SHINGLES if recipe.byte_mode else 0
        t0 = time.time()
        self.pieces, self.n_bytes, (self.h_data, self.h_off) = load_corpus(
            torch, corpus, recipe, STREAM_CHUNK_BYTES if streamed else None, keep_host_docs)
        self.t_gen = time.time() - t0
        self.n_docs = recipe.n_docs
        self.streamed = streamed

    def run_path(self, K, b, r, n, sig, keys, cid, mode_flags):
        for text, off, d0, d1 in self.pieces:
            self.sedd.sedd_minhash(text, off, n, K, 0, mode_flags, out=sig[d0:d1])
        self.sedd.sedd_lsh_keys(sig, b, r, out=keys)
        self.sedd.sedd_cluster(keys, out=cid)

    def measure(self, K, b, r, n, steps, warmup, mode_flags=None):
        torch, sedd = self.torch, self.sedd
        mode_flags = self.flags if mode_flags is None else mode_flags
        sig = torch.empty((self.n_docs, K), dtype=torch.uint32, device="cuda")
        keys = torch.empty((self.n_docs, b), dtype=torch.uint64, device="cuda")
        cid = torch.empty((self.n_docs,), dtype=torch.int64, device="cuda")
        for _ in range(warmup):
            self.run_path(K, b, r, n, sig, keys, cid, mode_flags)
        torch.cuda.synchronize()
        sedd.profile_enable(True)
        sedd.profile_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.run_path(K, b, r, n, sig, keys, cid, mode_flags)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        sedd.profile_enable(False)
        return elapsed, sedd.profile_read(), sig, keys, cid

    def shingle_count(self, n):
        tot = 0
        for text, off, d0, d1 in self.pieces:
            _, soff = self.sedd.debug_shingle_hashes_offsets(text, off, n, self.flags)
            tot += int(soff[-1])
        return tot

    def roofline(self, stages, steps, K, n_shingles):
        mh_ms, mh_spans = stages["minhash"]
        ops_step = n_shingles * ops_per_shingle(self.recipe, K)
        launches = max(1, mh_spans // max(1, steps))
        achieved = ops_step * steps / (mh_ms * 1e-3) / 1e12 if mh_ms else 0.0
        return {
            "kernel": "k_minhash" if self.recipe.byte_mode else "k_minhash_stream",
            "bound": "alu", "achieved": round(achieved, 3),
            "peak": round(PEAK_TOPS, 3), "unit": "TOP/s (int32 VALU lane-ops)",
            "frac": round(achieved / PEAK_TOPS, 4), "traffic": None,
            "ops_per_shingle": ops_per_shingle(self.recipe, K), "shingles_per_step": n_shingles,
            "ops_per_launch": ops_step // launches,
            "launches_per_step": launches, "avg_launch_ms": round(mh_ms / max(1, mh_spans), 4),
            "hash_evals_per_s": round(n_shingles * K * steps / (mh_ms * 1e-3), 1) if mh_ms else 0,
            "counted_as_work": "8 lane-ops per (shingle, function) + 8 per Horner step over token "
                               "records (4 per byte step); tokenisation and Eq. 1 per token, which "
                               "k_minhash_stream also does, are not counted",
            # the whole step against the same peak: what the path sustains end to end
            "whole_path_frac": None,
        }

    def parity_sample(self, oracle, np, sig, keys, n, K, b, r, ns, min_match, procs):
        """The oracle's whole path on the first ns documents against the GPU's results."""
        sedd = self.sedd
        ns = min(ns, self.h_off.size - 1)
        sub_off = self.h_off[: ns + 1]
        sub = self.h_data[: int(sub_off[-1])]
        o_sig = oracle.minhash_sharded(sub, sub_off, n, K, 0, self.flags, procs=procs)
        o_keys = oracle.lsh_keys(o_sig, b, r)
        o_cid = oracle.cluster(o_keys)
        o_vcid = oracle.cluster_verified(o_keys, o_sig, min_match)
        g_keys, g_sig = keys[:ns].contiguous(), sig[:ns].contiguous()
        ok = bool(np.array_equal(g_sig.cpu().numpy(), o_sig)
                  and np.array_equal(g_keys.cpu().numpy(), o_keys)
                  and np.array_equal(sedd.sedd_cluster(g_keys).cpu().numpy(), o_cid)
                  and np.array_equal(sedd.sedd_cluster_verified(g_keys, g_sig, min_match).cpu().numpy(),
                                     o_vcid))
        return ok, ns


def bucket_balance(torch, keys, n_buckets=None):
    """Per-band bucket sizes of a key matrix, summarised the way the paper's imbalance analysis
    does (Section 4.4 and the appendix tables): largest and mean bucket, the share of buckets
    above mean + 3 sigma ("outliers"), the share of all pair comparisons those buckets hold, and
    the comparisons relative to perfectly even buckets.  Counts by torch (sort + unique), outside
    the library."""
    n_docs, b = keys.shape
    k64 = keys.view(torch.int64)
    tot_pairs = tot_out_pairs = 0.0
    n_bk = n_out = 0
    max_bucket, even_pairs = 0, 0.0
    for j in range(b):
        if n_buckets is not None and n_buckets <= (1 << 26):
            cnt = torch.bincount(k64[:, j], minlength=n_buckets).to(torch.float64)
        else:
            _, c = torch.unique(k64[:, j], return_counts=True)
            cnt = c.to(torch.float64)
        mean, sd = cnt.mean(), cnt.std(unbiased=False)
        pairs = cnt * (cnt - 1) / 2
        out = cnt > mean + 3 * sd
        tot_pairs += float(pairs.sum())
        tot_out_pairs += float(pairs[out].sum())
        n_bk += int(cnt.numel())
        n_out += int(out.sum())
        max_bucket = max(max_bucket, int(cnt.max()))
        m = float(mean)
        even_pairs += cnt.numel() * m * (m - 1) / 2 if m > 1 else 0.0
    return {
        "buckets_per_band": round(n_bk / b, 1), "mean_bucket": round(n_docs * b / n_bk, 2),
        "max_bucket": max_bucket,
        "outlier_buckets_share": round(n_out / n_bk, 6),
        "outlier_share_of_pair_comparisons": round(tot_out_pairs / tot_pairs, 4) if tot_pairs else 0.0,
        "pair_comparisons": int(tot_pairs),
        "pair_comparisons_over_even_buckets": round(tot_pairs / even_pairs, 3) if even_pairs else None,
    }


def timed_calls(torch, sedd, fn, reps):
    fn()
    torch.cuda.synchronize()
    sedd.profile_enable(True)
    sedd.profile_read()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / reps
    sedd.profile_enable(False)
    st = sedd.profile_read()
    return ms, {k: round(v[0] / reps, 4) for k, v in st.items() if v[0]}


def fidelity(torch, sedd, np, sig, b, r, min_match, n_take):
    """The paper's fidelity figure (Section 4.3): set-Jaccard between the duplicates found by
    LSH + verification and by brute-force all-pairs comparison of the same MinHash signatures.
    Brute force = the same verified-cluster call with one key column that is equal for all
    documents, so every pair is a candidate."""
    n_take = min(n_take, sig.shape[0])
    s = sig[:n_take].contiguous()
    keys = sedd.sedd_lsh_keys(s, b, r)
    lsh = sedd.sedd_cluster_verified(keys, s, min_match).cpu().numpy()
    ones = torch.zeros((n_take, 1), dtype=torch.uint64, device="cuda")
    t0 = time.perf_counter()
    brute = sedd.sedd_cluster_verified(ones, s, min_match)
    torch.cuda.synchronize()
    t_brute = time.perf_counter() - t0
    brute = brute.cpu().numpy()
    ident = np.arange(n_take)
    d_lsh, d_brute = set(np.nonzero(lsh != ident)[0].tolist()), set(np.nonzero(brute != ident)[0].tolist())
    union = d_lsh | d_brute
    return {
        "documents": n_take, "min_match": min_match,
        "duplicates_lsh_verified": len(d_lsh), "duplicates_all_pairs": len(d_brute),
        "set_jaccard": round(len(d_lsh & d_brute) / len(union), 4) if union else 1.0,
        "all_pairs_ms": round(1e3 * t_brute, 2),
        "pairs_all_pairs": n_take * (n_take - 1) // 2,
        "paper_reports": "0.956 (RealNews) / 0.966 (C4) for SEDD against CPU MinHash, other data",
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--docs", type=int, default=0, help="override the document count")
    ap.add_argument("--config", type=int, default=DEFAULT_CONFIG, help="workload number 1..5")
    ap.add_argument("--K", type=int, default=0)
    ap.add_argument("--b", type=int, default=0)
    ap.add_argument("--r", type=int, default=0)
    ap.add_argument("--shingle-n", type=int, default=0)
    ap.add_argument("--sweep", action="store_true", help="config 5 parameter grid")
    ap.add_argument("--cpu-sample-docs", type=int, default=0,
                    help="documents the oracle is timed on (0: about 12 s of single-thread work)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--theta", type=float, default=0.8,
                    help="similarity threshold of the verified-cluster measurement")
    ap.add_argument("--no-host-leg", action="store_true",
                    help="skip the measurement with the text resident in pinned host memory")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed steps and the roofline (for profiler runs)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of the other workloads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference point for HBM "
                         "byte counters collected with rocprofv3 --pmc)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2501_01046_amd as sedd
    from paper_2501_01046_amd import corpus

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    sedd.lib()
    ncore = min(16, os.cpu_count() or 1)

    recipe = corpus.config(args.config)
    over = {}
    if args.K:
        over["K"] = args.K
    if args.b:
        over["b"] = args.b
    if args.r:
        over["r"] = args.r
    if args.shingle_n:
        over["shingle_n"] = args.shingle_n
    recipe = recipe.scaled(args.docs or recipe.n_docs, **over)
    streamed = args.config == 3
    # documents the oracle legs need on the host: about 12 s of single-thread oracle work
    cpu_docs = args.cpu_sample_docs or {1: 5000, 2: 60000, 3: 15000, 4: 400, 5: 60000}[args.config]
    cpu_docs = min(cpu_docs, recipe.n_docs)

    wl = Workload(torch, sedd, corpus, recipe, streamed, keep_host_docs=cpu_docs)
    n_docs, n_bytes, flags = wl.n_docs, wl.n_bytes, wl.flags
    h_data, h_off = wl.h_data, wl.h_off

    if args.sweep:
        return sweep(args, recipe, wl, sedd, corpus, np, torch)

    K, b, r, n = recipe.K, recipe.b, recipe.r, recipe.shingle_n
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    elapsed, stages, sig, keys, cid = wl.measure(K, b, r, n, args.steps, args.warmup)
    ms_per_step = 1e3 * elapsed / args.steps
    docs_per_s = n_docs * args.steps / elapsed
    text_gbps = n_bytes * args.steps / elapsed / 1e9

    n_shingles = wl.shingle_count(n)          # outside the timed region
    roofline = wl.roofline(stages, args.steps, K, n_shingles)
    if not args.docs and not over:
        roofline["traffic"], src = measured_traffic(recipe.name)
        if src:
            roofline["traffic_source"] = src
    roofline["whole_path_frac"] = round(
        n_shingles * ops_per_shingle(recipe, K) / (ms_per_step * 1e-3) / 1e12 / PEAK_TOPS, 4)
    stage_ms = {k: round(v[0] / args.steps, 4) for k, v in stages.items()}
    min_match = sedd.min_match_for(args.theta, K)

    out = {
        "metric": "MinHash+LSH docs/sec on 1 MI355X (minhash + band keys + clustering)",
        "value": round(docs_per_s, 1), "unit": "docs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64 (61-bit modular) / u32",
        "data": "synthetic",
        "config": {"workload": recipe.name, "n_docs": n_docs, "text_bytes": n_bytes,
                   "shingles": n_shingles, "shingle_n": n, "byte_shingles": bool(recipe.byte_mode),
                   "K": K, "b": b, "r": r, "corpus_seed": recipe.seed, "hash_seed": 0,
                   "minhash_calls_per_step": len(wl.pieces),
                   "piece_bytes": STREAM_CHUNK_BYTES if streamed else n_bytes},
        "text_GB_per_s": round(text_gbps, 3),
        "stage_ms_per_step": stage_ms,
        "duplicates_found": int((cid.cpu().numpy() != np.arange(n_docs)).sum()),
        "corpus_generation_s": round(wl.t_gen, 2),
        "scratch_bytes": sedd.sedd_scratch_bytes(),
        "exact_path_tiles": sedd.debug_stats()[sedd.STAT_SLOW_TILES],
    }

    if args.no_extras:
        out["roofline"] = roofline
        print(json.dumps(out))
        return 0

    # Ceiling of the hot loop on this chip, measured in the same job: the same kernel on full
    # tiles of caller-supplied shingle hashes (no tokenisation, no Eq. 1 work, no short tiles).
    def alu_ceiling():
        per, nd = 4096, 10000
        g = torch.Generator(device="cuda").manual_seed(0)
        xs = torch.randint(0, (1 << 61) - 1, (per * nd,), dtype=torch.int64, device="cuda",
                           generator=g).view(torch.uint64)
        soff = (torch.arange(nd + 1, dtype=torch.int64, device="cuda") * per).view(torch.uint64)
        o = torch.empty((nd, K), dtype=torch.uint32, device="cuda")
        for _ in range(40):                                   # clocks settle within ~50 ms
            sedd.debug_minhash_from_x(xs, soff, K, 0, out=o)
        torch.cuda.synchronize()
        sedd.profile_enable(True)
        sedd.profile_read()
        for _ in range(10):
            sedd.debug_minhash_from_x(xs, soff, K, 0, out=o)
        torch.cuda.synchronize()
        sedd.profile_enable(False)
        ms = sedd.profile_read()["minhash"][0] / 10
        return per * nd * K * OPS_PER_PAIR / (ms * 1e-3) / 1e12

    ceiling = alu_ceiling()
    roofline["hot_loop_ceiling"] = {
        "achieved": round(ceiling, 3), "frac": round(ceiling / PEAK_TOPS, 4),
        "what": "k_minhash on full tiles of given shingle hashes (same launch shape, same K)"}

    # Verified clusters (the paper's count-match step, theta = 0.8): outside the timed steps, on
    # the signatures and keys the last step left in HBM.
    vcid = torch.empty((n_docs,), dtype=torch.int64, device="cuda")
    v_ms, v_stage = timed_calls(torch, sedd,
                                lambda: sedd.sedd_cluster_verified(keys, sig, min_match, out=vcid), 3)
    h_vcid = vcid.cpu().numpy().copy()
    out["verified_clusters"] = {
        "theta": args.theta, "min_match": min_match, "ms_per_call": round(v_ms, 3),
        "stage_ms": v_stage,
        "duplicates_found": int((h_vcid != np.arange(n_docs)).sum()),
        "bucket_balance_61_bit_keys": bucket_balance(torch, keys),
    }

    # The paper's own candidate generation (dense buckets, 4 sqrt(N) of them) followed by the
    # all-pairs count-match verification, with the bucket-balance figures of its imbalance
    # analysis: also outside the timed steps.
    nbk = sedd.dense_bucket_count(n_docs)
    dkeys = torch.empty((n_docs, b), dtype=torch.uint64, device="cuda")

    def dense_flow():
        sedd.sedd_lsh_dense_keys(sig, b, r, nbk, out=dkeys)
        sedd.sedd_cluster_verified(dkeys, sig, min_match, out=vcid)
    d_ms, d_stage = timed_calls(torch, sedd, dense_flow, 3)
    bal = bucket_balance(torch, dkeys, nbk)
    v_s = d_stage.get("verify", 0.0) * 1e-3
    pairs = bal["pair_comparisons"]
    out["dense_buckets_verified"] = {
        "n_buckets": nbk, "ms_per_call": round(d_ms, 3), "stage_ms": d_stage,
        "bucket_balance": bal, "pairs_compared": pairs,
        "pairs_per_s": round(pairs / v_s, 1) if v_s else None,
        # what comparing every pair entry by entry would cost (one compare and one add per
        # pair and signature entry), for scale: the kernel bounds nearly all pairs from
        # one-bit sketches instead, so this exceeds the ALU peak
        "entrywise_equivalent_over_alu_peak": round(pairs * K * 2 / v_s / 1e12 / PEAK_TOPS, 3) if v_s else None,
        "duplicates_found": int((vcid.cpu().numpy() != np.arange(n_docs)).sum()),
        "whole_key_sort_needed": sedd.debug_last_regroup(),
    }
    del dkeys

    out["fidelity_vs_all_pairs"] = fidelity(torch, sedd, np, sig, b, r, min_match, 100_000)

    # The same path under the two other readings of "H hash functions": the paper's own modulus
    # (p = 4,294,967) for Eq. 1 and the K functions, and Eq. 1 itself to K different bases.
    # Outside the timed steps.  Reported per mode: throughput, the instruction-count fraction of
    # its hot kernel, and how well its signatures estimate the Jaccard similarity of planted pairs.
    paper = None
    rolling = None
    if n_docs <= 2_000_000 and not streamed:
        import oracle
        gen = corpus.Corpus(recipe)
        ppairs = []
        for dnum in range(min(n_docs, 200000)):
            kind, src, _ = gen.meta(dnum)
            if kind == 1 and max(h_off[dnum + 1] - h_off[dnum], h_off[src + 1] - h_off[src]) < 50000:
                ppairs.append((dnum, int(src)))
            if len(ppairs) >= 1500:
                break

        def doc(i):
            return h_data[int(h_off[i]):int(h_off[i + 1])].tobytes()
        J = np.array([jaccard_of_pair(oracle, doc(u), doc(v), n, recipe.byte_mode)
                      for u, v in ppairs]) if ppairs else None
        ia = torch.tensor([u for u, _ in ppairs], device="cuda", dtype=torch.int64)
        ib = torch.tensor([v for _, v in ppairs], device="cuda", dtype=torch.int64)

        def estimate_error(sg):
            if not ppairs:
                return None
            s32 = sg.view(torch.int32)
            e = (s32[ia] == s32[ib]).to(torch.float64).mean(dim=1).cpu().numpy() - J
            return {"mean": round(float(e.mean()), 5), "rms": round(float(np.sqrt((e ** 2).mean())), 5)}
        err61 = estimate_error(sig)
        n_long = int((np.diff(h_off.astype(np.int64)) >= 1_000_000).sum())
        h_cid61 = cid.cpu().numpy()

        def mode_leg(mode_flag, ops_ps, steps_m):
            el, st, m_sig, m_keys, m_cid = wl.measure(K, b, r, n, steps_m, 1, flags | mode_flag)
            mh = st["minhash"][0]
            tops = n_shingles * ops_ps * steps_m / (mh * 1e-3) / 1e12 if mh else 0.0
            h_mcid = m_cid.cpu().numpy()
            m_vcid = sedd.sedd_cluster_verified(m_keys, m_sig, min_match).cpu().numpy()
            leg = {
                "docs_per_s": round(n_docs * steps_m / el, 1),
                "ms_per_step": round(1e3 * el / steps_m, 3),
                "stage_ms_per_step": {k: round(v[0] / steps_m, 4) for k, v in st.items() if v[0]},
                "hot_kernel": {"ops_per_shingle": round(ops_ps, 1), "achieved_TOPs": round(tops, 3),
                               "frac_of_alu_peak": round(tops / PEAK_TOPS, 4),
                               "hash_evals_per_s": round(n_shingles * K * steps_m / (mh * 1e-3), 1)
                               if mh else 0},
                "jaccard_estimate": {"planted_pairs": len(ppairs),
                                     "mean_jaccard": round(float(J.mean()), 4) if ppairs else None,
                                     "error": estimate_error(m_sig), "error_61_bit_affine": err61,
                                     "sampling_rms_expected":
                                         round(float(np.sqrt((J * (1 - J) / K).mean())), 5) if ppairs else None},
                "duplicates_found": int((h_mcid != np.arange(n_docs)).sum()),
                "verified_duplicates_found": int((m_vcid != np.arange(n_docs)).sum()),
                "verified_duplicates_found_61_bit_affine": int((h_vcid != np.arange(n_docs)).sum()),
                # range exhaustion: documents of a million shingles or more leave minima near 0
                "documents_of_1MB_or_more": n_long,
                "largest_cluster": int(np.bincount(h_mcid).max()),
                "largest_cluster_61_bit_affine": int(np.bincount(h_cid61).max()),
                "largest_verified_cluster": int(np.bincount(m_vcid).max()),
                "largest_verified_cluster_61_bit_affine": int(np.bincount(h_vcid).max()),
            }
            del m_sig, m_keys, m_cid
            return leg

        paper = mode_leg(sedd.FLAG_PAPER_PRIME, ops_per_shingle_pp(recipe, K),
                         max(1, min(3, args.steps)))
        paper["modulus"] = 4294967
        # rolling family: per (shingle, function) about (mean token length + n - 1) modular
        # multiply-adds of 8 operations on word shingles, 2 on byte shingles
        if recipe.byte_mode:
            rf_mads = 2.0
        else:
            tokens = n_shingles + (n - 1) * n_docs
            rf_mads = (n_bytes - tokens) / max(1, tokens) + (n - 1)
        rolling = mode_leg(sedd.FLAG_ROLLING_FAMILY, K * rf_mads * OPS_PER_PAIR, 1)
        rolling["multiply_adds_per_evaluation"] = round(rf_mads, 2)
    out["paper_prime_mode"] = paper
    out["rolling_family_mode"] = rolling

    # The same path with the text resident in pinned HOST memory: pieces of at most 2 GB go
    # through two device staging buffers, the upload of piece i+1 on a copy stream overlapping
    # sedd_minhash of piece i.  Outside the timed steps; never the headline value.
    host_leg = None
    if not args.no_host_leg:
        host_leg = host_fed_leg(torch, sedd, np, wl, sig, keys, cid, K, b, r, n, args.steps)
    out["host_resident_input"] = host_leg

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(cpu_docs, h_off.size - 1)
        sub_off = h_off[: ns + 1]
        sub = h_data[: int(sub_off[-1])]
        t0 = time.perf_counter()
        o_sig = oracle.minhash(sub, sub_off, n, K, 0, flags)
        o_keys = oracle.lsh_keys(o_sig, b, r)
        oracle.cluster(o_keys)
        t_cpu = time.perf_counter() - t0
        # the same oracle as one worker thread per core over disjoint document ranges
        # (signatures only shard; band keys and clusters stay single-threaded), measured
        t0 = time.perf_counter()
        m_sig = oracle.minhash_sharded(sub, sub_off, n, K, 0, flags, procs=ncore)
        oracle.cluster(oracle.lsh_keys(m_sig, b, r))
        t_all = time.perf_counter() - t0
        cpu_baseline = {
            "value": round(ns / t_cpu, 2), "unit": "docs/s", "cores": 1, "kind": "oracle",
            "cpu_model": cpu_model(), "host_cores_visible": os.cpu_count(),
            "text_GB_per_s": round(int(sub_off[-1]) / t_cpu / 1e9, 5),
            "sample": f"first {ns} documents of the same corpus ({int(sub_off[-1])} bytes), "
                      f"minhash + band keys + clusters, single thread, {t_cpu:.1f} s",
            "all_cores": {"value": round(ns / t_all, 2), "unit": "docs/s", "cores": ncore,
                          "seconds": round(t_all, 2), "same_signatures": bool(np.array_equal(m_sig, o_sig))},
        }
        # the sample doubles as a parity spot check of the timed configuration
        parity, _ = wl.parity_sample(oracle, np, sig, keys, n, K, b, r, ns, min_match, ncore)
    out["roofline"] = roofline
    out["cpu_baseline"] = cpu_baseline
    out["parity_sample_ok"] = parity

    # A short run of the other workloads, so that every figure quoted for them has a record from
    # the same job: throughput, the dominant kernel's fraction of the ALU peak, and the oracle's
    # whole path on a prefix.  The large buffers of the headline workload are released first.
    per_config = None
    if not args.no_per_config and not args.docs and not over:
        del sig, keys, cid, vcid
        wl.pieces = []
        torch.cuda.empty_cache()
        per_config = []
        for c in (1, 2, 4):
            if c == args.config:
                continue
            per_config.append(short_run(torch, sedd, corpus, np, c, ncore, args.theta,
                                        None if args.no_cpu_baseline else 1))
    out["per_config"] = per_config
    print(json.dumps(out))
    return 0


def short_run(torch, sedd, corpus, np, c, ncore, theta, with_parity):
    rc = corpus.config(c)
    parity_docs = {1: 5000, 2: 20000, 3: 5000, 4: 1500, 5: 20000}[c]
    w = Workload(torch, sedd, corpus, rc, streamed=(c == 3), keep_host_docs=parity_docs)
    steps = 5 if c != 4 else 3
    el, st, sig, keys, cid = w.measure(rc.K, rc.b, rc.r, rc.shingle_n, steps, 1)
    nsh = w.shingle_count(rc.shingle_n)
    rl = w.roofline(st, steps, rc.K, nsh)
    ms = 1e3 * el / steps
    entry = {
        "workload": rc.name, "n_docs": rc.n_docs, "text_bytes": w.n_bytes, "shingles": nsh,
        "K": rc.K, "b": rc.b, "r": rc.r, "shingle_n": rc.shingle_n,
        "byte_shingles": bool(rc.byte_mode), "steps": steps,
        "docs_per_s": round(rc.n_docs * steps / el, 1),
        "text_GB_per_s": round(w.n_bytes * steps / el / 1e9, 3), "ms_per_step": round(ms, 3),
        "stage_ms_per_step": {k: round(v[0] / steps, 4) for k, v in st.items() if v[0]},
        "k_minhash_frac_of_alu_peak": rl["frac"],
        "whole_path_frac_of_alu_peak": round(
            nsh * ops_per_shingle(rc, rc.K) / (ms * 1e-3) / 1e12 / PEAK_TOPS, 4),
        "duplicates_found": int((cid.cpu().numpy() != np.arange(rc.n_docs)).sum()),
        "parity_sample_ok": None,
    }
    if c in (1, 2):
        entry["fidelity_vs_all_pairs"] = fidelity(torch, sedd, np, sig, rc.b, rc.r,
                                                  sedd.min_match_for(theta, rc.K), 100_000)
    if with_parity:
        import oracle
        ok, ns = w.parity_sample(oracle, np, sig, keys, rc.shingle_n, rc.K, rc.b, rc.r, parity_docs,
                                 sedd.min_match_for(theta, rc.K), ncore)
        entry["parity_sample_ok"] = ok
        entry["parity_sample_docs"] = ns
    del sig, keys, cid, w
    torch.cuda.empty_cache()
    return entry


def host_fed_leg(torch, sedd, np, wl, sig, keys, cid, K, b, r, n, steps):
    """The whole corpus in pinned host memory, fed through sedd_minhash_host_chunked: the library
    uploads pieces of at most 2 GB into two device staging buffers on its own stream while
    sedd_minhash works on the previous piece."""
    n_bytes, flags = wl.n_bytes, wl.flags
    chunk = min(STREAM_CHUNK_BYTES, max(64 << 20, n_bytes // 6))
    try:
        import psutil
        avail = psutil.virtual_memory().available
    except Exception:
        avail = 64 << 30
    # pinned copy of the text: leave half of the free host memory alone
    budget = int(min(n_bytes, max(1 << 30, avail // 2)))
    take, tot = [], 0
    for text, off, d0, d1 in wl.pieces:
        if tot >= budget:
            break
        take.append((text, off, d0, d1))
        tot += text.numel()
    leg_docs = take[-1][3]
    h_text = torch.empty(tot, dtype=torch.uint8, pin_memory=True)
    h_off = torch.empty(leg_docs + 1, dtype=torch.int64, pin_memory=True)
    at = 0
    for text, off, d0, d1 in take:
        h_text[at:at + text.numel()].copy_(text)                     # device -> pinned host
        h_off[d0:d1 + 1].copy_((off.view(torch.int64) + at).cpu())
        at += text.numel()
    torch.cuda.synchronize()
    h_sig = torch.empty((leg_docs, K), dtype=torch.uint32, device="cuda")

    def one_pass():
        sedd.sedd_minhash_host_chunked(h_text, h_off, n, K, 0, flags, chunk_bytes=chunk, out=h_sig)
        sedd.sedd_lsh_keys(h_sig, b, r, out=keys[:leg_docs])
        sedd.sedd_cluster(keys[:leg_docs], out=cid[:leg_docs])

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps
    reps = max(1, min(3, steps)) if tot < (8 << 30) else 1
    t_path = timed(one_pass, reps)
    same = bool(torch.equal(h_sig.view(torch.int32), sig[:leg_docs].view(torch.int32)))
    # the upload by itself, same piece size, through one device buffer
    stage = torch.empty(min(chunk, tot) + 16, dtype=torch.uint8, device="cuda")

    def upload_only():
        for a in range(0, tot, chunk):
            e = min(tot, a + chunk)
            stage[:e - a].copy_(h_text[a:e], non_blocking=True)
    t_copy = timed(upload_only, reps)
    leg = {
        "what": "text in pinned host memory through sedd_minhash_host_chunked (double-buffered "
                "upload overlapped with the hashing); then band keys and clusters of the same documents",
        "documents": leg_docs, "text_bytes": tot, "whole_corpus": bool(tot >= n_bytes),
        "piece_bytes": chunk,
        "ms_per_pass": round(1e3 * t_path, 3), "docs_per_s": round(leg_docs / t_path, 1),
        "text_GB_per_s": round(tot / t_path / 1e9, 3),
        "upload_only_ms_per_pass": round(1e3 * t_copy, 3),
        "upload_only_GB_per_s": round(tot / t_copy / 1e9, 3),
        "signatures_equal_device_resident_run": same,
    }
    if tot < n_bytes:
        leg["why_not_whole_corpus"] = (f"pinned copy bounded to half of the free host memory "
                                       f"({avail >> 30} GiB free)")
    # keys and cid held the whole corpus before this leg: restore them
    sedd.sedd_lsh_keys(sig, b, r, out=keys)
    sedd.sedd_cluster(keys, out=cid)
    sedd.sedd_release_scratch()              # the staging buffers are as large as two pieces
    return leg


def sweep(args, recipe, wl, sedd, corpus, np, torch):
    """Config 5: K x (b, r) x shingle length grid; throughput and the S-curve fit per setting.
    K = 64 admits none of the grid's (b, r) (all need b*r >= 128); it gets a signatures-only row."""
    import oracle
    n_docs, n_bytes = wl.n_docs, wl.n_bytes
    gen = corpus.Corpus(recipe)
    text, off, _, _ = wl.pieces[0]
    h_off = off.cpu().numpy()
    # planted pairs: near-duplicates and their sources, exact Jaccard from brute-force shingle sets
    rng = np.random.default_rng(0)
    cand = rng.choice(n_docs, size=min(n_docs, 60000), replace=False)
    pairs = []
    for dnum in cand:
        kind, src, _ = gen.meta(int(dnum))
        if kind == 1:
            pairs.append((int(dnum), int(src)))
        if len(pairs) >= 3000:
            break
    h_text = text.cpu().numpy()

    def doc(i):
        return h_text[int(h_off[i]):int(h_off[i + 1])].tobytes()

    def frac(n_sh, n, K, mh_ms):
        return round(n_sh * ops_per_shingle(recipe.scaled(n_docs, shingle_n=n), K)
                     / (mh_ms * 1e-3) / 1e12 / PEAK_TOPS, 4)

    results = []
    for n in (3, 5):
        J = np.array([jaccard_of_pair(oracle, doc(a), doc(b_), n, recipe.byte_mode)
                      for a, b_ in pairs])
        n_sh = wl.shingle_count(n)
        for K in (64, 128, 256, 512):
            grid = [(b, r) for (b, r) in ((8, 16), (16, 8), (32, 8), (64, 4)) if b * r <= K]
            for (b, r) in ((8, 16), (16, 8), (32, 8), (64, 4)):
                if b * r > K:
                    results.append({"n": n, "K": K, "b": b, "r": r, "skipped": "b*r > K"})
            if not grid:
                # signatures only: sedd_minhash timed by itself
                sig = torch.empty((n_docs, K), dtype=torch.uint32, device="cuda")
                sedd.sedd_minhash(text, off, n, K, 0, wl.flags, out=sig)
                torch.cuda.synchronize()
                sedd.profile_enable(True)
                sedd.profile_read()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    sedd.sedd_minhash(text, off, n, K, 0, wl.flags, out=sig)
                torch.cuda.synchronize()
                el = time.perf_counter() - t0
                sedd.profile_enable(False)
                st = sedd.profile_read()
                mh_ms = st["minhash"][0] / args.steps
                results.append({
                    "n": n, "K": K, "signatures_only": True,
                    "docs_per_s": round(n_docs * args.steps / el, 1),
                    "text_GB_per_s": round(n_bytes * args.steps / el / 1e9, 3),
                    "minhash_ms": round(mh_ms, 3),
                    "minhash_frac_of_alu_peak": frac(n_sh, n, K, mh_ms)})
                del sig
                continue
            for (b, r) in grid:
                elapsed, stages, sig, keys, cid = wl.measure(K, b, r, n, args.steps, 1)
                k_host = keys.cpu().numpy()
                ia = np.array([p[0] for p in pairs])
                ib = np.array([p[1] for p in pairs])
                hit = (k_host[ia] == k_host[ib]).any(axis=1)
                # binned recall against 1-(1-s^r)^b
                bins = np.linspace(0.0, 1.0, 11)
                dev2, used = 0.0, 0
                for lo, hi in zip(bins[:-1], bins[1:]):
                    msk = (J >= lo) & (J < hi if hi < 1.0 else J <= hi)
                    if msk.sum() >= 30:
                        want = (1 - (1 - J[msk] ** r) ** b).mean()
                        dev2 += (hit[msk].mean() - want) ** 2
                        used += 1
                mh_ms = stages["minhash"][0] / args.steps
                results.append({
                    "n": n, "K": K, "b": b, "r": r,
                    "docs_per_s": round(n_docs * args.steps / elapsed, 1),
                    "text_GB_per_s": round(n_bytes * args.steps / elapsed / 1e9, 3),
                    "minhash_ms": round(mh_ms, 3),
                    "minhash_frac_of_alu_peak": frac(n_sh, n, K, mh_ms),
                    "keys_cluster_ms": round((stages["lsh_keys"][0] + stages["sort"][0]
                                              + stages["union_find"][0]) / args.steps, 3),
                    "scurve_rms": round(float(np.sqrt(dev2 / max(1, used))), 4),
                    "scurve_bins": used, "planted_pairs": len(pairs),
                    "duplicates_found": int((cid.cpu().numpy() != np.arange(n_docs)).sum()),
                })
                del sig, keys, cid
    print(json.dumps({"metric": "config 5 parameter sweep", "workload": recipe.name,
                      "n_docs": n_docs, "text_bytes": n_bytes, "steps": args.steps,
                      "results": results}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
