#!/usr/bin/env python3
"""Benchmark of the MinHash-LSH hot path on one MI355X.

A step is one pass of the whole path (sedd_minhash -> sedd_lsh_keys -> sedd_cluster) over one
batch of synthetic input that is already resident in HBM.  The default workload is the medium
one the headline metric is quoted on: 1M web-text-shaped documents, 5-word shingles, K=128,
16 bands of 8 rows.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--docs N]
                    [--sweep] [--no-cpu-baseline] [--no-host-leg]

--config 3 keeps the whole text resident and feeds sedd_minhash 2 GB at a time; --config 5
--sweep runs the K x (b, r) x n grid and adds the planted-pair S-curve fit per setting.
After the timed steps the same buffers serve a few untimed measurements reported beside the
headline: verified clusters, the dense-bucket flow, the two alternative hash-function modes, and
the path fed from pinned host memory (the PCIe-inclusive rate).
The CPU oracle is timed on a bounded sample of the same corpus and reported beside the GPU
figure as `cpu_baseline`; it is a reported baseline, not the target.
"""
from __future__ import annotations

import argparse
import json
import os
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
# HBM bytes one k_minhash launch moves on the default workload (one 256 MB chunk), from the two
# rocprofv3 --pmc runs summarised in profiles/hbm_traffic_cfg2_medium_1M.txt (FETCH_SIZE x 2 KiB
# + WRITE_SIZE x 1 KiB, both scaled by a 1 GiB copy).  It is a recorded measurement, not
# collected by this script; it only applies to the default workload.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH_CFG2 = 592.7e6


def ops_per_shingle(recipe, K):
    if recipe.byte_mode:
        base = recipe.shingle_n * OPS_PER_BASE_STEP_BYTE
    else:
        base = (recipe.shingle_n - 1) * OPS_PER_BASE_STEP_WORD
    return K * OPS_PER_PAIR + base


def ops_per_shingle_pp(recipe, K):
    base = (2 if recipe.byte_mode else recipe.shingle_n - 1) * OPS_PER_BASE_STEP_PP
    return K * OPS_PER_PAIR_PP + base


def load_corpus(torch, corpus, recipe, stream_chunk=None):
    """Generate the corpus and place it in HBM.  Returns a list of (text, offsets, d0, d1)
    device pieces (one piece unless stream_chunk is given), total bytes, and the host arrays of
    the first piece (for the oracle sample)."""
    gen = corpus.Corpus(recipe)
    pieces = []
    total = 0
    first_host = None
    if stream_chunk is None:
        data, off = gen.generate()
        pieces.append((torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(), 0, recipe.n_docs))
        return pieces, int(data.size), (data, off)
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
        if first_host is None:
            first_host = (data, off)
        pieces.append((torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(), d0, d1))
        total += int(data.size)
        d0 = d1
    return pieces, total, first_host


def jaccard_of_pair(oracle, a: bytes, b: bytes, n: int, byte_mode: bool) -> float:
    sa = set(oracle.doc_shingles(a, n, byte_mode).tolist())
    sb = set(oracle.doc_shingles(b, n, byte_mode).tolist())
    if not sa and not sb:
        return 1.0
    return len(sa & sb) / len(sa | sb)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--docs", type=int, default=0, help="override the document count")
    ap.add_argument("--config", type=int, default=2, help="workload number 1..5")
    ap.add_argument("--K", type=int, default=0)
    ap.add_argument("--b", type=int, default=0)
    ap.add_argument("--r", type=int, default=0)
    ap.add_argument("--shingle-n", type=int, default=0)
    ap.add_argument("--sweep", action="store_true", help="config 5 parameter grid")
    ap.add_argument("--cpu-sample-docs", type=int, default=60000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--theta", type=float, default=0.8,
                    help="similarity threshold of the verified-cluster measurement")
    ap.add_argument("--no-host-leg", action="store_true",
                    help="skip the measurement with the text resident in pinned host memory")
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
    flags = sedd.FLAG_BYTE_SHINGLES if recipe.byte_mode else 0
    streamed = args.config == 3

    t0 = time.time()
    pieces, n_bytes, (h_data, h_off) = load_corpus(torch, corpus, recipe,
                                                   STREAM_CHUNK_BYTES if streamed else None)
    t_gen = time.time() - t0
    n_docs = recipe.n_docs

    def run_path(K, b, r, n, sig, keys, cid, mode_flags):
        for text, off, d0, d1 in pieces:
            sedd.sedd_minhash(text, off, n, K, 0, mode_flags, out=sig[d0:d1])
        sedd.sedd_lsh_keys(sig, b, r, out=keys)
        sedd.sedd_cluster(keys, out=cid)

    def measure(K, b, r, n, steps, warmup, mode_flags=flags):
        sig = torch.empty((n_docs, K), dtype=torch.uint32, device="cuda")
        keys = torch.empty((n_docs, b), dtype=torch.uint64, device="cuda")
        cid = torch.empty((n_docs,), dtype=torch.int64, device="cuda")
        for _ in range(warmup):
            run_path(K, b, r, n, sig, keys, cid, mode_flags)
        torch.cuda.synchronize()
        sedd.profile_enable(True)
        sedd.profile_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run_path(K, b, r, n, sig, keys, cid, mode_flags)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        sedd.profile_enable(False)
        return elapsed, sedd.profile_read(), sig, keys, cid

    def shingle_count(n):
        tot = 0
        for text, off, d0, d1 in pieces:
            _, soff = sedd.debug_shingle_hashes_offsets(text, off, n, flags)
            tot += int(soff[-1])
        return tot

    if args.sweep:
        return sweep(args, recipe, pieces, measure, shingle_count, sedd, corpus, np, torch,
                     n_docs, n_bytes, flags)

    K, b, r, n = recipe.K, recipe.b, recipe.r, recipe.shingle_n
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    elapsed, stages, sig, keys, cid = measure(K, b, r, n, args.steps, args.warmup)
    ms_per_step = 1e3 * elapsed / args.steps
    docs_per_s = n_docs * args.steps / elapsed
    text_gbps = n_bytes * args.steps / elapsed / 1e9

    n_shingles = shingle_count(n)          # outside the timed region
    mh_ms, mh_spans = stages["minhash"]
    ops_per_step = n_shingles * ops_per_shingle(recipe, K)
    launches_per_step = max(1, mh_spans // max(1, args.steps))
    avg_launch_ms = mh_ms / max(1, mh_spans)
    achieved = ops_per_step * args.steps / (mh_ms * 1e-3) / 1e12 if mh_ms else 0.0
    roofline = {
        "kernel": "k_minhash", "bound": "alu", "achieved": round(achieved, 3),
        "peak": round(PEAK_TOPS, 3), "unit": "TOP/s (int32 VALU lane-ops)",
        "frac": round(achieved / PEAK_TOPS, 4),
        "traffic": (MEASURED_TRAFFIC_BYTES_PER_LAUNCH_CFG2
                    if args.config == 2 and not args.docs and not over else None),
        "ops_per_shingle": ops_per_shingle(recipe, K), "shingles_per_step": n_shingles,
        "ops_per_launch": ops_per_step // launches_per_step,
        "launches_per_step": launches_per_step, "avg_launch_ms": round(avg_launch_ms, 4),
        "hash_evals_per_s": round(n_shingles * K * args.steps / (mh_ms * 1e-3), 1) if mh_ms else 0,
    }
    stage_ms = {k: round(v[0] / args.steps, 4) for k, v in stages.items()}

    # Ceiling of the hot loop on this chip, measured in the same job: the same kernel on full
    # tiles of caller-supplied shingle hashes (no tokenisation, no Eq. 1 work, no short tiles).
    def alu_ceiling():
        per, nd = 4096, 10000
        g = torch.Generator(device="cuda").manual_seed(0)
        xs = torch.randint(0, (1 << 61) - 1, (per * nd,), dtype=torch.int64, device="cuda",
                           generator=g).view(torch.uint64)
        soff = (torch.arange(nd + 1, dtype=torch.int64, device="cuda") * per).view(torch.uint64)
        out = torch.empty((nd, K), dtype=torch.uint32, device="cuda")
        for _ in range(40):                                   # clocks settle within ~50 ms
            sedd.debug_minhash_from_x(xs, soff, K, 0, out=out)
        torch.cuda.synchronize()
        sedd.profile_enable(True)
        sedd.profile_read()
        for _ in range(10):
            sedd.debug_minhash_from_x(xs, soff, K, 0, out=out)
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
    min_match = sedd.min_match_for(args.theta, K)
    vcid = torch.empty((n_docs,), dtype=torch.int64, device="cuda")
    sedd.sedd_cluster_verified(keys, sig, min_match, out=vcid)
    torch.cuda.synchronize()
    sedd.profile_enable(True)
    sedd.profile_read()
    t0 = time.perf_counter()
    for _ in range(3):
        sedd.sedd_cluster_verified(keys, sig, min_match, out=vcid)
    torch.cuda.synchronize()
    v_ms = 1e3 * (time.perf_counter() - t0) / 3
    sedd.profile_enable(False)
    v_stages = sedd.profile_read()
    verified = {
        "theta": args.theta, "min_match": min_match, "ms_per_call": round(v_ms, 3),
        "stage_ms": {k: round(v[0] / 3, 4) for k, v in v_stages.items() if v[0]},
        "duplicates_found": int((vcid.cpu().numpy() != np.arange(n_docs)).sum()),
    }
    h_vcid = vcid.cpu().numpy().copy()

    # The paper's own candidate generation (dense buckets, 4 sqrt(N) of them) followed by the
    # all-pairs count-match verification: also outside the timed steps.
    dense = None
    if n_docs <= 2_000_000:
        nbk = sedd.dense_bucket_count(n_docs)
        dkeys = torch.empty((n_docs, b), dtype=torch.uint64, device="cuda")
        sedd.sedd_lsh_dense_keys(sig, b, r, nbk, out=dkeys)
        sedd.sedd_cluster_verified(dkeys, sig, min_match, out=vcid)
        torch.cuda.synchronize()
        sedd.profile_enable(True)
        sedd.profile_read()
        t0 = time.perf_counter()
        for _ in range(3):
            sedd.sedd_lsh_dense_keys(sig, b, r, nbk, out=dkeys)
            sedd.sedd_cluster_verified(dkeys, sig, min_match, out=vcid)
        torch.cuda.synchronize()
        d_ms = 1e3 * (time.perf_counter() - t0) / 3
        sedd.profile_enable(False)
        d_stages = sedd.profile_read()
        pairs = 0
        for j in range(b):
            cnt = torch.bincount(dkeys[:, j].view(torch.int64), minlength=nbk).to(torch.float64)
            pairs += int((cnt * (cnt - 1) / 2).sum().item())
        v_s = d_stages["verify"][0] / 3 * 1e-3
        dense = {
            "n_buckets": nbk, "mean_bucket": round(n_docs / nbk, 1), "ms_per_call": round(d_ms, 3),
            "stage_ms": {k: round(v[0] / 3, 4) for k, v in d_stages.items() if v[0]},
            "pairs_compared": pairs,
            "pairs_per_s": round(pairs / v_s, 1) if v_s else None,
            # what comparing every pair entry by entry would cost (one compare and one add per
            # pair and signature entry), for scale: the kernel bounds nearly all pairs from
            # one-bit sketches instead, so this exceeds the ALU peak
            "entrywise_equivalent_TOPs": round(pairs * K * 2 / v_s / 1e12, 3) if v_s else None,
            "entrywise_equivalent_over_alu_peak": round(pairs * K * 2 / v_s / 1e12 / PEAK_TOPS, 3) if v_s else None,
            "duplicates_found": int((vcid.cpu().numpy() != np.arange(n_docs)).sum()),
        }
        del dkeys

    # The same path under the two other readings of "H hash functions": the paper's own modulus
    # (p = 4,294,967) for Eq. 1 and the K functions, and Eq. 1 itself to K different bases.
    # Outside the timed steps.  Reported per mode: throughput, the instruction-count fraction of
    # its hot kernel, and how well its signatures estimate the Jaccard similarity of planted pairs.
    paper = None
    rolling = None
    if n_docs <= 2_000_000 and not streamed:
        import oracle
        gen = corpus.Corpus(recipe)
        pairs = []
        for dnum in range(min(n_docs, 200000)):
            kind, src, _ = gen.meta(dnum)
            if kind == 1 and max(h_off[dnum + 1] - h_off[dnum], h_off[src + 1] - h_off[src]) < 50000:
                pairs.append((dnum, int(src)))
            if len(pairs) >= 1500:
                break

        def doc(i):
            return h_data[int(h_off[i]):int(h_off[i + 1])].tobytes()
        J = np.array([jaccard_of_pair(oracle, doc(u), doc(v), n, recipe.byte_mode)
                      for u, v in pairs]) if pairs else None
        ia = torch.tensor([u for u, _ in pairs], device="cuda", dtype=torch.int64)
        ib = torch.tensor([v for _, v in pairs], device="cuda", dtype=torch.int64)

        def estimate_error(sg):
            if not pairs:
                return None
            s32 = sg.view(torch.int32)
            e = (s32[ia] == s32[ib]).to(torch.float64).mean(dim=1).cpu().numpy() - J
            return {"mean": round(float(e.mean()), 5), "rms": round(float(np.sqrt((e ** 2).mean())), 5)}
        err61 = estimate_error(sig)
        n_long = int((np.diff(h_off.astype(np.int64)) >= 1_000_000).sum())
        h_cid61 = cid.cpu().numpy()

        def mode_leg(mode_flag, ops_ps, steps_m):
            el, st, m_sig, m_keys, m_cid = measure(K, b, r, n, steps_m, 1, flags | mode_flag)
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
                "jaccard_estimate": {"planted_pairs": len(pairs),
                                     "mean_jaccard": round(float(J.mean()), 4) if pairs else None,
                                     "error": estimate_error(m_sig), "error_61_bit_affine": err61,
                                     "sampling_rms_expected":
                                         round(float(np.sqrt((J * (1 - J) / K).mean())), 5) if pairs else None},
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

    # The same path with the text resident in pinned HOST memory: pieces of at most 2 GB go
    # through two device staging buffers, the upload of piece i+1 on a copy stream overlapping
    # sedd_minhash of piece i.  Outside the timed steps; never the headline value.
    host_leg = None
    if not args.no_host_leg:
        HOST_LEG_BYTES = 8 << 30
        chunk = min(STREAM_CHUNK_BYTES, max(64 << 20, n_bytes // 6))
        subs, tot = [], 0
        for text, off, d0, d1 in pieces:
            if tot >= HOST_LEG_BYTES:
                break
            h_t, h_o = text.cpu().numpy(), off.cpu().numpy()
            a, nd = 0, d1 - d0
            while a < nd and tot < HOST_LEG_BYTES:
                e = int(np.searchsorted(h_o, h_o[a] + np.uint64(chunk), side="right")) - 1
                e = min(nd, max(a + 1, e))
                lo, hi = int(h_o[a]), int(h_o[e])
                p_t = torch.empty(hi - lo, dtype=torch.uint8, pin_memory=True)
                p_t.numpy()[:] = h_t[lo:hi]
                p_o = torch.empty(e - a + 1, dtype=torch.int64, pin_memory=True)
                p_o.numpy()[:] = (h_o[a:e + 1] - h_o[a]).view(np.int64)
                subs.append((p_t, p_o, d0 + a, d0 + e))
                tot += hi - lo
                a = e
            del h_t, h_o
        leg_docs = subs[-1][3]                       # documents [0, leg_docs) take part
        stage = [(torch.empty(max(x[0].numel() for x in subs), dtype=torch.uint8, device="cuda"),
                  torch.empty(max(x[1].numel() for x in subs), dtype=torch.int64, device="cuda"))
                 for _ in range(2)]
        copy_s, comp_s = torch.cuda.Stream(), torch.cuda.current_stream()
        ref = sig[:leg_docs].clone()
        h_sig = torch.empty_like(ref)

        def one_pass(compute):
            done, copied = [None, None], {}

            def upload(i):
                t, o, _, _ = subs[i]
                st = stage[i % 2]
                with torch.cuda.stream(copy_s):
                    if done[i % 2] is not None:
                        copy_s.wait_event(done[i % 2])
                    st[0][:t.numel()].copy_(t, non_blocking=True)
                    st[1][:o.numel()].copy_(o, non_blocking=True)
                    ev = torch.cuda.Event()
                    ev.record(copy_s)
                    copied[i] = ev
            upload(0)
            for i in range(len(subs)):
                if i + 1 < len(subs):
                    upload(i + 1)
                comp_s.wait_event(copied[i])
                t, o, d0, d1 = subs[i]
                st = stage[i % 2]
                if compute:
                    sedd.sedd_minhash(st[0][:t.numel()], st[1][:o.numel()].view(torch.uint64), n, K,
                                      0, flags, out=h_sig[d0:d1])
                ev = torch.cuda.Event()
                ev.record(comp_s)
                done[i % 2] = ev
            if compute:
                sedd.sedd_lsh_keys(h_sig, b, r, out=keys[:leg_docs])
                sedd.sedd_cluster(keys[:leg_docs], out=cid[:leg_docs])

        def timed(compute, reps):
            one_pass(compute)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                one_pass(compute)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps
        reps = max(1, min(3, args.steps))
        t_path = timed(True, reps)
        same = bool(torch.equal(h_sig.view(torch.int32), ref.view(torch.int32)))
        t_copy = timed(False, reps)
        host_leg = {
            "what": "text in pinned host memory, double-buffered upload overlapped with sedd_minhash; "
                    "then band keys and clusters of the same documents",
            "documents": leg_docs, "text_bytes": tot, "pieces": len(subs), "piece_bytes": chunk,
            "ms_per_pass": round(1e3 * t_path, 3), "docs_per_s": round(leg_docs / t_path, 1),
            "text_GB_per_s": round(tot / t_path / 1e9, 3),
            "upload_only_ms_per_pass": round(1e3 * t_copy, 3),
            "upload_only_GB_per_s": round(tot / t_copy / 1e9, 3),
            "signatures_equal_device_resident_run": same,
        }
        # keys and cid held the whole corpus before this leg: restore them
        sedd.sedd_lsh_keys(sig, b, r, out=keys)
        sedd.sedd_cluster(keys, out=cid)
        del stage, subs, ref, h_sig

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_docs, h_off.size - 1)
        sub_off = h_off[: ns + 1]
        sub = h_data[: int(sub_off[-1])]
        t0 = time.perf_counter()
        o_sig = oracle.minhash(sub, sub_off, n, K, 0, flags)
        o_keys = oracle.lsh_keys(o_sig, b, r)
        o_cid = oracle.cluster(o_keys)
        t_cpu = time.perf_counter() - t0
        # the same oracle as one process per core over disjoint document ranges (signatures
        # only shard; band keys and clusters stay single-threaded), measured, not extrapolated
        ncore = min(16, os.cpu_count() or 1)
        t0 = time.perf_counter()
        m_sig = oracle.minhash_sharded(sub, sub_off, n, K, 0, flags, procs=ncore)
        oracle.cluster(oracle.lsh_keys(m_sig, b, r))
        t_all = time.perf_counter() - t0
        cpu_baseline = {
            "value": round(ns / t_cpu, 2), "unit": "docs/s", "cores": 1, "kind": "oracle",
            "text_GB_per_s": round(int(sub_off[-1]) / t_cpu / 1e9, 5),
            "sample": f"first {ns} documents of the same corpus ({int(sub_off[-1])} bytes), "
                      f"minhash + band keys + clusters, single thread, {t_cpu:.1f} s",
            "all_cores": {"value": round(ns / t_all, 2), "unit": "docs/s", "cores": ncore,
                          "seconds": round(t_all, 2), "same_signatures": bool(np.array_equal(m_sig, o_sig))},
        }
        # the sample doubles as a parity spot check of the timed configuration
        o_vcid = oracle.cluster_verified(o_keys, o_sig, min_match)
        s_vcid = sedd.sedd_cluster_verified(keys[:ns].contiguous(), sig[:ns].contiguous(), min_match)
        parity = bool(np.array_equal(sig[:ns].cpu().numpy(), o_sig)
                      and np.array_equal(keys[:ns].cpu().numpy(), o_keys)
                      and np.array_equal(
                          sedd.sedd_cluster(keys[:ns].contiguous()).cpu().numpy(), o_cid)
                      and np.array_equal(s_vcid.cpu().numpy(), o_vcid))

    out = {
        "metric": "MinHash+LSH docs/sec on 1 MI355X (minhash + band keys + clustering)",
        "value": round(docs_per_s, 1), "unit": "docs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64 (61-bit modular) / u32",
        "data": "synthetic",
        "config": {"workload": recipe.name, "n_docs": n_docs, "text_bytes": n_bytes,
                   "shingles": n_shingles, "shingle_n": n, "byte_shingles": bool(recipe.byte_mode),
                   "K": K, "b": b, "r": r, "corpus_seed": recipe.seed, "hash_seed": 0,
                   "minhash_calls_per_step": len(pieces)},
        "text_GB_per_s": round(text_gbps, 3),
        "stage_ms_per_step": stage_ms,
        "duplicates_found": int((cid.cpu().numpy() != np.arange(n_docs)).sum()),
        "corpus_generation_s": round(t_gen, 2),
        "scratch_bytes": sedd.sedd_scratch_bytes(),
        "exact_path_tiles": sedd.debug_stats()[sedd.STAT_SLOW_TILES],
        "verified_clusters": verified,
        "dense_buckets_verified": dense,
        "paper_prime_mode": paper,
        "rolling_family_mode": rolling,
        "host_resident_input": host_leg,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity_sample_ok": parity,
    }
    print(json.dumps(out))
    return 0


def sweep(args, recipe, pieces, measure, shingle_count, sedd, corpus, np, torch, n_docs, n_bytes,
          flags):
    """Config 5: K x (b, r) x shingle length grid; throughput and the S-curve fit per setting."""
    import oracle
    gen = corpus.Corpus(recipe)
    text, off, _, _ = pieces[0]
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

    results = []
    for n in (3, 5):
        J = np.array([jaccard_of_pair(oracle, doc(a), doc(b_), n, recipe.byte_mode)
                      for a, b_ in pairs])
        n_sh = shingle_count(n)
        for K in (64, 128, 256, 512):
            sig_time = None
            for (b, r) in ((8, 16), (16, 8), (32, 8), (64, 4)):
                if b * r > K:
                    results.append({"n": n, "K": K, "b": b, "r": r, "skipped": "b*r > K"})
                    continue
                elapsed, stages, sig, keys, cid = measure(K, b, r, n, args.steps, 1)
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
                    "minhash_frac_of_alu_peak": round(
                        n_sh * ops_per_shingle(recipe.scaled(n_docs, shingle_n=n), K)
                        / (mh_ms * 1e-3) / 1e12 / PEAK_TOPS, 4),
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
