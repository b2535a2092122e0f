#!/usr/bin/env python3
"""Benchmark of the MinHash-LSH hot path on one MI355X.

A step is one pass of the whole path (sedd_minhash -> sedd_lsh_keys -> sedd_cluster) over the
medium workload: 1M synthetic web-text-shaped documents, 5-word shingles, K=128, 16 bands of 8
rows, with the text and offsets already resident in HBM.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--docs N] [--config 2]

The CPU oracle is timed on a bounded sample of the same corpus and reported beside it as
`cpu_baseline`; it is a reported baseline, not the target.
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

# Algorithmic work of the dominant kernel: per (shingle, hash function) one 61-bit modular
# multiply-add, truncation and minimum = 8 integer VALU lane-operations in the best sequence
# known here (six 32x32+64 multiply-adds, one 3-input add, one minimum).
OPS_PER_PAIR = 8
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one 32-bit integer lane-operation per lane per clock
PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--docs", type=int, default=0, help="override the document count")
    ap.add_argument("--config", type=int, default=2, help="workload number 1..5")
    ap.add_argument("--cpu-sample-docs", type=int, default=20000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    if args.docs:
        recipe = recipe.scaled(args.docs)
    flags = sedd.FLAG_BYTE_SHINGLES if recipe.byte_mode else 0

    t0 = time.time()
    data, off = corpus.generate(recipe)
    t_gen = time.time() - t0
    n_docs, n_bytes = recipe.n_docs, int(data.size)
    d_data = torch.from_numpy(data).cuda()
    d_off = torch.from_numpy(off).cuda()
    sig = torch.empty((n_docs, recipe.K), dtype=torch.uint32, device="cuda")
    keys = torch.empty((n_docs, recipe.b), dtype=torch.uint64, device="cuda")
    cid = torch.empty((n_docs,), dtype=torch.int64, device="cuda")

    def step():
        sedd.sedd_minhash(d_data, d_off, recipe.shingle_n, recipe.K, 0, flags, out=sig)
        sedd.sedd_lsh_keys(sig, recipe.b, recipe.r, out=keys)
        sedd.sedd_cluster(keys, out=cid)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    sedd.profile_enable(True)
    sedd.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sedd.profile_enable(False)
    stages = sedd.profile_read()

    ms_per_step = 1e3 * elapsed / args.steps
    docs_per_s = n_docs * args.steps / elapsed
    text_gbps = n_bytes * args.steps / elapsed / 1e9

    # shingle count of the corpus (outside the timed region)
    _, soff = sedd.debug_shingle_hashes(d_data, d_off, recipe.shingle_n, flags)
    n_shingles = int(soff.cpu().numpy()[-1])
    mh_ms, mh_spans = stages["minhash"]
    pairs_per_step = n_shingles * recipe.K
    launches_per_step = max(1, mh_spans // max(1, args.steps))
    avg_launch_ms = mh_ms / max(1, mh_spans)
    achieved = pairs_per_step * args.steps * OPS_PER_PAIR / (mh_ms * 1e-3) / 1e12 if mh_ms else 0.0
    roofline = {
        "kernel": "k_minhash", "bound": "alu", "achieved": round(achieved, 3),
        "peak": round(PEAK_TOPS, 3), "unit": "TOP/s (int32 VALU lane-ops)",
        "frac": round(achieved / PEAK_TOPS, 4), "traffic": None,
        "ops_per_hash_eval": OPS_PER_PAIR, "hash_evals_per_step": pairs_per_step,
        "launches_per_step": launches_per_step, "avg_launch_ms": round(avg_launch_ms, 4),
        "hash_evals_per_s": round(pairs_per_step * args.steps / (mh_ms * 1e-3), 1) if mh_ms else 0,
    }
    stage_ms = {k: round(v[0] / args.steps, 4) for k, v in stages.items()}

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_docs, n_docs)
        sub_off = off[: ns + 1]
        sub = data[: int(sub_off[-1])]
        t0 = time.perf_counter()
        o_sig = oracle.minhash(sub, sub_off, recipe.shingle_n, recipe.K, 0, flags)
        o_keys = oracle.lsh_keys(o_sig, recipe.b, recipe.r)
        oracle.cluster(o_keys)
        t_cpu = time.perf_counter() - t0
        cpu_baseline = {
            "value": round(ns / t_cpu, 2), "unit": "docs/s", "cores": 1, "kind": "oracle",
            "text_GB_per_s": round(int(sub_off[-1]) / t_cpu / 1e9, 5),
            "sample": f"first {ns} documents of the same corpus ({int(sub_off[-1])} bytes), "
                      f"minhash + band keys + clusters, single thread, {t_cpu:.1f} s",
        }
        # the sample doubles as a parity spot check of the timed configuration
        parity = bool(np.array_equal(sig[:ns].cpu().numpy(), o_sig)
                      and np.array_equal(keys[:ns].cpu().numpy(), o_keys))

    out = {
        "metric": "MinHash+LSH docs/sec on 1 MI355X (minhash + band keys + clustering)",
        "value": round(docs_per_s, 1), "unit": "docs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64 (61-bit modular) / u32",
        "data": "synthetic",
        "config": {"workload": recipe.name, "n_docs": n_docs, "text_bytes": n_bytes,
                   "shingles": n_shingles, "shingle_n": recipe.shingle_n,
                   "byte_shingles": bool(recipe.byte_mode), "K": recipe.K, "b": recipe.b,
                   "r": recipe.r, "corpus_seed": recipe.seed, "hash_seed": 0},
        "text_GB_per_s": round(text_gbps, 3),
        "stage_ms_per_step": stage_ms,
        "duplicates_found": int((cid.cpu().numpy() != np.arange(n_docs)).sum()),
        "corpus_generation_s": round(t_gen, 2),
        "scratch_bytes": sedd.sedd_scratch_bytes(),
        "exact_path_tiles": sedd.debug_stats()[sedd.STAT_SLOW_TILES],
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity_sample_ok": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
