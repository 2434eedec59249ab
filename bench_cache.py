#!/usr/bin/env python3
"""Bench of the vectorised feature cache (section 4.3 of the paper; a "next" row of the scope).

A step is one tns_cache_fetch of a batch of ids: lookup, row gather (hits from the cache, misses
from the backing store), score update, eviction and insertion.  Synthetic workload in the paper's
proportions: rows of 172 floats (its edge-feature width), a cache of 1 % of the ids, Zipf-
distributed ids (section 4.3 reports power-law node access).  Prints one JSON line.

    python bench_cache.py [--steps K] [--warmup W] [--batch B] [--store device|pinned]
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--num-ids", type=int, default=1 << 24)
    ap.add_argument("--dim", type=int, default=172)
    ap.add_argument("--ratio", type=float, default=0.01)
    ap.add_argument("--batch", type=int, default=1 << 20)
    ap.add_argument("--policy", default="lru", choices=["lru", "lfu", "fifo"])
    ap.add_argument("--zipf", type=float, default=1.05)
    ap.add_argument("--store", default="device", choices=["device", "pinned"])
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench_cache.py: one GPU only", file=sys.stderr)
        return 2
    import numpy as np
    import torch
    from paper_2311_17410_amd import cache_binding as KB
    from oracle import cache_oracle as CO

    dev = torch.device("cuda", 0)
    n, d, B = args.num_ids, args.dim, args.batch
    cap = max(int(n * args.ratio), 1)
    policy = {"lru": 0, "lfu": 1, "fifo": 2}[args.policy]
    rng = np.random.default_rng(0)
    total = args.steps + args.warmup
    batches = [(rng.zipf(args.zipf, B) % n).astype(np.int32) for _ in range(total)]
    g = torch.Generator(device="cpu").manual_seed(0)
    if args.store == "device":
        store = torch.randn((n, d), dtype=torch.float32, device=dev)
    else:
        store = torch.randn((n, d), dtype=torch.float32, generator=g).pin_memory()
    cache = KB.Cache(n, cap, d, policy, 0.2)
    d_batches = [torch.from_numpy(b).to(dev) for b in batches]
    out = torch.empty((B, d), dtype=torch.float32, device=dev)
    hit = torch.empty(B, dtype=torch.uint8, device=dev)
    for i in range(args.warmup):
        cache.fetch(d_batches[i], store, out, hit)
    s0 = cache.stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, total):
        cache.fetch(d_batches[i], store, out, hit)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    s1 = cache.stats()
    hits, misses = s1["hits"] - s0["hits"], s1["misses"] - s0["misses"]
    # the last batch's rows must be the true rows
    ok = bool(torch.equal(out, store.to(dev)[d_batches[-1].long()] if args.store == "pinned" else store[d_batches[-1].long()]))
    row_bytes = 4 * d
    alg = B * (4 + 2 * row_bytes + 1) + 2 * 4 * cap + (s1["replaced"] - s0["replaced"]) / args.steps * 2 * row_bytes
    # CPU oracle on a few of the same batches (small id space would change the hit rate: same sizes)
    ref = CO.VectorCache(n, cap, d, policy, 0.2)
    h_store = store.cpu().numpy() if args.store == "device" else store.numpy()
    t0 = time.perf_counter()
    k = 0
    while k < total and time.perf_counter() - t0 < 15:
        ref.fetch(batches[k], h_store)
        k += 1
    cpu_s = time.perf_counter() - t0
    print(json.dumps({
        "metric": "feature rows fetched per second through the vectorised cache at 1 MI355X",
        "value": B / (ms * 1e-3), "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "dtype": "f32 rows (copied), int32 ids and scores",
        "data": "synthetic",
        "config": {"workload": f"cache: {n} ids x {d} floats, capacity {cap} ({args.ratio:.0%}), batch {B}, "
                               f"Zipf({args.zipf}) ids, policy {args.policy}, lambda 0.2, store in {args.store} memory"},
        "hit_rate": hits / max(hits + misses, 1), "rows_match_store": ok,
        "roofline": {"bound": "hbm" if args.store == "device" else "pcie", "achieved": alg / (ms * 1e-3) / 1e9,
                     "peak": 8000.0 if args.store == "device" else None, "unit": "GB/s",
                     "frac": alg / (ms * 1e-3) / 1e9 / 8000.0 if args.store == "device" else None,
                     "algorithmic_bytes_per_step": alg},
        "cpu_baseline": {"value": k * B / cpu_s, "unit": "rows/s", "cores": 1, "kind": "oracle",
                         "sample": f"the first {k} batches of the same sequence, {cpu_s:.1f} s"},
    }), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
