#!/usr/bin/env python3
"""Bench of multi-hop sampling (section 4.2 of the paper: the nodes sampled in one layer are the
targets of the next; a "next" row of the scope).

A step is one tns_run_khop call: every hop is a full pass of the hot path (sampling with the padding
removal fused in) whose queries are the dense output of the hop before, chained on the device.
Workload: the C5 recipe (uniform node ids, |V| = n/16, sorted U[0,1) times) with one first-hop query
per event.  Prints one JSON line.

    python bench_khop.py [--log2n 24] [--fanouts 10,10] [--steps K] [--warmup W]
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
    ap.add_argument("--log2n", type=int, default=24)
    ap.add_argument("--fanouts", default="10,10")
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--batch", type=int, default=0,
                    help="first-hop queries: the last BATCH events of the stream (a training mini-batch, section 6: 600-4000 "
                         "edges) instead of every event")
    ap.add_argument("--layout", default="blocks", choices=["blocks", "prefix"],
                    help="blocks: store built on the device in the default layout; prefix: host-built store in the prefix layout")
    ap.add_argument("--dense-only", action="store_true", help="pass no padded outputs: every hop writes its dense result only")
    ap.add_argument("--graph", action="store_true", help="capture the call into a HIP graph once and time replays")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench_khop.py: one GPU only", file=sys.stderr)
        return 2
    import numpy as np
    import torch
    from paper_2311_17410_amd import binding as B
    from paper_2311_17410_amd import workloads as W

    B.lib()
    dev = torch.device("cuda", 0)
    fanouts = [int(x) for x in args.fanouts.split(",")]
    wl = W.c5(log2_n=args.log2n)
    st = wl.streams[0]
    Q = st.n
    d_src, d_dst, d_ts = (torch.from_numpy(a).to(dev) for a in (st.src, st.dst, st.ts))
    if args.layout == "prefix":
        plan = B.Plan(st.num_nodes, fanouts[0], block_threshold=wl.tau, flags=B.TNS_FLAG_PREFIX_LAYOUT)
        for lo, hi in st.batches():
            B.tns_add_edges(plan.handle, 0, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
        plan.commit()
    else:
        plan = B.Plan(st.num_nodes, fanouts[0], block_threshold=wl.tau, flags=B.TNS_FLAG_DEVICE_INGEST)
        for lo, hi in st.batches():
            plan.add_edges_device(d_src[lo:hi], d_dst[lo:hi], d_ts[lo:hi])
    del d_dst
    node_entry = 32 if args.layout == "prefix" else 16

    q_src, q_ts, h_src, h_ts = d_src, d_ts, st.src, st.ts
    if args.batch:
        Q = min(args.batch, Q)
        q_src, q_ts, h_src, h_ts = d_src[-Q:].contiguous(), d_ts[-Q:].contiguous(), st.src[-Q:], st.ts[-Q:]
    hops, ws = plan.run_khop(fanouts, q_src, None, q_ts)           # allocates the per-hop buffers once
    torch.cuda.synchronize()
    p = lambda t: 0 if t is None else t.data_ptr()
    ptrs = [{k: p(v) for k, v in h.items() if k not in ("cap", "fanout")} for h in hops]
    if args.dense_only:
        for d in ptrs:
            d["nbr"] = d["eid"] = d["ts"] = d["count"] = 0
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        B.tns_run_khop(plan.handle, fanouts, float("inf"), Q, p(q_src), 0, p(q_ts), 0, 0, ptrs, ws.data_ptr(), ws.numel(),
                       torch.cuda.current_stream().cuda_stream)

    if args.graph:
        eager, graph, side = step, torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            eager()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_gpu = ev0.elapsed_time(ev1) / args.steps

    # queries per hop and the byte model (the library's counting pass on each hop's queries)
    n_q = [Q]
    for h in hops[:-1]:
        n_q.append(int(h["rowptr"][n_q[-1]].item()))
    alg, targets, t_end = 0, q_src, q_ts
    counters = torch.zeros(4, dtype=torch.int64, device=dev)
    for h, f, q in zip(hops, fanouts, n_q):
        plan.set_sampler(f, B.TNS_POLICY_RECENT, 0, 0)
        counters.zero_()
        B.tns_traffic_model(plan.handle, q, p(targets), 0, p(t_end), 0, 0, counters.data_ptr(), stream)
        torch.cuda.synchronize()
        nn, nb, npr, ne = (int(x) for x in counters.cpu())
        alg += 8 * q + node_entry * nn + 16 * nb + 4 * npr + 12 * ne + (0 if args.dense_only else (12 * f + 4) * q) + 8 * (q + 1) + 12 * ne
        targets, t_end = h["cmp_nbr"], h["cmp_ts"]
    total_q = sum(n_q)

    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        from oracle import khop_oracle
        adj = oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
        k = min(Q, 1 << 22)
        t0 = time.perf_counter()
        ref = khop_oracle.khop([adj], h_src[:k], None, h_ts[:k], None, fanouts, policy=0, threads=16)
        done = sum(r["num_queries"] for r in ref)
        ok = all(bool(np.array_equal(h["cmp_eid"][:len(r["cmp_eid"])].cpu().numpy(), r["cmp_eid"])) for h, r in zip(hops, ref))
        cpu_s = time.perf_counter() - t0
        cpu = {"value": done / cpu_s, "unit": "elements/s", "cores": 16, "kind": "oracle",
               "sample": f"the first {k} first-hop queries and everything they expand to ({done} queries), {cpu_s:.1f} s "
                         "including the comparison with the GPU output", "matches_gpu_on_sample": ok}
        adj.close()

    print(json.dumps({
        "metric": "hot-path elements/sec over all hops at 1 MI355X", "value": total_q / (ms * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "dtype": "int32 ids / fp32 timestamps (copied and compared, no arithmetic)", "data": "synthetic",
        "config": {"workload": f"{wl.name} recipe, n=2^{args.log2n}: "
                               + (f"first-hop queries = the last {Q} events" if args.batch else "one first-hop query per event")
                               + f", fan-outs {fanouts}, recent policy, unbounded window, hop h+1 = dense output of hop h",
                   "queries_per_hop": n_q, "hip_graph_replay": bool(args.graph), "layout": args.layout, "dense_only": bool(args.dense_only)},
        "roofline": {"bound": "hbm", "achieved": alg / (ms_gpu * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                     "frac": alg / (ms_gpu * 1e-3) / 1e9 / 8000.0, "traffic": None, "algorithmic_bytes_per_step": alg,
                     "ms_gpu_per_step": ms_gpu},
        "cpu_baseline": cpu,
    }), flush=True)
    plan.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
