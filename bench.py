#!/usr/bin/env python3
"""Bench of the sampling hot path on one MI355X.

A step is one pass of the whole path over one query batch: sampling kernel (node lookup,
block walk, in-block search, selection, padded write) followed by padding removal, on
inputs already resident in HBM.  Prints ONE JSON line (see the design doc for the byte model
behind `roofline`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--policy recent]
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def measured_traffic(workload: str, policy: str):
    """HBM bytes per launch of the sampling kernel from the committed rocprofv3 counter runs
    (profiles/traffic.json, written by hand from the --pmc summaries); None if not measured."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as fh:
            return json.load(fh).get(f"{workload}:{policy}")
    except OSError:
        return None


def cpu_baseline(wl, policy: int, seed: int, target_seconds: float, d_out, torch):
    """The CPU oracle as it stands, on a strided sample of the same query batch, all host cores
    the box grants.  Also compares the sampled rows with the GPU result."""
    import numpy as np
    import oracle
    st = wl.streams[0]
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or min(os.cpu_count() or 1, 16)
    log(f"cpu_baseline: building the oracle's per-node lists over {st.n} edges")
    t0 = time.time()
    adj = oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    build_s = time.time() - t0
    chunk = 1 << 20
    stride = 1
    done, spent, used, ok = 0, 0.0, threads, True
    pos = 0
    f = wl.fanout
    while spent < target_seconds and pos < st.n:
        sel = np.arange(pos, min(pos + chunk * stride, st.n), stride, dtype=np.int64)
        tg, te = st.src[sel], st.ts[sel]
        t0 = time.time()
        ref = adj.sample(tg, None, te, f, policy=policy, seed=seed, q_ids=sel, threads=threads)
        spent += time.time() - t0
        used = adj.threads_used
        if done == 0:          # parity of the sample against what the GPU wrote for the same queries
            idx = torch.from_numpy(sel).to(d_out["count"].device)
            g_eid = d_out["eid"].view(-1, f).index_select(0, idx).cpu().numpy()
            g_cnt = d_out["count"].index_select(0, idx).cpu().numpy()
            ok = bool(np.array_equal(g_eid, ref.eid) and np.array_equal(g_cnt, ref.count))
        done += len(sel)
        pos += chunk * stride
    # one thread, on a prefix sized for a few seconds
    n1 = min(st.n, 1 << 22)
    t0 = time.time()
    adj.sample(st.src[:n1], None, st.ts[:n1], f, policy=policy, seed=seed, q_ids=np.arange(n1, dtype=np.int64), threads=1)
    one_s = time.time() - t0
    adj.close()
    return {"value": done / spent, "unit": "elements/s", "cores": used, "kind": "oracle",
            "sample": f"the first {done} queries of the batch, in order, {spent:.1f} s "
                      f"(per-node list build {build_s:.1f} s not included)",
            "matches_gpu_on_sample": ok,
            "single_thread": {"value": n1 / one_s, "unit": "elements/s", "sample": f"the first {n1} queries, {one_s:.1f} s"}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5", help="C1..C5 (C5 = the headline: n = 2^28)")
    ap.add_argument("--log2n", type=int, default=None, help="override the stream length of C3/C5 (experiments)")
    ap.add_argument("--policy", default="recent", choices=["recent", "uniform"])
    ap.add_argument("--windowed", action="store_true", help="t_start = t_end - 0.25 span instead of -inf")
    ap.add_argument("--no-remap", action="store_true", help="disable the XCD-aware tile mapping")
    ap.add_argument("--placement", default="hbm", choices=["hbm", "hybrid", "host"],
                    help="hbm: the whole store in device memory (default); hybrid: edge data in page-locked host "
                         "memory, metadata on the device (the paper's placement); host: everything in host memory")
    ap.add_argument("--ingest", default="host", choices=["host", "device"],
                    help="host: tns_add_edges + tns_commit (default); device: the stream is copied to the GPU once and "
                         "ingested batch by batch with tns_add_edges_device")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="accepted for the recorded profile commands: the plain 1 GiB device copy of known traffic "
                         "now always runs (it also gives the box's streaming ceiling)")
    ap.add_argument("--layout", default="prefix", choices=["prefix", "blocks"],
                    help="prefix: a node's first 38 edge slots in its own line + up to three extension lines (default for "
                         "device-resident, host-built stores); blocks: every block placed on its own, records in the node line")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU oracle time budget (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2311_17410_amd import binding as B
    from paper_2311_17410_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    B.lib()
    dev = torch.device("cuda", 0)
    policy = B.TNS_POLICY_RECENT if args.policy == "recent" else B.TNS_POLICY_UNIFORM

    kw = {}
    if args.log2n is not None and args.workload.upper() in ("C3", "C5"):
        kw["log2_n"] = args.log2n
    log(f"generating {args.workload} {kw or ''}")
    wl = W.by_name(args.workload, **kw)
    Q, f = wl.total_edges, wl.fanout

    if args.placement != "hbm" or args.ingest == "device":
        args.layout = "blocks"          # the prefix layout is for host-built, device-resident stores
    node_entry_bytes = 32 if args.layout == "prefix" else 16
    log(f"ingesting {Q} edges into {wl.num_instances} instance(s), tau={wl.tau}, layout={args.layout}")
    t0 = time.time()
    plan = B.Plan(wl.num_nodes, f, policy=policy, block_threshold=wl.tau, num_instances=wl.num_instances,
                  seed=wl.seed,
                  flags=(B.TNS_FLAG_NO_XCD_REMAP if args.no_remap else 0)
                  | {"hbm": 0, "hybrid": B.TNS_FLAG_EDGES_ON_HOST, "host": B.TNS_FLAG_ALL_ON_HOST}[args.placement]
                  | (B.TNS_FLAG_DEVICE_INGEST if args.ingest == "device" else 0)
                  | (B.TNS_FLAG_PREFIX_LAYOUT if args.layout == "prefix" else 0))
    last = time.time()
    for i, st in enumerate(wl.streams):
        if args.ingest == "device":
            d_src, d_dst, d_ts = (torch.from_numpy(a).to(dev) for a in (st.src, st.dst, st.ts))
            torch.cuda.synchronize()
            t0 = time.time() if i == 0 else t0      # the one-off copy of the stream is not ingestion
        for lo, hi in st.batches():
            if args.ingest == "device":
                plan.add_edges_device(d_src[lo:hi], d_dst[lo:hi], d_ts[lo:hi], instance=i)
            else:
                B.tns_add_edges(plan.handle, i, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
            if time.time() - last > 20:
                log(f"  instance {i}: {hi}/{st.n} edges")
                last = time.time()
        if args.ingest == "device":
            del d_src, d_dst, d_ts
    ingest_s = time.time() - t0
    t0 = time.time()
    plan.commit()
    commit_s = time.time() - t0
    stats = plan.stats()
    log(f"store: {stats['num_blocks']} blocks, avg list {stats['avg_list_len']:.2f}, max {stats['max_list_len']}, "
        f"edge data {stats['edge_data_bytes'] / 2**30:.2f} GiB, metadata {stats['metadata_bytes'] / 2**30:.2f} GiB "
        f"(ingest {ingest_s:.1f} s, commit {commit_s:.1f} s)")

    targets, t_start, t_end, rowptr = wl.queries(window_frac=0.25 if args.windowed else None)
    d_targets = torch.from_numpy(targets).to(dev)
    d_te = torch.from_numpy(t_end).to(dev)
    d_tb = None if t_start is None else torch.from_numpy(t_start).to(dev)
    d_rp = torch.from_numpy(rowptr).to(dev) if wl.num_instances > 1 else None
    out = plan.alloc_outputs(Q, compact=True)
    p = lambda t: 0 if t is None else t.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    ws_bytes = out["workspace"].numel()

    def sample():
        B.tns_run(plan.handle, Q, p(d_targets), p(d_tb), p(d_te), p(d_rp), 0, p(out["nbr"]), p(out["eid"]),
                  p(out["ts"]), p(out["count"]), hip_stream=stream)

    def fused():
        B.tns_run(plan.handle, Q, p(d_targets), p(d_tb), p(d_te), p(d_rp), 0, p(out["nbr"]), p(out["eid"]),
                  p(out["ts"]), p(out["count"]), p(out["rowptr"]), p(out["cmp_nbr"]), p(out["cmp_eid"]),
                  p(out["cmp_ts"]), p(out["workspace"]), ws_bytes, stream)

    def compact():
        B.tns_compact(plan.handle, Q, p(out["nbr"]), p(out["eid"]), p(out["ts"]), p(out["count"]), p(out["rowptr"]),
                      p(out["cmp_nbr"]), p(out["cmp_eid"]), p(out["cmp_ts"]), p(out["workspace"]), ws_bytes, stream)

    # byte model: what the walk reads, counted by the library's own counting pass
    counters = torch.zeros(4, dtype=torch.int64, device=dev)
    B.tns_traffic_model(plan.handle, Q, p(d_targets), p(d_tb), p(d_te), p(d_rp), 0, counters.data_ptr(), stream)
    torch.cuda.synchronize()
    n_nodes, n_blocks, n_probes, n_edges = (int(x) for x in counters.cpu())
    q_in = 8 + (4 if d_tb is not None else 0) + (0 if d_rp is None else 0)
    bytes_sample = {"queries": q_in * Q, "node_entries": node_entry_bytes * n_nodes, "block_records": 16 * n_blocks,
                    "timestamp_probes": 4 * n_probes, "edge_gather": 12 * n_edges, "padded_write": (12 * f + 4) * Q}
    alg_sample = sum(bytes_sample.values())
    alg_compact = (4 + 4 + 12 * f) * Q + 8 * (Q + 1) + 12 * n_edges     # counts twice, padded once, rowptr, dense

    # The step: ONE tns_run with the dense outputs requested = sampling kernel with the padding
    # removal fused in (plus a tiny kernel that clears the chained scan's tile states).
    dense_write = 12 * n_edges + 8 * (Q + 1)
    alg_step = alg_sample + dense_write
    log(f"warm-up {args.warmup}, timing {args.steps} steps")
    for _ in range(args.warmup):
        fused()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record()
        fused()
        ev[k][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ms_kernel = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    assert not plan.status(out["workspace"]), "chained scan timed out"

    # for comparison, the same work as two steps: padded sampling, then stand-alone padding removal
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for k in range(args.steps):
        ev2[k][0].record()
        sample()
        ev2[k][1].record()
        compact()
        ev2[k][2].record()
    torch.cuda.synchronize()
    ms_sample = sum(e[0].elapsed_time(e[1]) for e in ev2) / args.steps
    ms_compact = sum(e[1].elapsed_time(e[2]) for e in ev2) / args.steps
    # the box's own streaming ceiling: a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB); the same
    # kernel gives rocprofv3 counter runs of this command a launch of known traffic (--calibrate-copy)
    a = torch.arange(1 << 28, dtype=torch.int32, device=dev)
    b = torch.empty_like(a)
    b.copy_(a)
    evc = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    evc[0].record()
    for _ in range(5):
        b.copy_(a)
    evc[1].record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * a.numel() * 4 / (evc[0].elapsed_time(evc[1]) * 1e-3) / 1e9
    del a, b
    total_k = int(out["rowptr"][-1].item())
    assert total_k == n_edges, (total_k, n_edges)

    # second row of the report: the same step under the other selection policy (a few steps, no oracle leg)
    other = None
    if args.placement == "hbm":
        other_name = "uniform" if args.policy == "recent" else "recent"
        plan.set_sampler(f, B.TNS_POLICY_UNIFORM if other_name == "uniform" else B.TNS_POLICY_RECENT, 0, wl.seed)
        counters.zero_()
        B.tns_traffic_model(plan.handle, Q, p(d_targets), p(d_tb), p(d_te), p(d_rp), 0, counters.data_ptr(), stream)
        for _ in range(2):
            fused()
        evo = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        evo[0].record()
        for _ in range(5):
            fused()
        evo[1].record()
        torch.cuda.synchronize()
        o_ms = evo[0].elapsed_time(evo[1]) / 5
        on, ob, op_, oe = (int(x) for x in counters.cpu())
        o_alg = q_in * Q + node_entry_bytes * on + 16 * ob + 4 * op_ + 12 * oe + (12 * f + 4) * Q + 12 * oe + 8 * (Q + 1)
        other = {"policy": other_name, "ms_per_step": o_ms, "value": Q / (o_ms * 1e-3), "unit": "elements/s",
                 "algorithmic_bytes_per_launch": o_alg, "frac": o_alg / (o_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "steps": 5}
        plan.set_sampler(f, policy, 0, wl.seed)
        fused()                      # the outputs hold the headline policy's result again (compared with the oracle below)
        torch.cuda.synchronize()

    achieved = alg_step / (ms_kernel * 1e-3) / 1e9
    per_step = sorted(e[0].elapsed_time(e[1]) for e in ev)
    traffic = measured_traffic(wl.name, args.policy) if args.placement == "hbm" else None
    moved = None
    if traffic:
        moved_gbs = traffic / (ms_kernel * 1e-3) / 1e9
        moved = {"GBs": moved_gbs, "frac_of_peak": moved_gbs / HBM_PEAK_GBS, "frac_of_copy_ceiling": moved_gbs / copy_gbs,
                 "waste_factor": traffic / alg_step}
    bytes_step = dict(bytes_sample, dense_write=dense_write)
    result = {
        "metric": "hot-path elements/sec at 1 MI355X + % of HBM/MFMA roofline",
        "value": Q / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / fp32 timestamps (copied and compared, no arithmetic)",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.description}; query i = (src[i], -inf, ts[i]); f={f}, tau={wl.tau}, "
                               f"policy={args.policy}, window={'0.25 span' if args.windowed else 'unbounded'}",
                   "queries": Q, "instances": wl.num_instances, "nodes_per_instance": wl.num_nodes,
                   "placement": args.placement, "ingest": args.ingest, "layout": args.layout},
        "roofline": {"bound": "hbm", "kernel": "tns_sample_kernel (padding removal fused)" if args.placement == "hbm" else "tns_sample_kernel + tns_compact kernels", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "moved": moved, "copy_ceiling_GBs": copy_gbs,
                     "algorithmic_bytes_per_launch": alg_step, "bytes_breakdown": bytes_step,
                     "ms_per_launch": ms_kernel, "ms_per_launch_median": per_step[len(per_step) // 2],
                     "ms_per_launch_min": per_step[0]},
        "two_kernel_path": {"sample_ms": ms_sample, "sample_GBs": alg_sample / (ms_sample * 1e-3) / 1e9,
                            "compact_ms": ms_compact, "compact_GBs": alg_compact / (ms_compact * 1e-3) / 1e9,
                            "xcd_remap": not args.no_remap},
        "other_policy": other,
        "sampled_edges_per_s": total_k / (ms_per_step * 1e-3),
        "per_query": {"block_records": n_blocks / Q, "timestamp_probes": n_probes / Q, "edges": n_edges / Q},
        "store": stats, "ingest_s": ingest_s, "commit_s": commit_s,
    }
    if args.cpu_seconds > 0 and wl.num_instances == 1:
        result["cpu_baseline"] = cpu_baseline(wl, policy, wl.seed, args.cpu_seconds, out, torch)
    else:
        result["cpu_baseline"] = None
    plan.close()
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
