#!/usr/bin/env python3
"""Bench of the sampling hot path on one MI355X.

A step is one pass of the whole path over one query batch: node lookup, block walk, in-block
search, selection, padded write and padding removal (one fused kernel), on inputs already
resident in HBM.  Prints ONE JSON line; the design doc explains the byte model behind `roofline`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--policy recent] [--layout blocks]

The line also carries: the same step under the other selection policy and in the other store
layout, the smaller configurations (C1-C4), the box's own streaming rates (read, write, copy
kernels of the library), and the CPU oracle timed on the host cores.
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


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


class Runner:
    """One committed plan of a workload with its query and output buffers on the device."""

    def __init__(self, B, torch, wl, layout: str, policy: int, flags: int = 0, ingest: str = "host", windowed: bool = False):
        self.B, self.torch, self.wl, self.layout = B, torch, wl, layout
        dev = torch.device("cuda", 0)
        self.Q, self.f = wl.total_edges, wl.fanout
        t0 = time.time()
        self.plan = B.Plan(wl.num_nodes, self.f, policy=policy, block_threshold=wl.tau, num_instances=wl.num_instances,
                           seed=wl.seed, flags=flags | (B.TNS_FLAG_PREFIX_LAYOUT if layout == "prefix" else 0)
                           | (B.TNS_FLAG_DEVICE_INGEST if ingest == "device" else 0))
        last = time.time()
        for i, st in enumerate(wl.streams):
            if ingest == "device":
                d_src, d_dst, d_ts = (torch.from_numpy(a).to(dev) for a in (st.src, st.dst, st.ts))
                torch.cuda.synchronize()
                t0 = time.time() if i == 0 else t0      # the one-off copy of the stream is not ingestion
            for lo, hi in st.batches():
                if ingest == "device":
                    self.plan.add_edges_device(d_src[lo:hi], d_dst[lo:hi], d_ts[lo:hi], instance=i)
                else:
                    B.tns_add_edges(self.plan.handle, i, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
                if time.time() - last > 20:
                    log(f"  {wl.name} [{layout}] instance {i}: {hi}/{st.n} edges")
                    last = time.time()
        self.ingest_s = time.time() - t0
        t0 = time.time()
        self.plan.commit()
        self.commit_s = time.time() - t0
        self.stats = self.plan.stats()
        targets, t_start, t_end, rowptr = wl.queries(window_frac=0.25 if windowed else None)
        self.d_targets = torch.from_numpy(targets).to(dev)
        self.d_te = torch.from_numpy(t_end).to(dev)
        self.d_tb = None if t_start is None else torch.from_numpy(t_start).to(dev)
        self.d_rp = torch.from_numpy(rowptr).to(dev) if wl.num_instances > 1 else None
        self.out = self.plan.alloc_outputs(self.Q, compact=True)
        self.stream = torch.cuda.current_stream().cuda_stream
        self.node_entry_bytes = 32 if layout == "prefix" else 16
        self.q_in = 8 + (4 if self.d_tb is not None else 0)

    def _p(self, t):
        return 0 if t is None else t.data_ptr()

    def fused(self):
        o, p = self.out, self._p
        self.B.tns_run(self.plan.handle, self.Q, p(self.d_targets), p(self.d_tb), p(self.d_te), p(self.d_rp), 0, p(o["nbr"]),
                       p(o["eid"]), p(o["ts"]), p(o["count"]), p(o["rowptr"]), p(o["cmp_nbr"]), p(o["cmp_eid"]), p(o["cmp_ts"]),
                       p(o["workspace"]), o["workspace"].numel(), self.stream)

    def dense_only(self):
        """The step without the padded rows: tns_run with the four padded outputs NULL writes the dense result only."""
        o, p = self.out, self._p
        self.B.tns_run(self.plan.handle, self.Q, p(self.d_targets), p(self.d_tb), p(self.d_te), p(self.d_rp), 0, 0, 0, 0, 0,
                       p(o["rowptr"]), p(o["cmp_nbr"]), p(o["cmp_eid"]), p(o["cmp_ts"]), p(o["workspace"]), o["workspace"].numel(),
                       self.stream)

    def sample(self):
        o, p = self.out, self._p
        self.B.tns_run(self.plan.handle, self.Q, p(self.d_targets), p(self.d_tb), p(self.d_te), p(self.d_rp), 0, p(o["nbr"]),
                       p(o["eid"]), p(o["ts"]), p(o["count"]), hip_stream=self.stream)

    def compact(self):
        o, p = self.out, self._p
        self.B.tns_compact(self.plan.handle, self.Q, p(o["nbr"]), p(o["eid"]), p(o["ts"]), p(o["count"]), p(o["rowptr"]),
                           p(o["cmp_nbr"]), p(o["cmp_eid"]), p(o["cmp_ts"]), p(o["workspace"]), o["workspace"].numel(), self.stream)

    def byte_model(self):
        """Algorithmic bytes of one step, from the library's counting pass (same walk, counters instead of
        outputs): what the method has to read and write, not what the memory system moved."""
        torch = self.torch
        counters = torch.zeros(4, dtype=torch.int64, device=self.d_targets.device)
        p = self._p
        self.B.tns_traffic_model(self.plan.handle, self.Q, p(self.d_targets), p(self.d_tb), p(self.d_te), p(self.d_rp), 0,
                                 counters.data_ptr(), self.stream)
        torch.cuda.synchronize()
        n_nodes, n_blocks, n_probes, n_edges = (int(x) for x in counters.cpu())
        Q, f = self.Q, self.f
        parts = {"queries": self.q_in * Q, "node_entries": self.node_entry_bytes * n_nodes, "block_records": 16 * n_blocks,
                 "timestamp_probes": 4 * n_probes, "edge_gather": 12 * n_edges, "padded_write": (12 * f + 4) * Q,
                 "dense_write": 12 * n_edges + 8 * (Q + 1)}
        return {"parts": parts, "step": sum(parts.values()), "sample": sum(parts.values()) - parts["dense_write"],
                "compact": (4 + 4 + 12 * f) * Q + 8 * (Q + 1) + 12 * n_edges,
                "per_query": {"block_records": n_blocks / max(Q, 1), "timestamp_probes": n_probes / max(Q, 1), "edges": n_edges / max(Q, 1)},
                "n_edges": n_edges}

    def time_steps(self, fn, steps: int, warmup: int):
        """(wall ms per step, [event ms per launch]) of `steps` calls of fn on the torch stream."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            ev[k][0].record()
            fn()
            ev[k][1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, [e[0].elapsed_time(e[1]) for e in ev]

    def close(self):
        self.plan.close()
        self.out = None


def streaming_rates(B, torch, read_per_write=None):
    """The box's own ceilings from the library's streaming kernels over 1 GiB (16-byte accesses, non-temporal hint),
    GB/s of bytes moved: read only, write only, a copy whose stores wait for all of a thread's loads (`copy`), the same
    with every store issued as soon as its own load has arrived (`copy_interleaved`, the launch the counter runs
    calibrate on), and a mix with the read:write byte ratio of the kernel under study (`mix`)."""
    dev = torch.device("cuda", 0)
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    a.fill_(1)
    s = torch.cuda.current_stream().cuda_stream

    def rate(fn, traffic):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return 5 * traffic / (e0.elapsed_time(e1) * 1e-3) / 1e9

    rates = {"read": rate(lambda: B.tns_hbm_probe(1, True, b.data_ptr(), a.data_ptr(), n, s), n),
             "write": rate(lambda: B.tns_hbm_probe(2, True, b.data_ptr(), a.data_ptr(), n, s), n),
             "copy": rate(lambda: B.tns_hbm_probe_mix(True, b.data_ptr(), n, a.data_ptr(), n, s), 2 * n),
             "copy_interleaved": rate(lambda: B.tns_hbm_probe(0, True, b.data_ptr(), a.data_ptr(), n, s), 2 * n)}
    if read_per_write:
        rb = n if read_per_write >= 1 else int(n * read_per_write) // 16 * 16
        wb = n if read_per_write <= 1 else int(n / read_per_write) // 16 * 16
        rates["mix"] = rate(lambda: B.tns_hbm_probe_mix(True, b.data_ptr(), wb, a.data_ptr(), rb, s), rb + wb)
        rates["mix_read_per_write"] = read_per_write
    del a, b
    return rates


def cpu_baseline(wl, policy: int, seed: int, target_seconds: float, out, torch):
    """The CPU oracle as it stands (OpenMP over queries) on all host cores the box grants, on a prefix of the
    same query batch sized by time; every output array of the sample is compared with what the GPU wrote."""
    import numpy as np
    import oracle
    st = wl.streams[0]
    nproc = os.cpu_count() or 1
    try:
        nproc = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        pass
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or nproc
    log(f"cpu_baseline: building the oracle's per-node lists over {st.n} edges ({threads} threads of {nproc} cores)")
    t0 = time.time()
    adj = oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    build_s = time.time() - t0
    chunk = 1 << 22
    done, spent, used, ok, compared = 0, 0.0, threads, True, 0
    f = wl.fanout
    while spent < target_seconds and done < st.n:
        lo, hi = done, min(done + chunk, st.n)
        sel = np.arange(lo, hi, dtype=np.int64)
        t0 = time.time()
        ref = adj.sample(st.src[lo:hi], None, st.ts[lo:hi], f, policy=policy, seed=seed, q_ids=sel, threads=threads)
        spent += time.time() - t0
        used = adj.threads_used
        if lo < 4 * chunk:   # parity against what the GPU wrote for the same queries (first 2^24): all four arrays
            g = {k: out[k].view(-1, f)[lo:hi].cpu().numpy() for k in ("nbr", "eid", "ts")}
            g_cnt = out["count"][lo:hi].cpu().numpy()
            ok = ok and bool(np.array_equal(g["eid"], ref.eid) and np.array_equal(g["nbr"], ref.nbr) and np.array_equal(g_cnt, ref.count)
                             and np.array_equal(g["ts"].view(np.int32), ref.ts.view(np.int32)))
            compared = hi
        done = hi
    n1 = min(st.n, 1 << 22)      # one thread, on a prefix sized for a few seconds
    t0 = time.time()
    adj.sample(st.src[:n1], None, st.ts[:n1], f, policy=policy, seed=seed, q_ids=np.arange(n1, dtype=np.int64), threads=1)
    one_s = time.time() - t0
    adj.close()
    return {"value": done / spent, "unit": "elements/s", "cores": used, "kind": "oracle", "nproc": nproc, "cpu_model": cpu_model(),
            "sample": f"the first {done} queries of the batch, in order, {spent:.1f} s "
                      f"(per-node list build {build_s:.1f} s not included)",
            "matches_gpu_on_sample": ok, "compared_queries": compared,
            "single_thread": {"value": n1 / one_s, "unit": "elements/s", "sample": f"the first {n1} queries, {one_s:.1f} s"}}


def measured_traffic(key: str):
    """HBM bytes per launch from the committed counter runs (profiles/traffic.json, written by
    `python -m paper_2311_17410_amd.traffic`) and whether the kernels have changed since."""
    from paper_2311_17410_amd import traffic as T
    return T.lookup(os.path.join(ROOT, "profiles", "traffic.json"), key)


def side_config(B, torch, W, name: str, layout: str, steps: int):
    """One of the smaller configurations: step time, rate, algorithmic fraction; the launch-bound ones (C1, C2)
    also as 100 launches back to back."""
    wl = W.by_name(name)
    r = Runner(B, torch, wl, layout, B.TNS_POLICY_RECENT)
    bm = r.byte_model()
    wall, ev = r.time_steps(r.fused, steps, 3)
    ms = sum(ev) / len(ev)
    assert not r.plan.status(r.out["workspace"])
    row = {"queries": r.Q, "instances": wl.num_instances, "ms_per_step": ms, "value": r.Q / (ms * 1e-3), "unit": "elements/s",
           "algorithmic_bytes_per_launch": bm["step"], "frac": bm["step"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "per_query": bm["per_query"], "store": {k: r.stats[k] for k in ("avg_list_len", "max_list_len", "edge_data_bytes", "metadata_bytes")}}
    if name in ("C1", "C2"):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(100):
            r.fused()
        e1.record()
        torch.cuda.synchronize()
        row["ms_per_step_100_back_to_back"] = e0.elapsed_time(e1) / 100
        row["note"] = "launch-bound: two launches per step (scan state clear + fused kernel)"
    r.close()
    return row


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
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
    ap.add_argument("--layout", default="blocks", choices=["blocks", "prefix"],
                    help="blocks: every block placed on its own, records in the node line (default); prefix: a node's "
                         "first 38 edge slots in its own line + up to three extension lines (host-built, device-resident stores)")
    ap.add_argument("--no-side", action="store_true", help="skip the other layout and the smaller configurations (profile runs)")
    ap.add_argument("--profile-run", action="store_true",
                    help="the command the committed rocprofv3 summaries were taken with: 3 steps, 1 warm-up, both layouts and "
                         "policies, no CPU oracle, no smaller configurations")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU oracle time budget (0 = skip)")
    args = ap.parse_args()
    if args.profile_run:
        args.steps, args.warmup, args.cpu_seconds = 3, 1, 0.0
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2311_17410_amd import binding as B
    from paper_2311_17410_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    B.lib()
    policy = B.TNS_POLICY_RECENT if args.policy == "recent" else B.TNS_POLICY_UNIFORM
    if args.placement != "hbm" or args.ingest == "device":
        args.layout = "blocks"          # the prefix layout is for host-built, device-resident stores
    plain = args.placement == "hbm" and args.ingest == "host" and not args.windowed

    kw = {}
    if args.log2n is not None and args.workload.upper() in ("C3", "C5"):
        kw["log2_n"] = args.log2n
    log(f"generating {args.workload} {kw or ''}")
    wl = W.by_name(args.workload, **kw)
    flags = (B.TNS_FLAG_NO_XCD_REMAP if args.no_remap else 0) | \
        {"hbm": 0, "hybrid": B.TNS_FLAG_EDGES_ON_HOST, "host": B.TNS_FLAG_ALL_ON_HOST}[args.placement]

    def measure_layout(layout: str, headline: bool):
        """The step in one layout: headline policy (timed as the contract asks), the other policy, and the
        two-kernel path; returns the runner (outputs hold the headline policy's result) and the figures."""
        log(f"ingesting {wl.total_edges} edges into {wl.num_instances} instance(s), tau={wl.tau}, layout={layout}")
        r = Runner(B, torch, wl, layout, policy, flags, args.ingest, args.windowed)
        st = r.stats
        log(f"store [{layout}]: {st['num_blocks']} blocks, avg list {st['avg_list_len']:.2f}, max {st['max_list_len']}, edge data "
            f"{st['edge_data_bytes'] / 2**30:.2f} GiB, metadata {st['metadata_bytes'] / 2**30:.2f} GiB (ingest {r.ingest_s:.1f} s, "
            f"commit {r.commit_s:.1f} s)")
        bm = r.byte_model()
        steps, warm = (args.steps, args.warmup) if headline else (5, 2)
        log(f"[{layout}] warm-up {warm}, timing {steps} steps")
        wall_ms, ev = r.time_steps(r.fused, steps, warm)
        assert not r.plan.status(r.out["workspace"]), "chained scan timed out"
        total_k = int(r.out["rowptr"][-1].item())
        assert total_k == bm["n_edges"], (total_k, bm["n_edges"])
        ms = sum(ev) / len(ev)
        kname = ("tns_sample_prefix_kernel" if layout == "prefix" else "tns_sample_kernel") + " (padding removal fused)"
        if args.placement != "hbm":
            kname = "tns_sample_kernel + tns_compact kernels"
        key = f"{wl.name}:{args.policy}:{layout}"
        tr = measured_traffic(key) if plain else None
        fig = {"layout": layout, "wall_ms_per_step": wall_ms, "ms_per_launch": ms, "ms_per_launch_median": sorted(ev)[len(ev) // 2],
               "ms_per_launch_min": min(ev), "kernel": kname, "byte_model": bm, "traffic": tr, "total_k": total_k,
               "store": st, "ingest_s": r.ingest_s, "commit_s": r.commit_s}
        # the same work as two steps: padded sampling, then stand-alone padding removal
        _, ev_s = r.time_steps(r.sample, 3, 1)
        _, ev_c = r.time_steps(r.compact, 3, 1)
        fig["two_kernel_path"] = {"sample_ms": sum(ev_s) / 3, "sample_GBs": bm["sample"] / (sum(ev_s) / 3 * 1e-3) / 1e9,
                                  "compact_ms": sum(ev_c) / 3, "compact_GBs": bm["compact"] / (sum(ev_c) / 3 * 1e-3) / 1e9,
                                  "xcd_remap": not args.no_remap}
        # the step for callers that only want the dense result: the padded rows are never written
        fig["dense_only"] = None
        if args.placement == "hbm" and not args.profile_run:      # (same kernel name: would blur the per-kernel counters)
            _, ev_d = r.time_steps(r.dense_only, 5, 2)
            assert not r.plan.status(r.out["workspace"])
            d_ms = sum(ev_d) / len(ev_d)
            d_alg = bm["step"] - bm["parts"]["padded_write"]
            fig["dense_only"] = {"ms_per_step": d_ms, "value": r.Q / (d_ms * 1e-3), "unit": "elements/s", "algorithmic_bytes_per_launch": d_alg,
                                 "frac": d_alg / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "steps": 5,
                                 "note": "tns_run with the padded outputs NULL: same walk, same dense rows and rowptr, no padded write"}
        # the same step under the other selection policy
        fig["other_policy"] = None
        if args.placement == "hbm":
            other_name = "uniform" if args.policy == "recent" else "recent"
            r.plan.set_sampler(r.f, B.TNS_POLICY_UNIFORM if other_name == "uniform" else B.TNS_POLICY_RECENT, 0, wl.seed)
            obm = r.byte_model()
            _, oev = r.time_steps(r.fused, 5, 2)
            o_ms = sum(oev) / len(oev)
            otr = measured_traffic(f"{wl.name}:{other_name}:{layout}") if plain else None
            fig["other_policy"] = {"policy": other_name, "ms_per_step": o_ms, "value": r.Q / (o_ms * 1e-3), "unit": "elements/s",
                                   "algorithmic_bytes_per_launch": obm["step"], "frac": obm["step"] / (o_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "traffic": otr, "steps": 5}
            r.plan.set_sampler(r.f, policy, 0, wl.seed)
        r.fused()                    # the outputs hold the headline policy's result (compared with the oracle by the caller)
        torch.cuda.synchronize()
        return r, fig

    r, head = measure_layout(args.layout, True)
    bm = head["byte_model"]
    tr0 = head["traffic"]
    if tr0 and not tr0["stale"]:
        ratio = tr0["fetch_bytes"] / tr0["write_bytes"]        # what the kernel moved
    else:
        written = bm["parts"]["padded_write"] + bm["parts"]["dense_write"]
        ratio = (bm["step"] - written) / written               # what the method needs
    rates = streaming_rates(B, torch, ratio)
    ms_kernel = head["ms_per_launch"]
    achieved = bm["step"] / (ms_kernel * 1e-3) / 1e9

    def moved_of(tr, alg, ms):
        if not tr or tr.get("bytes") is None:
            return None
        gbs = tr["bytes"] / (ms * 1e-3) / 1e9
        return {"GBs": gbs, "frac_of_peak": gbs / HBM_PEAK_GBS, "frac_of_copy_kernel": gbs / rates["copy"],
                "frac_of_mix_kernel": gbs / rates["mix"] if "mix" in rates else None, "waste_factor": tr["bytes"] / alg}

    tr = head["traffic"]
    roofline = {"bound": "hbm", "kernel": head["kernel"], "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None if not tr or tr["stale"] else tr["bytes"],
                "traffic_stale": bool(tr and tr["stale"]), "traffic_source": None if not tr else tr["source"],
                "moved": None if not tr or tr["stale"] else moved_of(tr, bm["step"], ms_kernel),
                "streaming_GBs": rates, "algorithmic_bytes_per_launch": bm["step"], "bytes_breakdown": bm["parts"],
                "ms_per_launch": ms_kernel, "ms_per_launch_median": head["ms_per_launch_median"],
                "ms_per_launch_min": head["ms_per_launch_min"]}
    if head["other_policy"] and head["other_policy"]["traffic"]:
        o = head["other_policy"]
        o["moved"] = None if o["traffic"]["stale"] else moved_of(o["traffic"], o["algorithmic_bytes_per_launch"], o["ms_per_step"])
        o["traffic"] = None if o["traffic"]["stale"] else o["traffic"]["bytes"]
    Q, f = r.Q, r.f
    result = {
        "metric": "hot-path elements/sec at 1 MI355X + % of HBM/MFMA roofline",
        "value": Q / (head["wall_ms_per_step"] * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["wall_ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / fp32 timestamps (copied and compared, no arithmetic)",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.description}; query i = (src[i], -inf, ts[i]); f={f}, tau={wl.tau}, "
                               f"policy={args.policy}, window={'0.25 span' if args.windowed else 'unbounded'}",
                   "queries": Q, "instances": wl.num_instances, "nodes_per_instance": wl.num_nodes,
                   "placement": args.placement, "ingest": args.ingest, "layout": args.layout},
        "roofline": roofline,
        "two_kernel_path": head["two_kernel_path"],
        "dense_only": head["dense_only"],
        "other_policy": head["other_policy"],
        "sampled_edges_per_s": head["total_k"] / (head["wall_ms_per_step"] * 1e-3),
        "per_query": bm["per_query"],
        "store": head["store"], "ingest_s": head["ingest_s"], "commit_s": head["commit_s"],
    }
    if args.cpu_seconds > 0 and wl.num_instances == 1:
        result["cpu_baseline"] = cpu_baseline(wl, policy, wl.seed, args.cpu_seconds, r.out, torch)
    else:
        result["cpu_baseline"] = None
    r.close()
    del r
    torch.cuda.empty_cache()

    result["other_layout"] = None
    result["other_configs"] = None
    if plain and not args.no_side:
        other_layout = "prefix" if args.layout == "blocks" else "blocks"
        r2, fig = measure_layout(other_layout, False)
        r2.close()
        del r2
        torch.cuda.empty_cache()
        b2 = fig["byte_model"]
        t2 = fig["traffic"]
        result["other_layout"] = {
            "layout": other_layout, "ms_per_step": fig["ms_per_launch"], "value": Q / (fig["ms_per_launch"] * 1e-3), "unit": "elements/s",
            "steps": 5, "algorithmic_bytes_per_launch": b2["step"], "frac": b2["step"] / (fig["ms_per_launch"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "bytes_breakdown": b2["parts"], "per_query": b2["per_query"],
            "traffic": None if not t2 or t2["stale"] else t2["bytes"], "traffic_stale": bool(t2 and t2["stale"]),
            "moved": None if not t2 or t2["stale"] else moved_of(t2, b2["step"], fig["ms_per_launch"]),
            "two_kernel_path": fig["two_kernel_path"], "dense_only": fig["dense_only"], "other_policy": fig["other_policy"],
            "store": fig["store"],
            "ingest_s": fig["ingest_s"], "commit_s": fig["commit_s"]}
        if fig["other_policy"] and fig["other_policy"]["traffic"]:
            o = fig["other_policy"]
            o["moved"] = None if o["traffic"]["stale"] else moved_of(o["traffic"], o["algorithmic_bytes_per_launch"], o["ms_per_step"])
            o["traffic"] = None if o["traffic"]["stale"] else o["traffic"]["bytes"]
        if wl.name == "C5" and not args.profile_run:
            log("the smaller configurations")
            result["other_configs"] = {name: side_config(B, torch, W, name, args.layout, 20) for name in ("C1", "C2", "C3", "C4")}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
