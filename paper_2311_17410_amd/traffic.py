"""HBM traffic of the sampling kernels from rocprofv3 counter runs.

    python -m paper_2311_17410_amd.traffic --kt DIR --fetch DIR --write DIR --workload C5 \
        --json profiles/traffic.json --summary profiles/tns_sample_kernels_C5.txt --command "..."

DIR are the output folders of three runs of the same bench command with `--output-format csv`:
`--kernel-trace --stats`, `--pmc FETCH_SIZE` and `--pmc WRITE_SIZE`.  Both counters are in KiB per
dispatch as the profiler prices them; each is scaled by the factor that makes the library's own copy
kernel (tns_probe_kernel<0, true>, which the bench runs over 1 GiB: reads 1 GiB, writes 1 GiB) come out
at its known size.  The JSON is stamped with a hash of the kernel sources; `lookup` tells a caller
whether the kernels have changed since the counters were taken.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re
import sys

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
PROBE_BYTES = 1 << 30

_SAMPLE = re.compile(r"tns_sample(_prefix)?_kernel<(\d), (true|false), (int|long), (true|false), (true|false)>")
_PROBE = re.compile(r"tns_probe_kernel<(\d), (true|false)>")


# sources that cannot change what the sampling kernels move: the feature cache and the device-side builder
NOT_SAMPLING = ("tns_cache.hip", "tns_ingest.hip", "tns_ingest.h")


def source_hash() -> str:
    """Hash of the sources behind the sampling step (kernels, layouts, host builders, launch code, probes)."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(CSRC, "*"))):
        if path.endswith((".hip", ".h", ".cpp")) and os.path.basename(path) not in NOT_SAMPLING:
            h.update(os.path.basename(path).encode())
            with open(path, "rb") as fh:
                h.update(fh.read())
    return h.hexdigest()[:16]


def lookup(json_path: str, key: str):
    """{"bytes", "fetch_bytes", "write_bytes", "stale", "source"} for `key` ("C5:recent:blocks"), or None."""
    try:
        with open(json_path) as fh:
            doc = json.load(fh)
    except (OSError, ValueError):
        return None
    e = doc.get("entries", {}).get(key)
    if e is None:
        return None
    return {"bytes": e["bytes"], "fetch_bytes": e["fetch_bytes"], "write_bytes": e["write_bytes"],
            "stale": doc.get("source_hash") != source_hash(), "source": "profiles/" + os.path.basename(doc.get("summary", "traffic.json"))}


def short_name(kernel: str):
    """(display name, traffic key suffix or None) of a kernel name from the profiler."""
    m = _SAMPLE.search(kernel)
    if m:
        layout = "prefix" if m.group(1) else "blocks"
        policy = "recent" if m.group(2) == "0" else "uniform"
        name = f"tns_sample{m.group(1) or ''}_kernel<{m.group(2)},{m.group(3)},{m.group(4)},{m.group(5)},{m.group(6)}>"
        fused_step = m.group(5) == "false" and m.group(6) == "true"
        return name, (f"{policy}:{layout}" if fused_step else None)
    m = _PROBE.search(kernel)
    if m:
        return f"tns_probe_kernel<{m.group(1)},{m.group(2)}>", None
    m = re.search(r"(tns_\w+)", kernel)
    return (m.group(1), None) if m else (None, None)


def _one(folder: str, pattern: str) -> str:
    hits = glob.glob(os.path.join(folder, "**", pattern), recursive=True)
    if not hits:
        raise SystemExit(f"traffic: no {pattern} under {folder}")
    return hits[0]


def read_counter(folder: str, counter: str):
    """{display name: [values per dispatch]} of one counter."""
    acc = collections.defaultdict(list)
    with open(_one(folder, "*counter_collection.csv")) as fh:
        for row in csv.DictReader(fh):
            if row["Counter_Name"] != counter:
                continue
            name, _ = short_name(row["Kernel_Name"])
            if name:
                acc[name].append(float(row["Counter_Value"]))
    return acc


def read_trace(folder: str):
    """{display name: [ms per dispatch]} from the kernel trace."""
    acc = collections.defaultdict(list)
    with open(_one(folder, "*kernel_trace.csv")) as fh:
        for row in csv.DictReader(fh):
            name, _ = short_name(row["Kernel_Name"])
            if name:
                acc[name].append((int(row["End_Timestamp"]) - int(row["Start_Timestamp"])) * 1e-6)
    return acc


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--kt", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--json", required=True)
    ap.add_argument("--summary", required=True)
    ap.add_argument("--command", default="python3 bench.py --profile-run", help="the profiled command, quoted in the summary")
    ap.add_argument("--title", default="")
    args = ap.parse_args(argv)

    trace = read_trace(args.kt)
    fetch = read_counter(args.fetch, "FETCH_SIZE")
    write = read_counter(args.write, "WRITE_SIZE")
    avg = lambda v: sum(v) / len(v)
    probe = "tns_probe_kernel<0,true>"
    if probe not in fetch or probe not in write:
        raise SystemExit("traffic: the copy probe launch is missing from the counter runs")
    k_fetch = PROBE_BYTES / (avg(fetch[probe]) * 1024.0)
    k_write = PROBE_BYTES / (avg(write[probe]) * 1024.0)

    entries = {}
    for kernel in sorted(set(fetch) | set(write)):
        name, key = short_name(kernel.replace(",", ", "))
        if key is None or kernel not in fetch or kernel not in write:
            continue
        fb, wb = avg(fetch[kernel]) * 1024.0 * k_fetch, avg(write[kernel]) * 1024.0 * k_write
        entries[f"{args.workload}:{key}"] = {"bytes": fb + wb, "fetch_bytes": fb, "write_bytes": wb, "kernel": kernel,
                                             "dispatches": len(fetch[kernel]), "avg_ms": avg(trace[kernel]) if kernel in trace else None}

    doc = {}
    if os.path.exists(args.json):
        try:
            with open(args.json) as fh:
                doc = json.load(fh)
        except ValueError:
            doc = {}
    h = source_hash()
    if doc.get("source_hash") != h:
        doc = {"entries": {}}           # counters of other kernel sources do not mix with these
    doc["source_hash"] = h
    doc["factors"] = {"FETCH_SIZE": k_fetch, "WRITE_SIZE": k_write}
    doc["summary"] = os.path.basename(args.summary)
    doc["note"] = ("HBM bytes per launch of the fused sampling kernels: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled so that "
                   "the library's 1 GiB copy kernel reads and writes 1 GiB; written by python -m paper_2311_17410_amd.traffic")
    doc.setdefault("entries", {}).update(entries)
    with open(args.json, "w") as fh:
        json.dump(doc, fh, indent=1, sort_keys=True)
        fh.write("\n")

    lines = [args.title or f"rocprofv3 summary: sampling kernels on {args.workload}", "MI355X, ROCm 7.2, one GPU; kernel sources " + h + ".",
             "Commands (from /tmp with TMPDIR=/tmp, R = repo root):", "",
             f"  rocprofv3 --kernel-trace --stats --output-format csv -d $R/gpurun_out/prof/kt -o kt -- {args.command}",
             f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d $R/gpurun_out/prof/fetch -o fetch -- {args.command}",
             f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d $R/gpurun_out/prof/write -o write -- {args.command}",
             f"  python3 -m paper_2311_17410_amd.traffic --kt gpurun_out/prof/kt --fetch gpurun_out/prof/fetch --write gpurun_out/prof/write "
             f"--workload {args.workload} --json profiles/traffic.json --summary profiles/{os.path.basename(args.summary)}", "",
             "Template arguments of the sampling kernels: <policy (0 recent, 1 uniform), inclusive window end, position type,",
             "counting pass (byte model), padding removal fused>.  <p,false,int,false,true> is the timed step.", "",
             "kernel trace (ms per dispatch): name, dispatches, avg, min, max"]
    for k in sorted(trace):
        v = trace[k]
        lines.append(f"  {k:52s} {len(v):4d} {avg(v):10.4f} {min(v):10.4f} {max(v):10.4f}")
    lines += ["", f"counter calibration on {probe} (copy of 1 GiB): FETCH_SIZE reads {avg(fetch[probe]):.0f} KiB -> factor {k_fetch:.4f}; "
                  f"WRITE_SIZE reads {avg(write[probe]):.0f} KiB -> factor {k_write:.4f}", "",
              "counters (KiB per dispatch as reported, avg): name, dispatches, FETCH_SIZE, WRITE_SIZE, scaled bytes read + written"]
    for k in sorted(set(fetch) | set(write)):
        fv, wv = fetch.get(k), write.get(k)
        fa, wa = (avg(fv) if fv else float("nan")), (avg(wv) if wv else float("nan"))
        lines.append(f"  {k:52s} {len(fv or wv):4d} {fa:16.0f} {wa:16.0f} {(fa * k_fetch + wa * k_write) * 1024 / 1e9:10.2f} GB")
    lines += ["", "traffic entries written to profiles/traffic.json (bytes per launch):"]
    for k, e in sorted(entries.items()):
        lines.append(f"  {k:24s} read {e['fetch_bytes'] / 1e9:8.2f} GB  written {e['write_bytes'] / 1e9:8.2f} GB  total {e['bytes'] / 1e9:8.2f} GB"
                     + (f"  avg {e['avg_ms']:.3f} ms" if e["avg_ms"] else ""))
    with open(args.summary, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    sys.exit(main())
