"""The script that turns rocprofv3 counter CSVs into profiles/traffic.json: calibration on the copy probe, one entry
per fused sampling kernel, and the staleness stamp that bench.py relies on (hand-made CSVs of the profiler's layout)."""
import json
import os

from paper_2311_17410_amd import traffic as T

BLOCKS = "void tns::(anonymous namespace)::tns_sample_kernel<0, false, int, false, true>(tns::SampleArgs, int, unsigned int, int, unsigned int)"
BLOCKS_U = "void tns::(anonymous namespace)::tns_sample_kernel<1, false, int, false, true>(tns::SampleArgs, int, unsigned int, int, unsigned int)"
PREFIX = "void tns::(anonymous namespace)::tns_sample_prefix_kernel<0, false, int, false, true>(tns::SampleArgs, int, unsigned int, int, unsigned int, unsigned int)"
SAMPLE_ONLY = "void tns::(anonymous namespace)::tns_sample_kernel<0, false, int, false, false>(tns::SampleArgs, int, unsigned int, int, unsigned int)"
COUNTING = "void tns::(anonymous namespace)::tns_sample_kernel<0, false, int, true, false>(tns::SampleArgs, int, unsigned int, int, unsigned int)"
COPY = "void (anonymous namespace)::tns_probe_kernel<0, true>(unsigned int __vector(4)*, unsigned int __vector(4) const*, long, unsigned int)"


def _counter_csv(path, counter, rows):
    os.makedirs(path, exist_ok=True)
    with open(os.path.join(path, "x_counter_collection.csv"), "w") as fh:
        fh.write('"Correlation_Id","Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n')
        for i, (name, value) in enumerate(rows):
            fh.write(f'{i},{i},"{name}","{counter}",{value}\n')


def _trace_csv(path, rows):
    os.makedirs(path, exist_ok=True)
    with open(os.path.join(path, "x_kernel_trace.csv"), "w") as fh:
        fh.write('"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"\n')
        t = 1000
        for name, ns in rows:
            fh.write(f'"KERNEL_DISPATCH","{name}",{t},{t + ns}\n')
            t += ns + 10


def test_entries_calibration_and_stamp(tmp_path):
    gib_kib = 1 << 20
    # the profiler prices the copy's reads at half their size: factor 2 for FETCH_SIZE, 1 for WRITE_SIZE
    _counter_csv(tmp_path / "fetch", "FETCH_SIZE", [(COPY, gib_kib / 2), (BLOCKS, 1000.0), (BLOCKS, 3000.0), (BLOCKS_U, 5000.0),
                                                    (PREFIX, 1500.0), (SAMPLE_ONLY, 7.0), (COUNTING, 9.0)])
    _counter_csv(tmp_path / "write", "WRITE_SIZE", [(COPY, gib_kib), (BLOCKS, 4000.0), (BLOCKS, 4000.0), (BLOCKS_U, 4100.0),
                                                    (PREFIX, 4000.0), (SAMPLE_ONLY, 7.0), (COUNTING, 9.0)])
    _trace_csv(tmp_path / "kt", [(COPY, 500000), (BLOCKS, 27000000), (BLOCKS, 27200000), (PREFIX, 26400000), (BLOCKS_U, 31000000)])
    out_json, out_txt = tmp_path / "traffic.json", tmp_path / "summary.txt"
    assert T.main(["--kt", str(tmp_path / "kt"), "--fetch", str(tmp_path / "fetch"), "--write", str(tmp_path / "write"),
                   "--workload", "C5", "--json", str(out_json), "--summary", str(out_txt)]) == 0
    doc = json.loads(out_json.read_text())
    assert abs(doc["factors"]["FETCH_SIZE"] - 2.0) < 1e-12 and abs(doc["factors"]["WRITE_SIZE"] - 1.0) < 1e-12
    assert sorted(doc["entries"]) == ["C5:recent:blocks", "C5:recent:prefix", "C5:uniform:blocks"]     # fused steps only
    e = doc["entries"]["C5:recent:blocks"]
    assert e["dispatches"] == 2
    assert e["fetch_bytes"] == 2000.0 * 1024 * 2.0 and e["write_bytes"] == 4000.0 * 1024 and e["bytes"] == e["fetch_bytes"] + e["write_bytes"]
    assert abs(e["avg_ms"] - 27.1) < 1e-9
    assert doc["entries"]["C5:recent:prefix"]["fetch_bytes"] == 1500.0 * 1024 * 2.0
    assert "tns_sample_prefix_kernel<0,false,int,false,true>" in out_txt.read_text()
    # lookup: fresh for the sources it was stamped with, stale for any other stamp, None for an unknown key
    got = T.lookup(str(out_json), "C5:recent:blocks")
    assert got["bytes"] == e["bytes"] and got["stale"] is False
    assert T.lookup(str(out_json), "C5:uniform:prefix") is None
    doc["source_hash"] = "0" * 16
    out_json.write_text(json.dumps(doc))
    assert T.lookup(str(out_json), "C5:recent:blocks")["stale"] is True


def test_committed_traffic_json_has_the_four_c5_entries():
    doc = json.load(open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "traffic.json")))
    for key in ("C5:recent:blocks", "C5:uniform:blocks", "C5:recent:prefix", "C5:uniform:prefix"):
        e = doc["entries"][key]
        assert e["bytes"] == e["fetch_bytes"] + e["write_bytes"] and 5e10 < e["bytes"] < 3e11
