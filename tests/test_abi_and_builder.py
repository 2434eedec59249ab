"""CPU-side checks of the product library: it loads without a GPU, exports every symbol the
header declares, validates arguments, and its host-side store builder produces the layout
the paper's sizing rule prescribes (checked against the structural oracle's layout and
closed forms).  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2311_17410_amd import binding as B
from paper_2311_17410_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tns.h")).read()
    declared = re.findall(r"TNS_API\s+[\w\s\*]+?\b(tns_\w+)\s*\(", hdr)
    assert sorted(declared) == sorted(B.EXPORTS)
    from paper_2311_17410_amd import cache_binding as KB
    hdr2 = open(os.path.join(ROOT, "include", "tns_cache.h")).read()
    declared2 = re.findall(r"TNS_API\s+[\w\s\*]+?\b(tns_\w+)\s*\(", hdr2)
    assert sorted(declared2) == sorted(KB.EXPORTS)
    declared = declared + declared2
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_struct_sizes_match_header():
    assert ctypes.sizeof(B.tns_config) == 48
    assert ctypes.sizeof(B.tns_stats_t) == 56


def test_argument_validation():
    for kw, status in [(dict(num_nodes=-1, fanout=10), B.TNS_EINVAL), (dict(num_nodes=4, fanout=0), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=65), B.TNS_EINVAL), (dict(num_nodes=4, fanout=3, policy=2), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, block_threshold=0), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, num_instances=0), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, sizing=3), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, inclusive_end=2), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=256), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=B.TNS_FLAG_PREFIX_LAYOUT | B.TNS_FLAG_DEVICE_INGEST), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=B.TNS_FLAG_PREFIX_LAYOUT | B.TNS_FLAG_EDGES_ON_HOST), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=B.TNS_FLAG_DEVICE_INGEST | B.TNS_FLAG_EDGES_ON_HOST), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=B.TNS_FLAG_DEVICE_INGEST | B.TNS_FLAG_NO_NODE_SLAB), B.TNS_EINVAL),
                       (dict(num_nodes=4, fanout=3, flags=B.TNS_FLAG_EDGES_ON_HOST | B.TNS_FLAG_ALL_ON_HOST), B.TNS_EINVAL)]:
        with pytest.raises(B.TnsError) as ei:
            B.tns_plan_create(**kw)
        assert ei.value.status == status
    h = B.tns_plan_create(num_nodes=4, fanout=3, num_instances=2)
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 0, [4], [0], [1.0])
    assert ei.value.status == B.TNS_ERANGE
    # a store built on the device takes no host batches, and a host-built one no device batches
    hd = B.tns_plan_create(num_nodes=4, fanout=3, flags=B.TNS_FLAG_DEVICE_INGEST)
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(hd, 0, [1], [0], [1.0])
    assert ei.value.status == B.TNS_ESTATE
    B.tns_destroy(hd)
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges_device(h, 0, 0, 0, 0, None, 0, None)
    assert ei.value.status == B.TNS_ESTATE
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 0, [-1], [0], [1.0])
    assert ei.value.status == B.TNS_ERANGE
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 2, [0], [0], [1.0])
    assert ei.value.status == B.TNS_ERANGE
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 0, [0], [0], [float("nan")])
    assert ei.value.status == B.TNS_EORDER
    # run before commit is a state error, reported without touching a GPU
    with pytest.raises(B.TnsError) as ei:
        B.tns_run(h, 1, 8, 0, 8, 8, 0, 8, 8, 8, 8)
    assert ei.value.status == B.TNS_ESTATE
    assert B.tns_workspace(h, 0) >= 0 and B.tns_workspace(h, 1 << 20) > 8 * 1024
    assert B.tns_stats(h)["num_edges"] == 0
    B.tns_destroy(h)
    assert B.lib().tns_destroy(None) == 0
    assert B.lib().tns_strerror(-2).decode().startswith("edges out of")


LAYOUTS = [0, B.TNS_FLAG_PREFIX_LAYOUT]


@pytest.mark.parametrize("layout", LAYOUTS)
def test_out_of_order_batch_rejected_and_store_unchanged(layout):
    h = B.tns_plan_create(num_nodes=2, fanout=3, block_threshold=4, flags=layout)
    B.tns_add_edges(h, 0, [0, 0], [1, 1], [1.0, 5.0])
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 0, [1, 0], [0, 0], [6.0, 4.0])
    assert ei.value.status == B.TNS_EORDER
    assert B.tns_stats(h)["num_edges"] == 2 and B.tns_stats(h)["num_blocks"] == 1
    B.tns_add_edges(h, 0, [0, 0], [1, 1], [7.0, 5.0])       # sorted inside the batch
    blk = B.tns_node_blocks(h, 0, 0)
    assert list(blk["cap"]) == [2, 2] and list(blk["t_min"]) == [1.0, 5.0] and list(blk["t_max"]) == [5.0, 7.0]
    B.tns_destroy(h)


def test_sizing_closed_forms():
    h = B.tns_plan_create(num_nodes=1, fanout=3, block_threshold=16)
    for i in range(100):
        B.tns_add_edges(h, 0, [0], [i], [float(i)])
    caps = list(B.tns_node_blocks(h, 0, 0)["cap"])
    assert caps[:6] == [1, 1, 2, 4, 8, 16] and set(caps[6:]) == {16}
    # 11 blocks > 7 inline records: the node's records moved to a 16-record directory run
    # (16-byte record + 4-byte cumulative edge count each)
    assert len(caps) == 11 and B.tns_stats(h)["metadata_bytes"] == 128 + 16 * (16 + 4)
    blk = B.tns_node_blocks(h, 0, 0)
    assert list(blk["t_min"][:4]) == [0.0, 1.0, 2.0, 4.0] and blk["t_max"][-1] == 99.0
    B.tns_destroy(h)
    h = B.tns_plan_create(num_nodes=2, fanout=3, block_threshold=8)
    B.tns_add_edges(h, 0, [0] * 5, [1] * 5, np.arange(5))
    B.tns_add_edges(h, 0, [0] * 3, [1] * 3, np.arange(5, 8))
    B.tns_add_edges(h, 0, [0] * 30, [1] * 30, np.arange(8, 38))
    B.tns_add_edges(h, 0, [0], [1], [40])
    assert list(B.tns_node_blocks(h, 0, 0)["cap"]) == [5, 5, 28, 8]
    st = B.tns_stats(h)
    assert st["wasted_slots"] == 7 and st["num_edges"] == 39 and st["max_list_len"] == 4
    # edge lines of 10 slots: the two 5-slot blocks share the node's own line, 28 slots take 3 lines,
    # the 8-slot block a line of its own; two node lines, no directory run
    assert st["edge_data_bytes"] == 5 * 128 and st["metadata_bytes"] == 2 * 128
    B.tns_destroy(h)


def test_prefix_layout_closed_forms():
    # same block lists as the default layout; the first blocks (1, 1, 2, 4, 8, 16 = 32 slots) are carved out
    # of the node's prefix (own line + three extension lines), the later ones get records in a directory run
    h = B.tns_plan_create(num_nodes=1, fanout=3, block_threshold=16, flags=B.TNS_FLAG_PREFIX_LAYOUT)
    for i in range(100):
        B.tns_add_edges(h, 0, [0], [i], [float(i)])
    blk = B.tns_node_blocks(h, 0, 0)
    caps = list(blk["cap"])
    assert caps[:6] == [1, 1, 2, 4, 8, 16] and set(caps[6:]) == {16} and len(caps) == 11
    assert list(blk["t_min"][:7]) == [0.0, 1.0, 2.0, 4.0, 8.0, 16.0, 32.0] and blk["t_max"][-1] == 99.0
    assert list(blk["size"]) == [1, 1, 2, 4, 8, 16, 16, 16, 16, 16, 4]
    st = B.tns_stats(h)
    # node entry 32 B + one run of 8 records for the five blocks outside the prefix; edge data: 96 B in the
    # node's line, 3 extension lines, 5 blocks of 16 slots in 2 lines each
    assert st["metadata_bytes"] == 32 + 8 * (16 + 4) and st["edge_data_bytes"] == 96 + (3 + 10) * 128
    assert st["wasted_slots"] == 12 and st["num_blocks"] == 11 and st["max_list_len"] == 11
    B.tns_destroy(h)
    # a first batch larger than the prefix: no prefix block at all
    h = B.tns_plan_create(num_nodes=2, fanout=3, block_threshold=8, flags=B.TNS_FLAG_PREFIX_LAYOUT)
    B.tns_add_edges(h, 0, [1] * 50, [0] * 50, np.arange(50))
    B.tns_add_edges(h, 0, [1] * 3, [0] * 3, np.arange(50, 53))
    assert list(B.tns_node_blocks(h, 0, 1)["cap"]) == [50, 8] and list(B.tns_node_blocks(h, 0, 1)["size"]) == [50, 3]
    B.tns_destroy(h)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("sizing", [0, 1, 2])
@pytest.mark.parametrize("tau,batch", [(1, 64), (48, 128), (8192, 1 << 12), (16, 1 << 14)])
def test_layout_matches_structural_oracle(oracle_lib, sizing, tau, batch, layout):
    st = W.zipf_stream(np.random.Generator(np.random.PCG64(9)), 1 << 14, 1 << 9, batch, 1.1, "normal")
    h = B.tns_plan_create(num_nodes=st.num_nodes, fanout=10, block_threshold=tau, sizing=sizing, flags=layout)
    for lo, hi in st.batches():
        B.tns_add_edges(h, 0, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi])
    bs = oracle_lib.BlockStore(st.num_nodes, tau, sizing)
    bs.add_stream(st.src, st.dst, st.ts, batch)
    ref = bs.blocks()
    os_ = bs.stats()
    ps = B.tns_stats(h)
    assert ps["num_blocks"] == os_["num_blocks"] and ps["wasted_slots"] == os_["wasted_slots"]
    assert ps["max_list_len"] == os_["max_list_len"] and abs(ps["avg_list_len"] - os_["avg_list_len"]) < 1e-12
    if sizing == 0:
        assert ps["wasted_slots"] < st.n          # waste bound of section 4.1
    starts = np.concatenate([[0], np.cumsum(np.bincount(ref["node"], minlength=st.num_nodes))])
    for v in range(st.num_nodes):
        got = B.tns_node_blocks(h, 0, v)
        sl = slice(starts[v], starts[v + 1])
        assert np.array_equal(got["cap"], ref["cap"][sl]) and np.array_equal(got["size"], ref["size"][sl])
        assert np.array_equal(got["t_min"], ref["t_min"][sl]) and np.array_equal(got["t_max"], ref["t_max"][sl])
    B.tns_destroy(h)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_instances_are_independent_in_the_builder(layout):
    h = B.tns_plan_create(num_nodes=3, fanout=2, block_threshold=4, num_instances=3, flags=layout)
    B.tns_add_edges(h, 0, [0, 1], [1, 2], [5.0, 6.0])
    B.tns_add_edges(h, 2, [0, 0, 0], [1, 2, 1], [1.0, 2.0, 3.0])   # older times are fine in another instance
    assert B.tns_stats(h, 0)["num_edges"] == 2 and B.tns_stats(h, 1)["num_edges"] == 0
    assert B.tns_stats(h, 2)["num_edges"] == 3 and B.tns_stats(h)["num_edges"] == 5
    assert list(B.tns_node_blocks(h, 2, 0)["cap"]) == [3]
    B.tns_destroy(h)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_tombstone_deletion_on_the_host(layout):
    h = B.tns_plan_create(num_nodes=3, fanout=2, block_threshold=4, flags=layout)
    B.tns_add_edges(h, 0, [0, 0, 1, 0], [1, 2, 0, 1], [1.0, 2.0, 3.0, 4.0])
    with pytest.raises(B.TnsError) as ei:
        B.tns_add_edges(h, 0, [0], [1], [9.0], eid=[-5])             # ids must be non-negative
    assert ei.value.status == B.TNS_EINVAL
    assert B.tns_delete_edges(h, 0, [0, 0, 1], [1, 7, 0]) == 1        # (0,1) exists; (0,7) and (1,0) do not
    assert B.tns_delete_edges(h, 0, [0], [1]) == 0                    # already deleted
    st = B.tns_stats(h)
    assert st["num_edges"] == 4 and st["num_blocks"] == 2             # layout preserved
    with pytest.raises(B.TnsError) as ei:
        B.tns_delete_edges(h, 0, [3], [0])
    assert ei.value.status == B.TNS_ERANGE
    with pytest.raises(B.TnsError) as ei:
        B.tns_delete_nodes(h, 0, [5])
    assert ei.value.status == B.TNS_ERANGE
    B.tns_delete_nodes(h, 0, [2])
    B.tns_delete_nodes(h, 0, [2], deleted=False)
    B.tns_destroy(h)


@pytest.mark.parametrize("script", ["bench.py", "bench_cache.py", "bench_ingest.py", "bench_khop.py"])
def test_benches_refuse_more_than_one_gpu(script):
    # one GPU per box: no collectives, no sharding; the benches say so instead of running
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, script), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
