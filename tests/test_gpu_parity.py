"""GPU parity: the HIP library, called through the C ABI binding, against the CPU oracle on
the same seeded inputs.  Every output array must match bit for bit (ids, counts, offsets
are integers; timestamps are copied fp32 values; no arithmetic produces a rounded float)."""
import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W
from _harness import assert_same, build_plan, gpu_sample, oracle_sample, with_layout
from conftest import progress

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("layout")]


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2311_17410_amd import binding
    binding.lib()          # fails loudly if the HIP library is not built
    return binding


def wl_of(stream, name="tiny", fanout=10, tau=48):
    return W.Workload(name, 0, [stream], fanout=fanout, tau=tau)


# ---- small cases: ties, every option, sizes that span tiles with a ragged tail ---------------

@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("inclusive", [0, 1])
@pytest.mark.parametrize("f", [1, 2, 10, 13, 16, 25, 64])
def test_tiny_streams_all_options(B, oracle_lib, policy, inclusive, f):
    st = W.tiny_stream(41, 3000, 23, 256, ties=True)
    wl = wl_of(st, fanout=f)
    targets, t_start, t_end = W.random_queries(42, st, 1000 + 37)      # ragged: not a multiple of 64
    for tau, sizing, batch in [(48, 0, 256), (1, 0, 7), (4, 2, 3000), (8192, 1, 375)]:
        plan = build_plan(B, wl, policy, inclusive, seed=3, tau=tau, sizing=sizing, batch=batch)
        for tb in (t_start, None):
            got = gpu_sample(plan, targets, tb, t_end)
            ref = oracle_sample(oracle_lib, wl, targets, tb, t_end, None, f, policy, inclusive, 3)
            assert_same(got, ref, oracle_lib, f"tau={tau} sizing={sizing} batch={batch} start={'y' if tb is not None else 'n'}")
        # stream-derived queries (query i = event i)
        got = gpu_sample(plan, st.src, None, st.ts)
        ref = oracle_sample(oracle_lib, wl, st.src, None, st.ts, None, f, policy, inclusive, 3)
        assert_same(got, ref, oracle_lib, "self queries")
        plan.close()


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("f", [1, 3, 10, 16])
def test_degrees_around_the_line_boundaries(B, oracle_lib, policy, f):
    """Node v ends with degree v (0..71): every fill of the node's own line (8 slots), of each extension line of the
    prefix layout (18, 28, 38) and of the first blocks outside it, with many equal timestamps across those
    boundaries; ingested one edge, a few edges and all edges per batch (three different block structures); queried at
    every event and a little before / after every distinct time, half-open and closed, with and without a window."""
    rng = np.random.default_rng(77)
    num_nodes = 72
    src = np.repeat(np.arange(num_nodes, dtype=np.int32), np.arange(num_nodes))
    rng.shuffle(src)
    n = len(src)
    dst = rng.integers(0, num_nodes, n, dtype=np.int32)
    ts = np.sort(rng.integers(0, 300, n)).astype(np.float32)
    times = np.unique(ts)
    q_t = np.concatenate([times, np.nextafter(times, np.float32(-np.inf)), np.nextafter(times, np.float32(np.inf))]).astype(np.float32)
    q_v = rng.integers(0, num_nodes, len(q_t), dtype=np.int32)
    targets = np.concatenate([src, q_v, np.repeat(np.arange(num_nodes, dtype=np.int32), 4)])
    t_end = np.concatenate([ts, q_t, np.tile(np.array([-1.0, 150.0, 299.0, 1e9], np.float32), num_nodes)])
    t_start = (t_end - np.float32(40.0)).astype(np.float32)
    for batch in (1, 37, n):
        st = W.Stream(num_nodes, src, dst, ts, batch)
        wl = wl_of(st, fanout=f)
        for incl in (0, 1):
            plan = build_plan(B, wl, policy, incl, seed=9)
            for tb in (None, t_start):
                got = gpu_sample(plan, targets, tb, t_end)
                ref = oracle_sample(oracle_lib, wl, targets, tb, t_end, None, f, policy, incl, 9)
                assert_same(got, ref, oracle_lib, f"batch={batch} incl={incl} window={'y' if tb is not None else 'n'}")
            plan.close()


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("f", [3, 10, 20])
def test_64_bit_edge_positions(B, oracle_lib, policy, f):
    # the kernels keep 64-bit positions once the edge array passes 8 GiB; forced here on a small store
    st = W.tiny_stream(43, 5000, 31, 300, ties=True)
    wl = wl_of(st, fanout=f, tau=16)
    targets, t_start, t_end = W.random_queries(44, st, 2000 + 3)
    plan = build_plan(B, wl, policy, 0, seed=8, flags=B.TNS_FLAG_WIDE_POSITIONS)
    for tb in (t_start, None):
        got = gpu_sample(plan, targets, tb, t_end)
        ref = oracle_sample(oracle_lib, wl, targets, tb, t_end, None, f, policy, 0, 8)
        assert_same(got, ref, oracle_lib, f"policy={policy} f={f}")
    plan.close()


def test_no_ties_long_lists_one_edge_per_batch(B, oracle_lib):
    st = W.tiny_stream(7, 700, 3, 1, ties=False)          # one edge per batch: longest possible lists
    wl = wl_of(st, fanout=10, tau=8)
    targets, t_start, t_end = W.random_queries(8, st, 513)
    for policy in (0, 1):
        plan = build_plan(B, wl, policy, 0, seed=11)
        assert plan.stats()["max_list_len"] > 20
        for tb in (t_start, None):
            got = gpu_sample(plan, targets, tb, t_end)
            ref = oracle_sample(oracle_lib, wl, targets, tb, t_end, None, 10, policy, 0, 11)
            assert_same(got, ref, oracle_lib, f"policy={policy}")
        plan.close()


def test_edge_cases(B, oracle_lib):
    import torch
    st = W.tiny_stream(5, 200, 6, 32)
    wl = wl_of(st, fanout=4)
    plan = build_plan(B, wl)
    # empty query batch: nothing launched that touches memory, rowptr = [0]
    got = gpu_sample(plan, np.array([], np.int32), None, np.array([], np.float32))
    assert got["count"].shape == (0,) and list(got["rowptr"]) == [0]
    # out-of-range ids, NaN and infinite bounds
    targets = np.array([-1, 6, 0, 0, 0, 0, 5, 2147483647, -2147483648], np.int32)
    t_end = np.array([1, 1, np.nan, np.inf, -np.inf, 10, 10, 10, 10], np.float32)
    t_start = np.array([0, 0, 0, -np.inf, -np.inf, np.nan, np.inf, 0, 0], np.float32)
    got = gpu_sample(plan, targets, t_start, t_end)
    ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, 4, 0, 0, 0)
    assert_same(got, ref, oracle_lib, "odd queries")
    assert list(got["count"][[0, 1, 2, 4, 5, 6, 7, 8]]) == [0] * 8
    # without compaction outputs
    got = gpu_sample(plan, targets, t_start, t_end, compact=False)
    assert_same(got, ref, None, "no compaction")
    plan.close()
    # a store with no edges at all
    empty = W.Workload("empty", 0, [W.Stream(5, np.array([], np.int32), np.array([], np.int32), np.array([], np.float32), 8)], fanout=3)
    plan = build_plan(B, empty)
    got = gpu_sample(plan, np.array([0, 4, 9], np.int32), None, np.array([1, 2, 3], np.float32))
    assert np.all(got["count"] == 0) and np.all(got["nbr"] == -1) and list(got["rowptr"]) == [0, 0, 0, 0]
    plan.close()
    # argument errors are reported, nothing is launched
    plan = build_plan(B, wl)
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.TnsError) as ei:
        B.tns_run(plan.handle, 2, t.data_ptr(), 0, t.data_ptr(), 0, 0, t.data_ptr(), t.data_ptr(), t.data_ptr(), 0)
    assert ei.value.status == B.TNS_EINVAL
    with pytest.raises(B.TnsError) as ei:
        B.tns_run(plan.handle, 2, t.data_ptr(), 0, t.data_ptr(), 0, 0, t.data_ptr(), t.data_ptr(), t.data_ptr(),
                  t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), 8)
    assert ei.value.status == B.TNS_ESIZE
    plan.close()


def test_incremental_commit(B, oracle_lib):
    st = W.tiny_stream(61, 4000, 40, 500, ties=True)
    wl = wl_of(st, fanout=10, tau=16)
    plan = B.Plan(st.num_nodes, 10, block_threshold=16, flags=with_layout(B, 0))
    targets, t_start, t_end = W.random_queries(62, st, 777)
    for upto in (500, 1500, 4000):
        lo = 0 if upto == 500 else (500 if upto == 1500 else 1500)
        for a in range(lo, upto, 500):
            B.tns_add_edges(plan.handle, 0, st.src[a:a + 500], st.dst[a:a + 500], st.ts[a:a + 500])
        before = gpu_sample(plan, targets, t_start, t_end) if upto > 500 else None
        plan.commit()
        part = W.Workload("part", 0, [W.Stream(st.num_nodes, st.src[:upto], st.dst[:upto], st.ts[:upto], 500)], fanout=10, tau=16)
        ref = oracle_sample(oracle_lib, part, targets, t_start, t_end, None, 10, 0, 0, 0)
        assert_same(gpu_sample(plan, targets, t_start, t_end), ref, oracle_lib, f"after commit of {upto}")
        if before is not None:      # uncommitted edges were not visible
            assert_same(before, prev_ref, oracle_lib, "snapshot semantics")
        prev_ref = ref
    plan.close()


def test_query_id_base_and_chunked_runs(B, oracle_lib):
    st = W.tiny_stream(71, 5000, 5, 512, ties=False)
    wl = wl_of(st, fanout=6)
    plan = build_plan(B, wl, policy=1, seed=77)
    ref = oracle_sample(oracle_lib, wl, st.src, None, st.ts, None, 6, 1, 0, 77)
    whole = gpu_sample(plan, st.src, None, st.ts)
    assert_same(whole, ref, oracle_lib, "whole")
    cut = 2111
    a = gpu_sample(plan, st.src[:cut], None, st.ts[:cut], compact=False)
    b = gpu_sample(plan, st.src[cut:], None, st.ts[cut:], compact=False, query_id_base=cut)
    assert np.array_equal(np.concatenate([a["eid"], b["eid"]]), ref.eid)
    plan.close()


def test_standalone_compaction_equals_fused(B, oracle_lib):
    import torch
    st = W.tiny_stream(81, 6000, 50, 512, ties=True)
    wl = wl_of(st, fanout=7)
    plan = build_plan(B, wl)
    targets, t_start, t_end = W.random_queries(82, st, 5000 + 13)
    fused = gpu_sample(plan, targets, t_start, t_end)                 # tns_run with the dense outputs
    ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, 7, 0, 0, 0)
    assert_same(fused, ref, oracle_lib, "fused")
    # the same through tns_run (padded only) + tns_compact
    dev = torch.device("cuda", 0)
    Q = len(targets)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    dt, dtb, dte = d(targets), d(t_start), d(t_end)
    out = plan.alloc_outputs(Q, compact=True)
    p = lambda t: t.data_ptr()
    B.tns_run(plan.handle, Q, p(dt), p(dtb), p(dte), 0, 0, p(out["nbr"]), p(out["eid"]), p(out["ts"]), p(out["count"]))
    B.tns_compact(plan.handle, Q, p(out["nbr"]), p(out["eid"]), p(out["ts"]), p(out["count"]), p(out["rowptr"]),
                  p(out["cmp_nbr"]), p(out["cmp_eid"]), p(out["cmp_ts"]), p(out["workspace"]), out["workspace"].numel())
    torch.cuda.synchronize()
    total = int(out["rowptr"][-1].item())
    assert np.array_equal(out["rowptr"].cpu().numpy(), fused["rowptr"])
    for k in ("cmp_nbr", "cmp_eid"):
        assert np.array_equal(out[k][:total].cpu().numpy(), fused[k])
    assert np.array_equal(out["cmp_ts"][:total].cpu().numpy().view(np.int32), fused["cmp_ts"].view(np.int32))
    plan.close()


def test_bounded_wait_of_the_chained_scan_ends(B):
    # failure handling, forced from the host: the tile tickets start at 1, so tile 0 never exists and the
    # first tile's look-back can only end by its bound; every kernel must still finish, and the error
    # word of the workspace must say what happened
    import time
    import torch
    st = W.tiny_stream(17, 40000, 500, 4096, ties=False)
    wl = wl_of(st, fanout=10)
    plan = build_plan(B, wl, 0, flags=B.TNS_TEST_FLAG_LOST_TILE)
    dev = torch.device("cuda", 0)
    d_t, d_e = torch.from_numpy(st.src).to(dev), torch.from_numpy(st.ts).to(dev)
    t0 = time.time()
    out = plan.run(d_t, None, d_e)
    torch.cuda.synchronize()
    assert time.time() - t0 < 60
    assert plan.status(out["workspace"]), "the time-out must be reported"
    assert int(out["rowptr"][-1].item()) == 0, "after a time-out the dense total reads 0"
    plan.close()


def test_step_replayed_from_a_hip_graph(B, oracle_lib):
    # tns_run only enqueues kernels (the chained scan's state is cleared by a kernel, not by a memset),
    # so a step can be captured once and replayed; every replay is checked, with eager work in between
    import torch
    st = W.tiny_stream(91, 20000, 300, 2048, ties=True)
    wl = wl_of(st, fanout=10)
    dev = torch.device("cuda", 0)
    d_t, d_e = torch.from_numpy(st.src).to(dev), torch.from_numpy(st.ts).to(dev)
    for policy in (0, 1):
        plan = build_plan(B, wl, policy, seed=5)
        ref = oracle_sample(oracle_lib, wl, st.src, None, st.ts, None, 10, policy, 0, 5)
        out = plan.alloc_outputs(st.n, compact=True)
        plan.run(d_t, None, d_e, out=out)                      # eager once: loads the code objects
        torch.cuda.synchronize()
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            plan.run(d_t, None, d_e, out=out)
        for rep in range(3):
            for name, t in out.items():
                if name != "workspace":
                    t.zero_()
            assert float((d_e * 2).sum().item()) > 0          # unrelated eager work and a synchronisation
            graph.replay()
            torch.cuda.synchronize()
            total = int(out["rowptr"][-1].item())
            got = dict(nbr=out["nbr"].cpu().numpy().reshape(st.n, 10), eid=out["eid"].cpu().numpy().reshape(st.n, 10),
                       ts=out["ts"].cpu().numpy().reshape(st.n, 10), count=out["count"].cpu().numpy(),
                       rowptr=out["rowptr"].cpu().numpy(), cmp_nbr=out["cmp_nbr"][:total].cpu().numpy(),
                       cmp_eid=out["cmp_eid"][:total].cpu().numpy(), cmp_ts=out["cmp_ts"][:total].cpu().numpy())
            assert_same(got, ref, oracle_lib, f"policy={policy} replay {rep}")
        del graph
        plan.close()


# ---- deletion (tombstones) -------------------------------------------------------------------------

@pytest.mark.parametrize("policy", [0, 1])
def test_deleted_edges_and_nodes_are_ignored(B, oracle_lib, policy):
    st = W.zipf_stream(np.random.Generator(np.random.PCG64(5)), 1 << 13, 1 << 6, 1 << 9, 1.1, "normal")   # a hub with long blocks
    wl = wl_of(st, fanout=6, tau=64)
    plan = build_plan(B, wl, policy, 0, seed=21)
    rng = np.random.default_rng(3)
    present = np.ones(st.n, np.uint8)
    victims = rng.choice(st.n, st.n // 5, replace=False).astype(np.int32)
    present[victims] = 0
    assert B.tns_delete_edges(plan.handle, 0, st.src[victims], victims) == len(victims)
    dead_nodes = np.array([3, 17], np.int32)
    B.tns_delete_nodes(plan.handle, 0, dead_nodes)
    targets, t_start, t_end = W.random_queries(6, st, 3000 + 11)
    before = gpu_sample(plan, targets, t_start, t_end)              # not committed yet: still the old store
    full = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, 6, policy, 0, 21)
    assert_same(before, full, oracle_lib, "before commit")
    plan.commit()
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts, present=present)
    for tb in (t_start, None):
        ref = adj.sample(targets, tb, t_end, 6, policy=policy, seed=21)
        dead = np.isin(targets, dead_nodes)                          # a deleted target returns nothing
        ref.count[dead] = 0; ref.nbr[dead] = -1; ref.eid[dead] = -1; ref.ts[dead] = 0
        got = gpu_sample(plan, targets, tb, t_end)
        assert_same(got, ref, oracle_lib, f"after deletion, start={'y' if tb is not None else 'n'}")
    # edges appended after a deletion land in the same tail blocks; the tombstones stay
    more = W.tiny_stream(9, 500, st.num_nodes, 500, ties=False)
    ts2 = (more.ts + st.ts[-1] + 1).astype(np.float32)
    B.tns_add_edges(plan.handle, 0, more.src, more.dst, ts2)
    plan.commit()
    src_all = np.concatenate([st.src, more.src]); dst_all = np.concatenate([st.dst, more.dst]); ts_all = np.concatenate([st.ts, ts2])
    adj2 = oracle_lib.Adjacency(st.num_nodes, src_all, dst_all, ts_all, present=np.concatenate([present, np.ones(500, np.uint8)]))
    t_end2 = (t_end + np.float32(ts2[-1] - st.ts[-1])).astype(np.float32)
    ref = adj2.sample(targets, None, t_end2, 6, policy=policy, seed=21)
    dead = np.isin(targets, dead_nodes)
    ref.count[dead] = 0; ref.nbr[dead] = -1; ref.eid[dead] = -1; ref.ts[dead] = 0
    assert_same(gpu_sample(plan, targets, None, t_end2), ref, oracle_lib, "after append")
    B.tns_delete_nodes(plan.handle, 0, dead_nodes, deleted=False)
    plan.commit()
    ref = adj2.sample(targets, None, t_end2, 6, policy=policy, seed=21)
    assert_same(gpu_sample(plan, targets, None, t_end2), ref, oracle_lib, "after restoring the nodes")
    plan.close()


# ---- multi-hop --------------------------------------------------------------------------------

def oracle_khop(oracle, wl, targets, t_start, t_end, inst_rowptr, fanouts, delta, policy, seed, base=0):
    """The chained reference (oracle/khop_oracle.py) over the workload's instances, as tuples per hop."""
    from oracle import khop_oracle
    adjs = [oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts) for st in wl.streams]
    hops = khop_oracle.khop(adjs, targets, t_start, t_end, inst_rowptr, fanouts, delta=delta, policy=policy, seed=seed,
                            query_id_base=base, threads=8)
    for a in adjs:
        a.close()
    return [(h["padded"], h["rowptr"], h["cmp_nbr"], h["cmp_eid"], h["cmp_ts"]) for h in hops]


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("fanouts,delta", [([10, 10], float("inf")), ([3, 2, 4], 40.0), ([1, 1, 1, 1], float("inf"))])
def test_khop_matches_chained_oracle(B, oracle_lib, policy, fanouts, delta):
    import torch
    st = W.tiny_stream(91, 4000, 37, 256, ties=True)
    wl = wl_of(st, fanout=fanouts[0])
    plan = build_plan(B, wl, policy, 0, seed=9)
    targets, t_start, t_end = W.random_queries(92, st, 700 + 5)
    dev = torch.device("cuda", 0)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    hops, ws = plan.run_khop(fanouts, d(targets), d(t_start), d(t_end), delta=delta, query_id_base=1000)
    torch.cuda.synchronize()
    assert not plan.status(ws), "a hop's chained scan reported a timeout"
    ref = oracle_khop(oracle_lib, wl, targets, t_start, t_end, None, fanouts, delta, policy, 9, base=1000)
    n = len(targets)
    for h, (r, rowptr, cn, ce, ct) in enumerate(ref):
        f = fanouts[h]
        g = hops[h]
        assert np.array_equal(g["count"][:n].cpu().numpy(), r.count), f"hop {h} count"
        assert np.array_equal(g["eid"][:n * f].cpu().numpy().reshape(n, f), r.eid), f"hop {h} eid"
        assert np.array_equal(g["nbr"][:n * f].cpu().numpy().reshape(n, f), r.nbr), f"hop {h} nbr"
        assert np.array_equal(g["ts"][:n * f].cpu().numpy().reshape(n, f).view(np.int32), r.ts.view(np.int32)), f"hop {h} ts"
        assert np.array_equal(g["rowptr"][:n + 1].cpu().numpy(), rowptr), f"hop {h} rowptr"
        tot = int(rowptr[-1])
        assert np.array_equal(g["cmp_eid"][:tot].cpu().numpy(), ce) and np.array_equal(g["cmp_nbr"][:tot].cpu().numpy(), cn)
        assert np.array_equal(g["cmp_ts"][:tot].cpu().numpy().view(np.int32), ct.view(np.int32))
        n = tot
    plan.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_khop_without_padded_outputs(B, oracle_lib, policy):
    """Hops whose four padded outputs are NULL write their dense result only: rowptr and the dense arrays of every hop
    equal the oracle chain's; a hop that passes some padded outputs but not all is refused."""
    import torch
    fanouts, delta = [10, 3, 12], 25.0
    st = W.tiny_stream(93, 4000, 37, 256, ties=True)
    wl = wl_of(st, fanout=fanouts[0])
    plan = build_plan(B, wl, policy, 0, seed=9)
    targets, t_start, t_end = W.random_queries(94, st, 700 + 5)
    dev = torch.device("cuda", 0)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    d_t, d_b, d_e = d(targets), d(t_start), d(t_end)
    hops, ws = plan.run_khop(fanouts, d_t, d_b, d_e, delta=delta)          # allocates the buffers; result overwritten below
    torch.cuda.synchronize()
    for h in hops:
        for k in ("rowptr", "cmp_nbr", "cmp_eid", "cmp_ts"):
            h[k].fill_(-7)
    p = lambda t: t.data_ptr()
    ptrs = [dict(nbr=0, eid=0, ts=0, count=0, rowptr=p(h["rowptr"]), cmp_nbr=p(h["cmp_nbr"]), cmp_eid=p(h["cmp_eid"]), cmp_ts=p(h["cmp_ts"]))
            for h in hops]
    B.tns_run_khop(plan.handle, fanouts, delta, len(targets), p(d_t), p(d_b), p(d_e), 0, 0, ptrs, ws.data_ptr(), ws.numel(),
                   torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert not plan.status(ws)
    ref = oracle_khop(oracle_lib, wl, targets, t_start, t_end, None, fanouts, delta, policy, 9, base=0)
    n = len(targets)
    for h, (r, rowptr, cn, ce, ct) in enumerate(ref):
        g = hops[h]
        assert np.array_equal(g["rowptr"][:n + 1].cpu().numpy(), rowptr), f"hop {h} rowptr"
        tot = int(rowptr[-1])
        assert np.array_equal(g["cmp_eid"][:tot].cpu().numpy(), ce) and np.array_equal(g["cmp_nbr"][:tot].cpu().numpy(), cn)
        assert np.array_equal(g["cmp_ts"][:tot].cpu().numpy().view(np.int32), ct.view(np.int32))
        n = tot
    ptrs[1]["count"] = p(hops[1]["count"])            # some padded outputs but not all
    with pytest.raises(B.TnsError):
        B.tns_run_khop(plan.handle, fanouts, delta, len(targets), p(d_t), p(d_b), p(d_e), 0, 0, ptrs, ws.data_ptr(), ws.numel(),
                       torch.cuda.current_stream().cuda_stream)
    plan.close()


def test_khop_batched_instances_and_c2(B, oracle_lib):
    import torch
    dev = torch.device("cuda", 0)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    for wl in (W.c4(instances=8, log2_n=12), W.c2()):
        targets, t_start, t_end, rowptr = wl.queries()
        rp = rowptr if wl.num_instances > 1 else None
        plan = build_plan(B, wl, 0, 0)
        fanouts = [10, 10] if wl.num_instances > 1 else [10, 5]
        hops, ws = plan.run_khop(fanouts, d(targets), None, d(t_end), None if rp is None else d(rp))
        torch.cuda.synchronize()
        assert not plan.status(ws), "a hop's chained scan reported a timeout"
        ref = oracle_khop(oracle_lib, wl, targets, None, t_end, rp, fanouts, float("inf"), 0, 0)
        n = len(targets)
        for h, (r, rowptr_h, cn, ce, ct) in enumerate(ref):
            f = fanouts[h]
            assert np.array_equal(hops[h]["count"][:n].cpu().numpy(), r.count), (wl.name, h)
            assert np.array_equal(hops[h]["eid"][:n * f].cpu().numpy().reshape(n, f), r.eid), (wl.name, h)
            assert np.array_equal(hops[h]["rowptr"][:n + 1].cpu().numpy(), rowptr_h), (wl.name, h)
            n = int(rowptr_h[-1])
            assert np.array_equal(hops[h]["cmp_eid"][:n].cpu().numpy(), ce), (wl.name, h)
        plan.close()


# ---- the configurations --------------------------------------------------------------------

def _check_config(B, oracle, wl, threads=16, window=True, policies=(0, 1)):
    targets, t_start, t_end, rowptr = wl.queries(window_frac=0.25)
    rp = rowptr if wl.num_instances > 1 else None
    adjs = [oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts) for st in wl.streams]
    for policy in policies:
        plan = build_plan(B, wl, policy, 0, seed=wl.seed)
        for tb in ((None, t_start) if window else (None,)):
            progress(f"{wl.name} policy={policy} windowed={tb is not None}")
            got = gpu_sample(plan, targets, tb, t_end, rp)
            ref = oracle_sample(oracle, wl, targets, tb, t_end, rp, wl.fanout, policy, 0, wl.seed, threads=threads, adjs=adjs)
            assert_same(got, ref, oracle, f"{wl.name} policy={policy}")
        plan.close()
    for a in adjs:
        a.close()


def test_c1(B, oracle_lib):
    _check_config(B, oracle_lib, W.c1())


def test_c1_literal_id_range(B, oracle_lib):
    _check_config(B, oracle_lib, W.literal_range("C1"))


def test_c2(B, oracle_lib):
    _check_config(B, oracle_lib, W.c2())


def test_c2_literal_id_range(B, oracle_lib):
    _check_config(B, oracle_lib, W.literal_range("C2"), window=False)


def test_c2_inclusive_and_no_remap(B, oracle_lib):
    wl = W.c2()
    targets, _, t_end, _ = wl.queries()
    for incl, flags in ((1, 0), (0, B.TNS_FLAG_NO_XCD_REMAP)):
        plan = build_plan(B, wl, 0, incl, flags=flags)
        got = gpu_sample(plan, targets, None, t_end)
        ref = oracle_sample(oracle_lib, wl, targets, None, t_end, None, wl.fanout, 0, incl, 0, threads=16)
        assert_same(got, ref, oracle_lib, f"incl={incl} flags={flags}")
        plan.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_host_placement_gives_the_same_results(B, oracle_lib, policy):
    # section 4.1: edge data in page-locked host memory with the metadata on the device (hybrid),
    # or everything in host memory; also a second commit after more edges (the arrays grow)
    wl = W.c2()
    st = wl.streams[0]
    targets, t_start, t_end, _ = wl.queries(window_frac=0.25)
    ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, wl.fanout, policy, 0, 5, threads=16)
    for flags in (B.TNS_FLAG_EDGES_ON_HOST, B.TNS_FLAG_ALL_ON_HOST):
        plan = B.Plan(wl.num_nodes, wl.fanout, policy=policy, block_threshold=wl.tau, seed=5, flags=with_layout(B, flags))
        half = st.n // 2
        for lo, hi in ((0, half), (half, st.n)):
            for a in range(lo, hi, st.batch):
                b = min(a + st.batch, hi)
                plan.add_edges(st.src[a:b], st.dst[a:b], st.ts[a:b])
            plan.commit()
        got = gpu_sample(plan, targets, t_start, t_end)
        assert_same(got, ref, oracle_lib, f"policy={policy} flags={flags}")
        plan.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_dense_only_run(B, oracle_lib, policy):
    """tns_run with the four padded outputs NULL writes the dense result only: rowptr and the dense arrays equal the
    oracle's compaction of its padded result; a plan that removes the padding in a step of its own refuses the form."""
    import torch
    wl = W.c2()
    targets, t_start, t_end, _ = wl.queries(window_frac=0.25)
    plan = build_plan(B, wl, policy, 0, seed=3)
    dev = torch.device("cuda", plan.device)
    Q, f = len(targets), wl.fanout
    d = [torch.from_numpy(a).to(dev) for a in (targets, t_start, t_end)]
    full = plan.alloc_outputs(Q, compact=True)
    out = {k: full[k] for k in ("rowptr", "cmp_nbr", "cmp_eid", "cmp_ts", "workspace")}
    plan.run(d[0], d[1], d[2], out=out)
    torch.cuda.synchronize()
    assert not plan.status(out["workspace"])
    ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, f, policy, 0, 3, threads=16)
    rowptr, cn, ce, ct = oracle_lib.compact(ref)
    total = int(rowptr[-1])
    assert np.array_equal(out["rowptr"].cpu().numpy(), rowptr)
    assert np.array_equal(out["cmp_eid"][:total].cpu().numpy(), ce) and np.array_equal(out["cmp_nbr"][:total].cpu().numpy(), cn)
    assert np.array_equal(out["cmp_ts"][:total].cpu().numpy().view(np.int32), ct.view(np.int32))
    # without the dense outputs there is nothing left to write: refused
    with pytest.raises(B.TnsError):
        plan.run(d[0], d[1], d[2], out={}, compact=False)
    # a plan with deleted edges removes the padding in a second step, which reads the padded rows
    st = wl.streams[0]
    assert B.tns_delete_edges(plan.handle, 0, st.src[:1], np.array([0], np.int32)) == 1
    plan.commit()
    with pytest.raises(B.TnsError):
        plan.run(d[0], d[1], d[2], out=out)
    plan.close()


def test_c3_zipf_hub(B, oracle_lib):
    progress("generating C3")
    _check_config(B, oracle_lib, W.c3())


def test_c4_batched_instances(B, oracle_lib):
    progress("generating C4")
    _check_config(B, oracle_lib, W.c4())
