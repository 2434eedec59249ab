"""Pins for the layout-free CPU oracle (oracle/tns_oracle.c).

Each test ties the oracle to something other than itself: the worked example the paper
states in section 2.1, closed forms, numpy library routines, brute force over all edges,
and invariants that hold for any input.  A dropped term, wrong sign, off-by-one or
swapped operand in the oracle fails at least one of them.
"""
import os

import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers (test-local)

def brute_force(num_nodes, src, dst, ts, eid, target, t_s, t_e, f, inclusive):
    """All edges of `target` inside the window by a scan over the whole stream, ordered by
    (time, arrival); returns the newest min(f, c) newest-first plus c and the full list."""
    cands = []
    if 0 <= target < num_nodes:
        for i in range(len(src)):
            if src[i] != target:
                continue
            t = ts[i]
            if t < t_s:
                continue
            if inclusive:
                if t > t_e:
                    continue
            elif t >= t_e:
                continue
            cands.append((float(t), i))
    cands.sort()          # python sort is stable on (time, arrival index)
    order = [i for _, i in cands]
    newest_first = order[::-1][:f]
    return newest_first, len(order), order


def check_rows(out, q, rows, dst, eid, ts, f):
    k = len(rows)
    assert out.count[q] == k
    assert list(out.nbr[q, :k]) == [dst[i] for i in rows]
    assert list(out.eid[q, :k]) == [eid[i] for i in rows]
    assert list(out.ts[q, :k]) == [ts[i] for i in rows]
    assert np.all(out.nbr[q, k:] == -1) and np.all(out.eid[q, k:] == -1) and np.all(out.ts[q, k:] == 0.0)


# ---------------------------------------------------------------- P1 worked example

def _load_worked_example():
    edges, queries = [], []
    with open(os.path.join(GOLDEN, "worked_example_sec2_1.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if "->" in line:
                lhs, rhs = line.split("->")
                node, t = lhs.split()
                queries.append((int(node), float(t), [int(x) for x in rhs.split()]))
            else:
                s, d, t = line.split()
                edges.append((int(s), int(d), float(t)))
    return edges, queries


def test_p1_worked_example_section_2_1(oracle_lib):
    edges, queries = _load_worked_example()
    src = np.array([e[0] for e in edges], np.int32)
    dst = np.array([e[1] for e in edges], np.int32)
    ts = np.array([e[2] for e in edges], np.float32)
    adj = oracle_lib.Adjacency(3, src, dst, ts)
    for node, t, expect in queries:
        for pol in (0, 1):
            out = adj.sample([node], None, [t], fanout=4, policy=pol, inclusive_end=1)
            assert out.count[0] == len(expect)
            assert sorted(out.nbr[0, :len(expect)]) == sorted(expect)     # C sampled twice
        rec = adj.sample([node], None, [t], fanout=4, policy=0, inclusive_end=1)
        assert list(rec.ts[0, :2]) == [23.0, 12.0]                        # closest to t first
    # Algorithm 1's half-open window excludes the edge at the query time itself
    out = adj.sample([0], None, [23.0], fanout=4, inclusive_end=0)
    assert out.count[0] == 1 and out.nbr[0, 0] == 2 and out.ts[0, 0] == 12.0
    # a later query sees the 30 s edge to B first, and the window start cuts the 12 s edge
    out = adj.sample([0], None, [31.0], fanout=4)
    assert list(out.nbr[0, :3]) == [1, 2, 2] and out.count[0] == 3
    out = adj.sample([0], [20.0], [31.0], fanout=4)
    assert list(out.ts[0, :2]) == [30.0, 23.0] and out.count[0] == 2
    # fan-out smaller than the candidate count: the most recent ones only
    out = adj.sample([0], None, [31.0], fanout=2)
    assert list(out.ts[0]) == [30.0, 23.0] and out.count[0] == 2


# ---------------------------------------------------------------- P2 closed form

@pytest.mark.parametrize("f", [1, 3, 10])
def test_p2_closed_form_single_node(oracle_lib, f):
    m = 40
    src = np.zeros(m, np.int32)
    dst = np.arange(100, 100 + m, dtype=np.int32)
    ts = np.arange(m, dtype=np.float32)
    adj = oracle_lib.Adjacency(1, src, dst, ts)
    for x in range(0, m + 3):
        out = adj.sample([0], None, [float(x)], fanout=f)
        k = min(f, x, m) if x <= m else min(f, m)
        top = min(x, m)
        assert out.count[0] == k
        assert list(out.eid[0, :k]) == [top - 1 - j for j in range(k)]
        assert list(out.nbr[0, :k]) == [100 + top - 1 - j for j in range(k)]
        inc = adj.sample([0], None, [float(x)], fanout=f, inclusive_end=1)
        top_i = min(x + 1, m)
        assert inc.count[0] == min(f, top_i)
        assert list(inc.eid[0, :inc.count[0]]) == [top_i - 1 - j for j in range(inc.count[0])]
        for w in (0, 1, 4, 50):
            win = adj.sample([0], [float(x - w)], [float(x)], fanout=f)
            assert win.count[0] == min(f, w, top, max(0, top - max(x - w, 0)))


# ---------------------------------------------------------------- P3 / P4 library reductions

def test_p3_full_window_is_csr_row_reversed(oracle_lib):
    st = W.tiny_stream(11, 500, 17, 64, ties=True)
    deg = np.bincount(st.src, minlength=st.num_nodes)
    f = int(deg.max()) + 1
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    order = np.argsort(st.src, kind="stable")
    starts = np.concatenate([[0], np.cumsum(deg)])
    targets = np.arange(st.num_nodes, dtype=np.int32)
    out = adj.sample(targets, None, np.full(st.num_nodes, np.inf, np.float32), fanout=f)
    for v in range(st.num_nodes):
        row = order[starts[v]:starts[v + 1]][::-1]
        assert out.count[v] == len(row)
        assert np.array_equal(out.eid[v, :len(row)], row.astype(np.int32))
        assert np.array_equal(out.nbr[v, :len(row)], st.dst[row])
        assert np.array_equal(out.ts[v, :len(row)], st.ts[row])


@pytest.mark.parametrize("inclusive,side", [(0, "left"), (1, "right")])
def test_p4_fanout_one_is_searchsorted(oracle_lib, inclusive, side):
    st = W.tiny_stream(5, 800, 9, 100, ties=True)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    targets, _, t_end = W.random_queries(6, st, 600, with_start=False)
    out = adj.sample(targets, None, t_end, fanout=1, inclusive_end=inclusive)
    for q in range(len(targets)):
        v = targets[q]
        if not (0 <= v < st.num_nodes):
            assert out.count[q] == 0
            continue
        idx = np.nonzero(st.src == v)[0]
        pos = np.searchsorted(st.ts[idx], t_end[q], side=side) - 1
        if pos < 0:
            assert out.count[q] == 0
        else:
            assert out.count[q] == 1 and out.eid[q, 0] == idx[pos]


# ---------------------------------------------------------------- P5 brute force

@pytest.mark.parametrize("f", [1, 2, 10, 64])
@pytest.mark.parametrize("inclusive", [0, 1])
def test_p5_brute_force_tiny(oracle_lib, f, inclusive):
    for seed in range(4):
        st = W.tiny_stream(100 + seed, 64, 5, 16, ties=(seed % 2 == 0))
        eid = np.arange(st.n, dtype=np.int32)
        adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
        targets, t_start, t_end = W.random_queries(200 + seed, st, 120)
        out = adj.sample(targets, t_start, t_end, fanout=f, inclusive_end=inclusive)
        out_nostart = adj.sample(targets, None, t_end, fanout=f, inclusive_end=inclusive)
        for q in range(len(targets)):
            rows, c, _ = brute_force(st.num_nodes, st.src, st.dst, st.ts, eid, int(targets[q]),
                                     float(t_start[q]), float(t_end[q]), f, inclusive)
            check_rows(out, q, rows, st.dst, eid, st.ts, f)
            rows, c, _ = brute_force(st.num_nodes, st.src, st.dst, st.ts, eid, int(targets[q]),
                                     -np.inf, float(t_end[q]), f, inclusive)
            check_rows(out_nostart, q, rows, st.dst, eid, st.ts, f)


def test_p5_brute_force_c1(oracle_lib):
    wl = W.c1()
    st = wl.streams[0]
    eid = np.arange(st.n, dtype=np.int32)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    targets, _, t_end, _ = wl.queries()
    out = adj.sample(targets, None, t_end, fanout=wl.fanout)
    tw, t_start, _, _ = wl.queries(window_frac=0.25)
    outw = adj.sample(targets, t_start, t_end, fanout=wl.fanout)
    for q in range(0, st.n, 3):
        rows, _, _ = brute_force(st.num_nodes, st.src, st.dst, st.ts, eid, int(targets[q]), -np.inf,
                                 float(t_end[q]), wl.fanout, 0)
        check_rows(out, q, rows, st.dst, eid, st.ts, wl.fanout)
        rows, _, _ = brute_force(st.num_nodes, st.src, st.dst, st.ts, eid, int(targets[q]), float(t_start[q]),
                                 float(t_end[q]), wl.fanout, 0)
        check_rows(outw, q, rows, st.dst, eid, st.ts, wl.fanout)


# ---------------------------------------------------------------- P6 invariants at size

def check_invariants(st, targets, t_start, t_end, out, f, inclusive=0, recent=True, self_queries=False):
    """Properties that hold at any size; also used by the GPU parity tests on C5."""
    q = len(targets)
    cnt = out.count.astype(np.int64)
    assert cnt.min() >= 0 and cnt.max() <= f
    slot = np.arange(f)[None, :]
    filled = slot < cnt[:, None]
    assert np.all(out.nbr[~filled] == -1) and np.all(out.eid[~filled] == -1) and np.all(out.ts[~filled] == 0.0)
    e = out.eid[filled].astype(np.int64)
    qq = np.broadcast_to(np.arange(q)[:, None], (q, f))[filled]
    assert np.all((e >= 0) & (e < st.n))
    assert np.array_equal(st.src[e], targets[qq])
    assert np.array_equal(st.dst[e], out.nbr[filled])
    assert np.array_equal(st.ts[e], out.ts[filled])
    if inclusive:
        assert np.all(st.ts[e] <= t_end[qq])
    else:
        assert np.all(st.ts[e] < t_end[qq])
    if t_start is not None:
        assert np.all(st.ts[e] >= t_start[qq])
    if self_queries and not inclusive:
        assert np.all(e < qq)               # a query taken from event i only sees earlier events
    if recent:
        d = np.diff(out.eid.astype(np.int64), axis=1)
        both = filled[:, 1:] & filled[:, :-1]
        assert np.all(d[both] < 0)          # newest first, strictly


def test_p6_invariants_and_counts_c2(oracle_lib):
    wl = W.c2()
    st = wl.streams[0]
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    targets, t_start, t_end, _ = wl.queries(window_frac=0.25)
    for tb in (None, t_start):
        out = adj.sample(targets, tb, t_end, fanout=wl.fanout, threads=8)
        check_invariants(st, targets, tb, t_end, out, wl.fanout, self_queries=True)
        # count == min(f, c) with c recomputed by numpy on per-node sorted arrays
        order = np.argsort(st.src, kind="stable")
        deg = np.bincount(st.src, minlength=st.num_nodes)
        starts = np.concatenate([[0], np.cumsum(deg)])
        ts_sorted = st.ts[order]
        sel = np.arange(0, st.n, 97)
        for q in sel:
            v = targets[q]
            seg = ts_sorted[starts[v]:starts[v + 1]]
            hi = np.searchsorted(seg, t_end[q], side="left")
            lo = 0 if tb is None else np.searchsorted(seg, tb[q], side="left")
            assert out.count[q] == min(wl.fanout, max(hi - lo, 0))
        rowptr, cn, ce, ct = oracle_lib.compact(out)
        assert rowptr[0] == 0 and np.all(np.diff(rowptr) == out.count) and rowptr[-1] == out.count.sum()


def test_o5_compaction_is_masked_flatten(oracle_lib):
    st = W.tiny_stream(3, 300, 7, 50)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    targets, t_start, t_end = W.random_queries(4, st, 200)
    out = adj.sample(targets, t_start, t_end, fanout=5)
    rowptr, cn, ce, ct = oracle_lib.compact(out)
    mask = np.arange(5)[None, :] < out.count[:, None]
    assert np.array_equal(rowptr, np.concatenate([[0], np.cumsum(out.count, dtype=np.int64)]))
    assert np.array_equal(cn, out.nbr[mask]) and np.array_equal(ce, out.eid[mask]) and np.array_equal(ct, out.ts[mask])
    empty = oracle_lib.Sampled(0, 5)
    rp, a, b, c = oracle_lib.compact(empty)
    assert list(rp) == [0] and len(a) == 0


# ---------------------------------------------------------------- P8 uniform policy

def test_p8_generator_matches_published_splitmix64_vectors(oracle_lib):
    # Outputs of the splitmix64 generator for seed 1234567 as published with its reference
    # implementation; slot j of query 0 uses the (j+1)-th output, and c = 2^32 returns its
    # upper half unchanged.
    published = [6457827717110365317, 3203168211198807973, 9817491932198370423,
                 4593380528125082431, 16408922859458223821]
    for j, z in enumerate(published):
        assert oracle_lib.pick(1234567, 0, 10, j, 1 << 32) == z >> 32
    # counter = q*f + j + 1
    assert oracle_lib.pick(1234567, 1, 3, 1, 1 << 32) == published[4] >> 32
    # scaling: floor(u * c / 2^32)
    for c in (1, 2, 7, 1000, (1 << 32) - 1):
        for j, z in enumerate(published):
            assert oracle_lib.pick(1234567, 0, 10, j, c) == ((z >> 32) * c) >> 32


def test_p8_uniform_contract(oracle_lib):
    st = W.tiny_stream(21, 600, 4, 64, ties=True)
    eid = np.arange(st.n, dtype=np.int32)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    targets, t_start, t_end = W.random_queries(22, st, 300)
    f, seed = 6, 99
    uni = adj.sample(targets, t_start, t_end, fanout=f, policy=1, seed=seed)
    rec = adj.sample(targets, t_start, t_end, fanout=f, policy=0)
    q_ids = np.arange(1000, 1300, dtype=np.int64)
    uni_ids = adj.sample(targets, t_start, t_end, fanout=f, policy=1, seed=seed, q_ids=q_ids)
    for q in range(len(targets)):
        _, c, order = brute_force(st.num_nodes, st.src, st.dst, st.ts, eid, int(targets[q]),
                                  float(t_start[q]), float(t_end[q]), f, 0)
        if c <= f:      # everything is taken, same as recent
            assert uni.count[q] == rec.count[q] == c
            assert np.array_equal(uni.eid[q], rec.eid[q])
        else:
            assert uni.count[q] == f
            for j in range(f):
                assert uni.eid[q, j] == order[oracle_lib.pick(seed, q, f, j, c)]
                assert uni_ids.eid[q, j] == order[oracle_lib.pick(seed, 1000 + q, f, j, c)]
                assert uni.eid[q, j] in order


def test_p8_uniform_distribution_chi_square(oracle_lib):
    c, f, nq = 1000, 10, 100_000
    src = np.zeros(c, np.int32)
    dst = np.arange(c, dtype=np.int32)
    ts = np.arange(c, dtype=np.float32)
    adj = oracle_lib.Adjacency(1, src, dst, ts)
    out = adj.sample(np.zeros(nq, np.int32), None, np.full(nq, 1e9, np.float32), fanout=f, policy=1, seed=7,
                     threads=8)
    assert np.all(out.count == f)
    hist = np.bincount(out.eid.ravel(), minlength=c)
    expected = nq * f / c
    chi2 = float(((hist - expected) ** 2 / expected).sum())
    # 999 degrees of freedom: mean 999, sd ~44.7; 6 sd either side
    assert 999 - 6 * 44.7 < chi2 < 999 + 6 * 44.7
    # different seeds give different picks, same seed the same picks
    again = adj.sample(np.zeros(100, np.int32), None, np.full(100, 1e9, np.float32), fanout=f, policy=1, seed=7)
    other = adj.sample(np.zeros(100, np.int32), None, np.full(100, 1e9, np.float32), fanout=f, policy=1, seed=8)
    assert np.array_equal(again.eid, out.eid[:100]) and not np.array_equal(other.eid, again.eid)


# ---------------------------------------------------------------- arrival-order rules and errors

def test_batches_sort_inside_reject_across(oracle_lib):
    src = np.zeros(6, np.int32)
    dst = np.arange(6, dtype=np.int32)
    ts = np.array([1, 3, 2, 2, 5, 4], np.float32)       # out of order inside the stream
    # one batch: stable sort by time -> arrival order among the two edges at time 2 is kept
    adj = oracle_lib.Adjacency(1, src, dst, ts)
    out = adj.sample([0], None, [np.inf], fanout=6)
    assert list(out.eid[0]) == [4, 5, 1, 3, 2, 0]
    # batches [0,3) and [3,6): second batch starts at time 2 < 3 already stored -> rejected
    with pytest.raises(oracle_lib.OracleError) as ei:
        oracle_lib.Adjacency(1, src, dst, ts, batch_rowptr=[0, 3, 6])
    assert ei.value.code == -2
    # batches [0,2) and [2,6) are fine only if the second starts no earlier than 3
    ts2 = np.array([1, 3, 4, 3, 5, 4], np.float32)
    adj2 = oracle_lib.Adjacency(1, src, dst, ts2, batch_rowptr=[0, 2, 6])
    out2 = adj2.sample([0], None, [np.inf], fanout=6)
    assert list(out2.eid[0]) == [4, 5, 2, 3, 1, 0]
    with pytest.raises(oracle_lib.OracleError) as ei:
        oracle_lib.Adjacency(1, np.array([0, 1], np.int32), dst[:2], ts[:2])
    assert ei.value.code == -3
    with pytest.raises(oracle_lib.OracleError) as ei:
        oracle_lib.Adjacency(1, src[:2], dst[:2], np.array([0, np.nan], np.float32))
    assert ei.value.code == -2


def test_deleted_edges_are_absent(oracle_lib):
    st = W.tiny_stream(31, 200, 3, 32)
    rng = np.random.default_rng(0)
    present = (rng.random(st.n) > 0.3).astype(np.uint8)
    full = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts, present=present)
    keep = np.nonzero(present)[0]
    ref = oracle_lib.Adjacency(st.num_nodes, st.src[keep], st.dst[keep], st.ts[keep], eid=keep.astype(np.int32))
    targets, t_start, t_end = W.random_queries(32, st, 100)
    for pol in (0, 1):
        a = full.sample(targets, t_start, t_end, fanout=4, policy=pol, seed=5)
        b = ref.sample(targets, t_start, t_end, fanout=4, policy=pol, seed=5)
        assert np.array_equal(a.eid, b.eid) and np.array_equal(a.count, b.count)


def test_edge_cases(oracle_lib):
    adj = oracle_lib.Adjacency(4, np.array([], np.int32), np.array([], np.int32), np.array([], np.float32))
    out = adj.sample([0, 3, 7, -1], None, [1.0, 2.0, 3.0, 4.0], fanout=3)
    assert np.all(out.count == 0) and np.all(out.nbr == -1)
    out = adj.sample(np.array([], np.int32), None, np.array([], np.float32), fanout=3)
    assert out.count.shape == (0,)
    adj = oracle_lib.Adjacency(2, np.array([0, 0], np.int32), np.array([1, 1], np.int32), np.array([1, 2], np.float32))
    out = adj.sample([0, 0, 0, 0], [np.nan, 0, -np.inf, 3], [5, np.nan, np.inf, 2], fanout=3)
    assert list(out.count) == [0, 0, 2, 0]
