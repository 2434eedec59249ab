"""Pins for the multi-hop oracle (oracle/khop_oracle.py): each ties the chain to something other than
itself, chosen so that an off-by-one in the next targets, the next window, the fp32 window start, the
per-hop query-id base or the per-instance offsets fails one of them.  No GPU."""
import os

import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def K(oracle_lib):
    from oracle import khop_oracle
    return khop_oracle


def _load_two_hop_example():
    edges, queries = [], []
    with open(os.path.join(GOLDEN, "two_hop_example_sec2_1.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if ";" in line:
                q, hop1, hop2 = (part.split() for part in line.split(";"))
                queries.append((int(q[0]), float(q[1]), [int(x) for x in hop1], {int(x) for x in hop2}))
            else:
                s, d, t = line.split()
                edges.append((int(s), int(d), float(t)))
    return edges, queries


def test_two_hop_toy_example_of_section_2_1(oracle_lib, K):
    # hop 1 of A at 23 s returns C twice (edges at 12 s and 23 s, closed window); the outermost
    # sampled nodes are D and A
    edges, queries = _load_two_hop_example()
    src = np.array([e[0] for e in edges], np.int32)
    dst = np.array([e[1] for e in edges], np.int32)
    ts = np.array([e[2] for e in edges], np.float32)
    order = np.argsort(ts, kind="stable")
    adj = oracle_lib.Adjacency(4, src[order], dst[order], ts[order])
    for node, t, hop1, hop2 in queries:
        hops = K.khop([adj], [node], None, [t], None, [3, 3], policy=0, inclusive_end=1)
        assert list(hops[0]["cmp_nbr"]) == hop1
        assert list(hops[0]["cmp_ts"]) == [23.0, 12.0]
        assert hops[1]["num_queries"] == 2
        assert set(int(x) for x in hops[1]["cmp_nbr"]) == hop2
        # the second layer's queries are C at 23 s and C at 12 s: the one at 12 s cannot see the edge at 23 s
        rp = hops[1]["rowptr"]
        assert np.all(hops[1]["cmp_ts"][rp[1]:rp[2]] <= 12.0)
        assert hops[1]["cmp_ts"][rp[0]:rp[1]].max() == 23.0
    adj.close()


def _newest_before(src, ts, v, t):
    """Brute force: index of the newest edge of v strictly before t (ties: later arrival wins), or -1."""
    best = -1
    for i in range(len(src)):
        if src[i] == v and ts[i] < t and (best < 0 or ts[i] >= ts[best]):
            best = i
    return best


def test_fanout_one_is_a_temporal_walk(oracle_lib, K):
    # fan-outs 1,1,1 against a walk written out edge by edge: an error in which node or which
    # time is handed to the next layer changes the walk
    st = W.tiny_stream(5, 300, 12, 64, ties=True)
    starts = np.array([0, 3, 7, 11, 5, 5], np.int32)
    t0 = np.array([st.ts[-1] + 1, st.ts[150], st.ts[40], st.ts[-1], st.ts[10], -1.0], np.float32)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    hops = K.khop([adj], starts, None, t0, None, [1, 1, 1], policy=0)
    walks = []
    for v, t in zip(starts, t0):
        path = []
        for _ in range(3):
            i = _newest_before(st.src, st.ts, v, t)
            if i < 0:
                break
            path.append(i)
            v, t = st.dst[i], st.ts[i]
        walks.append(path)
    for h in range(3):
        expect = [w[h] for w in walks if len(w) > h]          # edge index == edge id in this stream
        assert list(hops[h]["cmp_eid"]) == expect, h
        assert hops[h]["num_queries"] == (len(starts) if h == 0 else len([w for w in walks if len(w) >= h]))
    adj.close()


def test_window_start_is_subtracted_in_fp32(oracle_lib, K):
    # times near 2^24, where fp32 has a spacing of 2: end - delta is rounded before it is compared.
    # Node 0 -> node 1 at T; node 1 has edges at T-2 and T-4 (exact in fp32).  delta = 3: in fp32
    # T - 3 rounds to T - 4 (ties to even), so the edge at T-4 is inside the second layer's window;
    # computed in double (T - 3 exactly) it would be outside.
    T = np.float32(2 ** 24 + 8)
    src = np.array([1, 1, 0], np.int32)
    dst = np.array([5, 6, 1], np.int32)
    ts = np.array([T - 4, T - 2, T], np.float32)
    assert np.float32(T - np.float32(3.0)) == np.float32(T - 4) and float(T) - 3.0 > float(T - 4)
    adj = oracle_lib.Adjacency(8, src, dst, ts)
    hops = K.khop([adj], [0], None, [T + 2], None, [4, 4], delta=3.0, policy=0)
    assert list(hops[0]["cmp_nbr"]) == [1]
    assert list(hops[1]["cmp_nbr"]) == [6, 5]
    # with delta = 1 the start is T - 1 -> rounds to T (ties to even): nothing older than T qualifies
    hops = K.khop([adj], [0], None, [T + 2], None, [4, 4], delta=1.0, policy=0)
    assert list(hops[1]["cmp_nbr"]) == []
    adj.close()


def test_window_of_later_hops_against_brute_force(oracle_lib, K):
    st = W.tiny_stream(9, 500, 9, 64, ties=True)
    targets, t_start, t_end = W.random_queries(10, st, 40)
    delta = np.float32(30.0)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    hops = K.khop([adj], targets, t_start, t_end, None, [2, 3], delta=float(delta), policy=0)
    q = 0
    for i in range(len(targets)):
        for j in range(hops[0]["padded"].count[i]):
            v, te = hops[0]["padded"].nbr[i, j], hops[0]["padded"].ts[i, j]
            tb = np.float32(te - delta)
            cand = [e for e in range(st.n) if st.src[e] == v and tb <= st.ts[e] < te]
            cand.sort(key=lambda e: (st.ts[e], e))
            expect = cand[::-1][:3]
            rp = hops[1]["rowptr"]
            assert list(hops[1]["cmp_eid"][rp[q]:rp[q + 1]]) == expect, (i, j)
            q += 1
    assert q == hops[1]["num_queries"]
    adj.close()


def test_query_id_bases_per_hop(oracle_lib, K):
    # uniform policy: hop h draws with ids base + cap_1 + ... + cap_{h-1} + i, caps being the most
    # queries a hop can have (Q, Q f1, Q f1 f2), not the numbers it happens to have
    st = W.tiny_stream(21, 3000, 6, 256, ties=False)       # long lists: more candidates than slots
    targets, _, t_end = W.random_queries(22, st, 50)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    fanouts, base, seed = [2, 3, 2], 1000, 77
    hops = K.khop([adj], targets, None, t_end, None, fanouts, policy=1, seed=seed, query_id_base=base)
    Q = len(targets)
    firsts = [base, base + Q, base + Q + Q * 2]
    tg, te = targets, t_end
    for h, f in enumerate(fanouts):
        n = len(tg)
        assert n == hops[h]["num_queries"] and n > 0
        ref = adj.sample(tg, None, te, f, policy=1, seed=seed, q_ids=np.arange(firsts[h], firsts[h] + n, dtype=np.int64))
        assert np.array_equal(ref.eid, hops[h]["padded"].eid), h
        assert (ref.count == f).any()          # the generator was used
        keep = np.arange(f)[None, :] < ref.count[:, None]
        tg, te = ref.nbr[keep], ref.ts[keep]
    # and the picks really depend on the id: a shifted base changes the result
    other = K.khop([adj], targets, None, t_end, None, fanouts, policy=1, seed=seed, query_id_base=base + 1)
    assert not np.array_equal(other[1]["padded"].eid, hops[1]["padded"].eid)
    adj.close()


def test_two_instances_equal_two_separate_chains(oracle_lib, K):
    a = W.tiny_stream(31, 800, 10, 64, ties=True)
    b = W.tiny_stream(32, 600, 10, 64, ties=True)
    ta, _, ea = W.random_queries(33, a, 30)
    tb, _, eb = W.random_queries(34, b, 45)
    adj_a = oracle_lib.Adjacency(a.num_nodes, a.src, a.dst, a.ts)
    adj_b = oracle_lib.Adjacency(b.num_nodes, b.src, b.dst, b.ts)
    fanouts = [3, 2, 2]
    both = K.khop([adj_a, adj_b], np.concatenate([ta, tb]), None, np.concatenate([ea, eb]), [0, 30, 75], fanouts, policy=0)
    only_a = K.khop([adj_a], ta, None, ea, None, fanouts, policy=0)
    only_b = K.khop([adj_b], tb, None, eb, None, fanouts, policy=0)
    for h in range(3):
        na, nb = only_a[h]["num_queries"], only_b[h]["num_queries"]
        assert list(both[h]["inst_rowptr"]) == [0, na, na + nb], h
        assert np.array_equal(both[h]["cmp_eid"], np.concatenate([only_a[h]["cmp_eid"], only_b[h]["cmp_eid"]])), h
        assert np.array_equal(both[h]["cmp_nbr"], np.concatenate([only_a[h]["cmp_nbr"], only_b[h]["cmp_nbr"]])), h
        assert np.array_equal(both[h]["padded"].count, np.concatenate([only_a[h]["padded"].count, only_b[h]["padded"].count])), h
    adj_a.close()
    adj_b.close()


def test_two_instances_uniform_ids_are_global_positions(oracle_lib, K):
    # uniform policy with several instances: a query's generator id is its position in the whole hop
    # (all instances), not its position inside its instance
    a = W.tiny_stream(41, 2500, 5, 256, ties=False)
    b = W.tiny_stream(42, 2500, 5, 256, ties=False)
    ta, _, ea = W.random_queries(43, a, 20)
    tb, _, eb = W.random_queries(44, b, 25)
    adjs = [oracle_lib.Adjacency(s.num_nodes, s.src, s.dst, s.ts) for s in (a, b)]
    fanouts, base, seed = [2, 2], 500, 3
    hops = K.khop(adjs, np.concatenate([ta, tb]), None, np.concatenate([ea, eb]), [0, 20, 45], fanouts, policy=1,
                  seed=seed, query_id_base=base)
    firsts = [base, base + 45]
    tg, te, offs = np.concatenate([ta, tb]), np.concatenate([ea, eb]), np.array([0, 20, 45])
    for h, f in enumerate(fanouts):
        got = hops[h]["padded"]
        drew = False
        for i, adj in enumerate(adjs):
            lo, hi = int(offs[i]), int(offs[i + 1])
            ref = adj.sample(tg[lo:hi], None, te[lo:hi], f, policy=1, seed=seed,
                             q_ids=np.arange(firsts[h] + lo, firsts[h] + hi, dtype=np.int64))
            assert np.array_equal(ref.eid, got.eid[lo:hi]), (h, i)
            drew = drew or bool((ref.count == f).any())
        assert drew
        keep = np.arange(f)[None, :] < got.count[:, None]
        offs = np.concatenate([[0], np.cumsum(got.count)])[offs]
        tg, te = got.nbr[keep], got.ts[keep]
    for adj in adjs:
        adj.close()
