"""GPU parity of the device-side store builder (tns_add_edges_device): after ingestion on the GPU
the block structure per node must equal the structural oracle's (capacities, sizes, time ranges:
the paper's section 4.1 insertion with the b_v = min(deg, tau) rule) and sampling must equal the
definition oracle bit for bit, for both policies."""
import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W
from _harness import assert_same, gpu_sample, oracle_sample
from conftest import progress

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2311_17410_amd import binding
    binding.lib()
    return binding


def to_dev(a, dtype):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def device_plan(B, wl, policy=0, seed=0, tau=None, sizing=0, batch=None, fanout=None, eids=None, inclusive_end=0):
    plan = B.Plan(wl.num_nodes, fanout or wl.fanout, policy=policy, block_threshold=tau or wl.tau,
                  num_instances=wl.num_instances, sizing=sizing, seed=seed, inclusive_end=inclusive_end,
                  flags=B.TNS_FLAG_DEVICE_INGEST)
    for i, st in enumerate(wl.streams):
        src, dst, ts = to_dev(st.src, np.int32), to_dev(st.dst, np.int32), to_dev(st.ts, np.float32)
        eid = None if eids is None else to_dev(eids, np.int32)
        step = batch or st.batch
        for lo in range(0, st.n, step):
            hi = min(lo + step, st.n)
            plan.add_edges_device(src[lo:hi], dst[lo:hi], ts[lo:hi], None if eid is None else eid[lo:hi], instance=i)
    plan.commit()        # nothing to upload; allowed
    return plan


def wl_of(stream, fanout=10, tau=48):
    return W.Workload("tiny", 0, [stream], fanout=fanout, tau=tau)


@pytest.mark.parametrize("sizing", [0, 1, 2])
@pytest.mark.parametrize("tau,batch", [(1, 64), (48, 128), (8192, 1 << 12), (16, 1 << 14), (4, 1)])
def test_block_structure_matches_structural_oracle(B, oracle_lib, sizing, tau, batch):
    n = 1 << 14 if batch > 1 else 1 << 10
    st = W.zipf_stream(np.random.Generator(np.random.PCG64(9)), n, 1 << 9, batch, 1.1, "normal")
    wl = wl_of(st, tau=tau)
    plan = device_plan(B, wl, tau=tau, sizing=sizing)
    bs = oracle_lib.BlockStore(st.num_nodes, tau, sizing)
    bs.add_stream(st.src, st.dst, st.ts, batch)
    ref, os_, ps = bs.blocks(), bs.stats(), plan.stats()
    assert ps["num_edges"] == st.n
    assert ps["num_blocks"] == os_["num_blocks"] and ps["wasted_slots"] == os_["wasted_slots"]
    assert ps["max_list_len"] == os_["max_list_len"] and abs(ps["avg_list_len"] - os_["avg_list_len"]) < 1e-12
    starts = np.concatenate([[0], np.cumsum(np.bincount(ref["node"], minlength=st.num_nodes))])
    for v in range(st.num_nodes):
        got = plan.node_blocks(v)
        sl = slice(starts[v], starts[v + 1])
        assert np.array_equal(got["cap"], ref["cap"][sl]) and np.array_equal(got["size"], ref["size"][sl]), v
        assert np.array_equal(got["t_min"], ref["t_min"][sl]) and np.array_equal(got["t_max"], ref["t_max"][sl]), v
    # and sampling over it
    targets, t_start, t_end = W.random_queries(10, st, 2000 + 5)
    for policy in (0, 1):
        plan.set_sampler(10, policy, 0, 4)
        got = gpu_sample(plan, targets, t_start, t_end)
        assert_same(got, oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, 10, policy, 0, 4), oracle_lib,
                    f"sizing={sizing} tau={tau} batch={batch} policy={policy}")
    plan.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_ties_and_unsorted_batches(B, oracle_lib, policy):
    # many equal timestamps; inside every batch the arrival order is shuffled, so the device has to
    # sort by time (stable: equal times keep their arrival order); explicit edge ids
    st = W.tiny_stream(41, 6000, 23, 500, ties=True)
    rng = np.random.default_rng(1)
    perm = np.concatenate([lo + rng.permutation(min(500, st.n - lo)) for lo in range(0, st.n, 500)])
    sh = W.Stream(st.num_nodes, st.src[perm], st.dst[perm], st.ts[perm], 500)
    eids = (np.arange(st.n, dtype=np.int32) * 3 + 7).astype(np.int32)
    wl = wl_of(sh, fanout=7, tau=16)
    plan = device_plan(B, wl, policy, seed=9, eids=eids)
    adj = oracle_lib.Adjacency(sh.num_nodes, sh.src, sh.dst, sh.ts, eid=eids, batch_rowptr=list(range(0, st.n, 500)) + [st.n])
    targets, t_start, t_end = W.random_queries(42, st, 3000 + 1)
    for tb in (t_start, None):
        ref = adj.sample(targets, tb, t_end, 7, policy=policy, seed=9)
        assert_same(gpu_sample(plan, targets, tb, t_end), ref, oracle_lib, f"policy={policy}")
    # signed zeros compare equal: arrival order decides, the stored sign is kept
    z = B.Plan(2, 4, flags=B.TNS_FLAG_DEVICE_INGEST)
    ts = np.array([0.0, -0.0, 0.0, -0.0, -1.0], np.float32)
    z.add_edges_device(to_dev([0] * 5, np.int32), to_dev([1, 0, 1, 0, 1], np.int32), to_dev(ts, np.float32))
    got = gpu_sample(z, np.array([0], np.int32), None, np.array([1.0], np.float32))
    assert list(got["eid"][0]) == [3, 2, 1, 0] and list(np.signbit(got["ts"][0])) == [True, False, True, False]
    z.close()
    plan.close()


def test_rejected_batches_change_nothing(B, oracle_lib):
    st = W.tiny_stream(5, 900, 6, 300)
    wl = wl_of(st, fanout=5)
    plan = device_plan(B, wl)
    targets, t_start, t_end = W.random_queries(6, st, 500)
    ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, 5, 0, 0, 0)
    late = float(st.ts[-1]) + 10
    bad = [
        (dict(src=[0, 6], dst=[1, 1], ts=[late, late]), B.TNS_ERANGE),
        (dict(src=[0, -1], dst=[1, 1], ts=[late, late]), B.TNS_ERANGE),
        (dict(src=[0, 1], dst=[1, 1], ts=[late, np.nan]), B.TNS_EORDER),
        (dict(src=[0, 1], dst=[1, 1], ts=[late, -1.0]), B.TNS_EORDER),       # older than node 1's newest edge
        (dict(src=[0, 1], dst=[1, 1], ts=[late, late], eid=[5, -3]), B.TNS_EINVAL),
    ]
    for kw, status in bad:
        with pytest.raises(B.TnsError) as ei:
            plan.add_edges_device(to_dev(kw["src"], np.int32), to_dev(kw["dst"], np.int32), to_dev(kw["ts"], np.float32),
                                  to_dev(kw["eid"], np.int32) if "eid" in kw else None)
        assert ei.value.status == status, kw
        assert plan.stats()["num_edges"] == st.n
        assert_same(gpu_sample(plan, targets, t_start, t_end), ref, oracle_lib, f"after rejected batch {kw}")
    # an empty batch is fine, and the store still accepts good ones
    plan.add_edges_device(to_dev([], np.int32), to_dev([], np.int32), to_dev([], np.float32))
    plan.add_edges_device(to_dev([2], np.int32), to_dev([3], np.int32), to_dev([late], np.float32))
    got = gpu_sample(plan, np.array([2], np.int32), None, np.array([late + 1], np.float32))
    assert got["eid"][0, 0] == st.n and got["nbr"][0, 0] == 3
    plan.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_deletion_on_a_device_built_store(B, oracle_lib, policy):
    st = W.zipf_stream(np.random.Generator(np.random.PCG64(5)), 1 << 13, 1 << 6, 1 << 9, 1.1, "normal")
    wl = wl_of(st, fanout=6, tau=64)
    plan = device_plan(B, wl, policy, seed=21)
    rng = np.random.default_rng(3)
    present = np.ones(st.n, np.uint8)
    victims = rng.choice(st.n, st.n // 5, replace=False).astype(np.int32)
    present[victims] = 0
    twice = np.concatenate([victims, victims[:100]])                   # a repeated request hits only once
    assert B.tns_delete_edges(plan.handle, 0, st.src[twice], twice) == len(victims)
    dead_nodes = np.array([3, 17], np.int32)
    B.tns_delete_nodes(plan.handle, 0, dead_nodes)
    targets, t_start, t_end = W.random_queries(6, st, 3000 + 11)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts, present=present)
    dead = np.isin(targets, dead_nodes)
    for tb in (t_start, None):
        ref = adj.sample(targets, tb, t_end, 6, policy=policy, seed=21)
        ref.count[dead] = 0; ref.nbr[dead] = -1; ref.eid[dead] = -1; ref.ts[dead] = 0
        assert_same(gpu_sample(plan, targets, tb, t_end), ref, oracle_lib, "after deletion")
    # appending after a deletion keeps the tombstones
    more = W.tiny_stream(9, 500, st.num_nodes, 500, ties=False)
    ts2 = (more.ts + st.ts[-1] + 1).astype(np.float32)
    plan.add_edges_device(to_dev(more.src, np.int32), to_dev(more.dst, np.int32), to_dev(ts2, np.float32))
    B.tns_delete_nodes(plan.handle, 0, dead_nodes, deleted=False)
    adj2 = oracle_lib.Adjacency(st.num_nodes, np.concatenate([st.src, more.src]), np.concatenate([st.dst, more.dst]),
                                np.concatenate([st.ts, ts2]), present=np.concatenate([present, np.ones(500, np.uint8)]))
    t_end2 = (t_end + np.float32(ts2[-1] - st.ts[-1])).astype(np.float32)
    ref = adj2.sample(targets, None, t_end2, 6, policy=policy, seed=21)
    assert_same(gpu_sample(plan, targets, None, t_end2), ref, oracle_lib, "after append and restore")
    assert plan.stats()["num_edges"] == st.n + 500
    plan.close()


def test_instances_and_c2_c3(B, oracle_lib):
    for wl in (W.c4(instances=8, log2_n=12), W.c2(), W.c3()):
        progress(f"device ingestion of {wl.name}")
        targets, t_start, t_end, rowptr = wl.queries(window_frac=0.25)
        rp = rowptr if wl.num_instances > 1 else None
        adjs = [oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts) for st in wl.streams]
        plan = device_plan(B, wl, 0, seed=wl.seed)
        for policy in (0, 1):
            plan.set_sampler(wl.fanout, policy, 0, wl.seed)
            got = gpu_sample(plan, targets, t_start, t_end, rp)
            ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, rp, wl.fanout, policy, 0, wl.seed, threads=16, adjs=adjs)
            assert_same(got, ref, oracle_lib, f"{wl.name} policy={policy}")
        # same block statistics as the host builder on the same stream
        host = B.Plan(wl.num_nodes, wl.fanout, block_threshold=wl.tau, num_instances=wl.num_instances)
        for i, st in enumerate(wl.streams):
            host.add_stream(st, instance=i)
        hs, ds = host.stats(), plan.stats()
        for k in ("num_blocks", "num_edges", "wasted_slots", "max_list_len"):
            assert hs[k] == ds[k], (wl.name, k)
        host.close()
        plan.close()
        for a in adjs:
            a.close()


@pytest.mark.parametrize("batch", [1_500_000, 2_500_000])
def test_large_batches_through_both_pipelines(B, oracle_lib, batch):
    """Zipf stream of 2^22 edges in ragged batches of 1.5 M edges (the short planning pipeline: at most 2^21 edges per
    batch, here 367 sort tiles with a ragged last one) and of 2.5 M edges (the general pipeline): sampling equals the
    definition, block statistics equal the host builder's on the same batches."""
    wl = W.c3(log2_n=22)
    st = wl.streams[0]
    progress(f"device ingestion of 2^22 edges in batches of {batch}")
    plan = device_plan(B, wl, 0, seed=wl.seed, batch=batch)
    targets, t_start, t_end, _ = wl.queries(window_frac=0.25)
    adj = oracle_lib.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    for policy in (0, 1):
        plan.set_sampler(wl.fanout, policy, 0, wl.seed)
        got = gpu_sample(plan, targets, t_start, t_end)
        ref = oracle_sample(oracle_lib, wl, targets, t_start, t_end, None, wl.fanout, policy, 0, wl.seed, threads=16, adjs=[adj])
        assert_same(got, ref, oracle_lib, f"batch={batch} policy={policy}")
    host = B.Plan(wl.num_nodes, wl.fanout, block_threshold=wl.tau)
    for lo in range(0, st.n, batch):
        hi = min(lo + batch, st.n)
        B.tns_add_edges(host.handle, 0, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
    hs, ds = host.stats(), plan.stats()
    for k in ("num_blocks", "num_edges", "wasted_slots", "max_list_len"):
        assert hs[k] == ds[k], k
    host.close()
    plan.close()
    adj.close()
