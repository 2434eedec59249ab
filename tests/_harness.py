"""Shared helpers of the GPU parity tests: run a workload through the HIP library and through
the CPU oracle and compare every output array bit for bit."""
import numpy as np

LAYOUT_FLAGS = 0          # set by the `layout` fixture (conftest.py): flag of the store layout under test


def with_layout(B, flags):
    """`flags` plus the flag of the layout under test; skips the test if the two cannot be combined."""
    if LAYOUT_FLAGS and flags & (B.TNS_FLAG_EDGES_ON_HOST | B.TNS_FLAG_ALL_ON_HOST | B.TNS_FLAG_DEVICE_INGEST | B.TNS_FLAG_NO_NODE_SLAB):
        import pytest
        pytest.skip("this plan's flags exclude the prefix layout")
    return flags | LAYOUT_FLAGS


def build_plan(B, wl, policy=0, inclusive_end=0, seed=0, fanout=None, tau=None, sizing=0, batch=None, flags=0):
    flags = with_layout(B, flags)
    plan = B.Plan(wl.num_nodes, fanout or wl.fanout, policy=policy, block_threshold=tau or wl.tau,
                  num_instances=wl.num_instances, sizing=sizing, inclusive_end=inclusive_end, seed=seed, flags=flags)
    for i, st in enumerate(wl.streams):
        step = batch or st.batch
        for lo in range(0, st.n, step):
            hi = min(lo + step, st.n)
            B.tns_add_edges(plan.handle, i, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
    plan.commit()
    return plan


def gpu_sample(plan, targets, t_start, t_end, inst_rowptr=None, compact=True, query_id_base=0):
    import torch
    dev = torch.device("cuda", plan.device)
    d_targets = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).to(dev)
    d_te = torch.from_numpy(np.ascontiguousarray(t_end, dtype=np.float32)).to(dev)
    d_tb = None if t_start is None else torch.from_numpy(np.ascontiguousarray(t_start, dtype=np.float32)).to(dev)
    d_rp = None
    if plan.num_instances > 1:
        d_rp = torch.from_numpy(np.ascontiguousarray(inst_rowptr, dtype=np.int64)).to(dev)
    out = plan.run(d_targets, d_tb, d_te, d_rp, compact=compact, query_id_base=query_id_base)
    torch.cuda.synchronize(dev)
    Q, f = len(targets), plan.fanout
    res = dict(nbr=out["nbr"].cpu().numpy().reshape(Q, f), eid=out["eid"].cpu().numpy().reshape(Q, f),
               ts=out["ts"].cpu().numpy().reshape(Q, f), count=out["count"].cpu().numpy())
    if compact:
        assert not plan.status(out["workspace"]), "chained scan reported a timeout"
        rowptr = out["rowptr"].cpu().numpy()
        total = int(rowptr[-1])
        res.update(rowptr=rowptr, cmp_nbr=out["cmp_nbr"][:total].cpu().numpy(),
                   cmp_eid=out["cmp_eid"][:total].cpu().numpy(), cmp_ts=out["cmp_ts"][:total].cpu().numpy())
    return res


def oracle_sample(oracle, wl, targets, t_start, t_end, inst_rowptr, fanout, policy, inclusive_end, seed, threads=8,
                  query_id_base=0, adjs=None):
    """The definition, instance by instance (the batched form must equal separate runs)."""
    parts = []
    for i, st in enumerate(wl.streams):
        lo, hi = (0, len(targets)) if inst_rowptr is None else (int(inst_rowptr[i]), int(inst_rowptr[i + 1]))
        adj = adjs[i] if adjs is not None else oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
        q_ids = np.arange(query_id_base + lo, query_id_base + hi, dtype=np.int64)
        parts.append(adj.sample(targets[lo:hi], None if t_start is None else t_start[lo:hi], t_end[lo:hi], fanout,
                                policy=policy, inclusive_end=inclusive_end, seed=seed, q_ids=q_ids, threads=threads))
        if adjs is None:
            adj.close()
    if len(parts) == 1:
        return parts[0]
    out = oracle.Sampled(0, fanout)
    out.nbr = np.concatenate([p.nbr for p in parts])
    out.eid = np.concatenate([p.eid for p in parts])
    out.ts = np.concatenate([p.ts for p in parts])
    out.count = np.concatenate([p.count for p in parts])
    return out


def assert_same(got, ref, oracle=None, what=""):
    for name in ("count", "eid", "nbr", "ts"):
        a, b = got[name], getattr(ref, name)
        if name == "ts":          # bit-exact, also for the sign of zero
            a, b = a.view(np.int32), b.view(np.int32)
        if not np.array_equal(a, b):
            bad = np.argwhere(a != b)[:5]
            raise AssertionError(f"{what}: {name} differs at {bad.tolist()} (gpu {a[tuple(bad[0])]}, oracle {b[tuple(bad[0])]})")
    if "rowptr" in got and oracle is not None:
        rowptr, cn, ce, ct = oracle.compact(ref)
        assert np.array_equal(got["rowptr"], rowptr), f"{what}: rowptr"
        assert np.array_equal(got["cmp_nbr"], cn) and np.array_equal(got["cmp_eid"], ce), f"{what}: compacted ids"
        assert np.array_equal(got["cmp_ts"].view(np.int32), ct.view(np.int32)), f"{what}: compacted ts"
