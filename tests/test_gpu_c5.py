"""C5 at full size (n = 2^28 events = queries, |V| = 2^24), in the launch configuration
bench.py times: one tns_run with the dense outputs over the whole batch.  Every variant (recent,
uniform, windowed, the device-built store, and both policies on the prefix layout) is compared
with the oracle on EVERY query, in chunks of 2^24 so the host never holds the 32 GB padded
result; plus the size-independent invariants on two chunks."""
import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W
from conftest import progress

pytestmark = pytest.mark.gpu

CHUNK = 1 << 24


@pytest.fixture(scope="module")
def c5():
    import torch
    assert torch.cuda.is_available()
    import oracle
    from paper_2311_17410_amd import binding as B
    B.lib()
    progress("C5: generating the stream")
    wl = W.c5()
    st = wl.streams[0]
    progress("C5: ingesting 2^28 edges in 2^17-edge batches")
    plan = B.Plan(st.num_nodes, wl.fanout, block_threshold=wl.tau)
    for i, (lo, hi) in enumerate(st.batches()):
        B.tns_add_edges(plan.handle, 0, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
        if i % 512 == 511:
            progress(f"C5: {hi} edges ingested")
    plan.commit()
    progress("C5: building the oracle's per-node lists")
    adj = oracle.Adjacency(st.num_nodes, st.src, st.dst, st.ts)
    dev = torch.device("cuda", 0)
    d = dict(targets=torch.from_numpy(st.src).to(dev), t_end=torch.from_numpy(st.ts).to(dev))
    out = plan.alloc_outputs(st.n, compact=True)
    yield dict(wl=wl, st=st, plan=plan, adj=adj, d=d, out=out, oracle=oracle, B=B, torch=torch)
    adj.close()
    plan.close()


def _compare_chunk(c5, c, policy, t_start_np, seed, base_row):
    """Chunk c of the GPU result against the oracle; returns the dense offset after the chunk."""
    st, out, oracle, f = c5["st"], c5["out"], c5["oracle"], c5["wl"].fanout
    lo, hi = c * CHUNK, min((c + 1) * CHUNK, st.n)
    q_ids = np.arange(lo, hi, dtype=np.int64)
    tb = None if t_start_np is None else t_start_np[lo:hi]
    ref = c5["adj"].sample(st.src[lo:hi], tb, st.ts[lo:hi], f, policy=policy, seed=seed, q_ids=q_ids, threads=16)
    g = lambda name, a, b: out[name][a:b].cpu().numpy()
    assert np.array_equal(g("count", lo, hi), ref.count), f"count, chunk {c}"
    assert np.array_equal(g("eid", lo * f, hi * f).reshape(-1, f), ref.eid), f"eid, chunk {c}"
    assert np.array_equal(g("nbr", lo * f, hi * f).reshape(-1, f), ref.nbr), f"nbr, chunk {c}"
    assert np.array_equal(g("ts", lo * f, hi * f).reshape(-1, f).view(np.int32), ref.ts.view(np.int32)), f"ts, chunk {c}"
    rowptr, cn, ce, ct = oracle.compact(ref)
    if base_row is None:                    # sampled chunk: take the chunk's own base from the GPU rowptr
        base_row = int(out["rowptr"][lo].item())
    assert np.array_equal(g("rowptr", lo, hi + 1), rowptr + base_row), f"rowptr, chunk {c}"
    a, b = base_row, base_row + int(rowptr[-1])
    assert np.array_equal(g("cmp_eid", a, b), ce) and np.array_equal(g("cmp_nbr", a, b), cn), f"dense ids, chunk {c}"
    assert np.array_equal(g("cmp_ts", a, b).view(np.int32), ct.view(np.int32)), f"dense ts, chunk {c}"
    return b, ref


def _run(c5, t_start=None):
    c5["plan"].run(c5["d"]["targets"], t_start, c5["d"]["t_end"], out=c5["out"])
    c5["torch"].cuda.synchronize()
    # the fused kernel's bounded wait must not have run out
    assert not c5["plan"].status(c5["out"]["workspace"])


def test_c5_recent_every_query(c5):
    B, st = c5["B"], c5["st"]
    c5["plan"].set_sampler(c5["wl"].fanout, B.TNS_POLICY_RECENT, 0, 0)
    progress("C5 recent: GPU run over 2^28 queries")
    _run(c5)
    row = 0
    for c in range((st.n + CHUNK - 1) // CHUNK):
        row, ref = _compare_chunk(c5, c, 0, None, 0, row)
        if c in (0, 9):
            lo, hi = c * CHUNK, (c + 1) * CHUNK
            check_invariants_chunk(st, lo, hi, ref, c5["wl"].fanout)
        progress(f"C5 recent: chunk {c} matches")
    assert int(c5["out"]["rowptr"][st.n].item()) == row


def check_invariants_chunk(st, lo, hi, ref, f):
    """P6 on one chunk: every filled slot is an earlier edge of the target with the stored values,
    newest first; padding exact."""
    cnt = ref.count.astype(np.int64)
    filled = np.arange(f)[None, :] < cnt[:, None]
    e = ref.eid[filled].astype(np.int64)
    qq = (np.arange(lo, hi)[:, None] + np.zeros((1, f), np.int64))[filled]
    assert np.all(e < qq) and np.all(e >= 0)
    assert np.array_equal(st.src[e], st.src[qq]) and np.array_equal(st.dst[e], ref.nbr[filled])
    assert np.array_equal(st.ts[e], ref.ts[filled]) and np.all(st.ts[e] < st.ts[qq])
    d = np.diff(ref.eid.astype(np.int64), axis=1)
    assert np.all(d[filled[:, 1:]] < 0)
    assert np.all(ref.eid[~filled] == -1) and np.all(ref.nbr[~filled] == -1) and np.all(ref.ts[~filled] == 0)


def _compare_all(c5, label, policy, t_start_np, seed):
    st = c5["st"]
    row = 0
    for c in range((st.n + CHUNK - 1) // CHUNK):
        row, _ = _compare_chunk(c5, c, policy, t_start_np, seed, row)
        progress(f"{label}: chunk {c} matches")
    assert int(c5["out"]["rowptr"][st.n].item()) == row


def test_c5_uniform_every_query(c5):
    B = c5["B"]
    c5["plan"].set_sampler(c5["wl"].fanout, B.TNS_POLICY_UNIFORM, 0, 4)
    progress("C5 uniform: GPU run over 2^28 queries")
    _run(c5)
    _compare_all(c5, "C5 uniform", 1, None, 4)


def test_c5_windowed_every_query(c5):
    B, st, torch = c5["B"], c5["st"], c5["torch"]
    c5["plan"].set_sampler(c5["wl"].fanout, B.TNS_POLICY_RECENT, 0, 0)
    t_start = (st.ts - np.float32(0.25) * np.float32(st.ts[-1] - st.ts[0])).astype(np.float32)
    d_tb = torch.from_numpy(t_start).to(c5["d"]["t_end"].device)
    progress("C5 windowed: GPU run over 2^28 queries")
    _run(c5, d_tb)
    _compare_all(c5, "C5 windowed", 0, t_start, 0)


def test_c5_store_built_on_the_device(c5):
    """The same stream ingested on the GPU (tns_add_edges_device, 2^17-edge batches): same block
    statistics as the host builder, and the full-size run matches the oracle on every query."""
    B, st, torch, wl = c5["B"], c5["st"], c5["torch"], c5["wl"]
    dplan = B.Plan(st.num_nodes, wl.fanout, block_threshold=wl.tau, flags=B.TNS_FLAG_DEVICE_INGEST)
    d_dst = torch.from_numpy(st.dst).to(c5["d"]["t_end"].device)
    progress("C5 device-built: ingesting 2^28 edges on the GPU")
    for i, (lo, hi) in enumerate(st.batches()):
        dplan.add_edges_device(c5["d"]["targets"][lo:hi], d_dst[lo:hi], c5["d"]["t_end"][lo:hi])
        if i % 512 == 511:
            progress(f"C5 device-built: {hi} edges ingested")
    del d_dst
    hs, ds = c5["plan"].stats(), dplan.stats()
    for k in ("num_blocks", "num_edges", "wasted_slots", "max_list_len"):
        assert hs[k] == ds[k], k
    progress("C5 device-built: GPU run over 2^28 queries")
    dplan.run(c5["d"]["targets"], None, c5["d"]["t_end"], out=c5["out"])
    torch.cuda.synchronize()
    assert not dplan.status(c5["out"]["workspace"])
    _compare_all(c5, "C5 device-built", 0, None, 0)
    dplan.close()


def test_c5_prefix_layout_every_query(c5):
    """The same stream in the prefix layout (TNS_FLAG_PREFIX_LAYOUT): same block statistics as the default layout,
    and both policies match the oracle on every query of the full-size run."""
    B, st, torch, wl = c5["B"], c5["st"], c5["torch"], c5["wl"]
    pplan = B.Plan(st.num_nodes, wl.fanout, block_threshold=wl.tau, flags=B.TNS_FLAG_PREFIX_LAYOUT)
    progress("C5 prefix layout: ingesting 2^28 edges")
    for i, (lo, hi) in enumerate(st.batches()):
        B.tns_add_edges(pplan.handle, 0, st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], None)
        if i % 512 == 511:
            progress(f"C5 prefix layout: {hi} edges ingested")
    pplan.commit()
    hs, ps = c5["plan"].stats(), pplan.stats()
    for k in ("num_blocks", "num_edges", "wasted_slots", "max_list_len"):
        assert hs[k] == ps[k], k
    for label, policy, seed in (("C5 prefix recent", B.TNS_POLICY_RECENT, 0), ("C5 prefix uniform", B.TNS_POLICY_UNIFORM, 4)):
        pplan.set_sampler(wl.fanout, policy, 0, seed)
        progress(f"{label}: GPU run over 2^28 queries")
        pplan.run(c5["d"]["targets"], None, c5["d"]["t_end"], out=c5["out"])
        torch.cuda.synchronize()
        assert not pplan.status(c5["out"]["workspace"])
        _compare_all(c5, label, 1 if policy == B.TNS_POLICY_UNIFORM else 0, None, seed)
    pplan.close()
