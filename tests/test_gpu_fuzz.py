"""Seeded differential test: random small configurations (stream shape, tau, sizing method, ingestion
batching, host or device builder, fan-out, policy, window convention, deletions, several instances) through
the HIP library and through the CPU oracle; every output array must match bit for bit."""
import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W
from _harness import assert_same, gpu_sample

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2311_17410_amd import binding
    binding.lib()
    return binding


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    num_nodes = int(rng.choice([1, 2, 7, 40, 300]))
    n = int(rng.integers(1, 4000))
    ties = bool(rng.integers(0, 2))
    src = (rng.zipf(1.3, n) % num_nodes).astype(np.int32) if rng.integers(0, 2) else rng.integers(0, num_nodes, n, dtype=np.int32)
    dst = rng.integers(0, num_nodes, n, dtype=np.int32)
    ts = (np.sort(rng.integers(0, max(n // 4, 2), n)).astype(np.float32) if ties
          else np.sort(rng.standard_normal(n)).astype(np.float32))
    return dict(rng=rng, num_nodes=num_nodes, n=n, src=src, dst=dst, ts=ts,
                tau=int(rng.choice([1, 3, 16, 48, 1000])), sizing=int(rng.integers(0, 3)),
                batch=int(rng.choice([1, 5, 64, 1000, 5000])), f=int(rng.choice([1, 2, 5, 10, 11, 16, 17, 33, 64])),
                policy=int(rng.integers(0, 2)), incl=int(rng.integers(0, 2)), device_built=bool(rng.integers(0, 2)),
                delete=bool(rng.integers(0, 3) == 0), wide=bool(rng.integers(0, 4) == 0), seed=int(rng.integers(0, 1 << 30)))


@pytest.mark.parametrize("seed", range(160))
def test_random_configuration(B, oracle_lib, seed, layout):
    import torch
    c = _case(seed)
    if layout and c["device_built"]:
        pytest.skip("the device builder writes the default layout")
    rng, n = c["rng"], c["n"]
    if c["batch"] == 1 and n > 600:          # one edge per batch: keep the number of ingestion calls small
        n = 600
        c["src"], c["dst"], c["ts"] = c["src"][:n], c["dst"][:n], c["ts"][:n]
    flags = (B.TNS_FLAG_DEVICE_INGEST if c["device_built"] else 0) | (B.TNS_FLAG_WIDE_POSITIONS if c["wide"] else 0) | layout
    plan = B.Plan(c["num_nodes"], c["f"], policy=c["policy"], block_threshold=c["tau"], sizing=c["sizing"],
                  inclusive_end=c["incl"], seed=c["seed"], flags=flags)
    bounds = list(range(0, n, c["batch"])) + [n]
    if c["device_built"]:
        d = [torch.from_numpy(a).cuda() for a in (c["src"], c["dst"], c["ts"])]
        for lo, hi in zip(bounds[:-1], bounds[1:]):
            plan.add_edges_device(d[0][lo:hi], d[1][lo:hi], d[2][lo:hi])
    else:
        for lo, hi in zip(bounds[:-1], bounds[1:]):
            plan.add_edges(c["src"][lo:hi], c["dst"][lo:hi], c["ts"][lo:hi])
        plan.commit()
    present = None
    if c["delete"]:
        present = np.ones(n, np.uint8)
        victims = rng.choice(n, max(n // 4, 1), replace=False).astype(np.int32)
        present[victims] = 0
        assert B.tns_delete_edges(plan.handle, 0, c["src"][victims], victims) == len(victims)
        if not c["device_built"]:
            plan.commit()
    st = W.Stream(c["num_nodes"], c["src"], c["dst"], c["ts"], c["batch"])
    targets, t_start, t_end = W.random_queries(seed, st, int(rng.integers(1, 3000)))
    adj = oracle_lib.Adjacency(c["num_nodes"], c["src"], c["dst"], c["ts"], present=present, batch_rowptr=bounds)
    for tb in (t_start, None):
        ref = adj.sample(targets, tb, t_end, c["f"], policy=c["policy"], inclusive_end=c["incl"], seed=c["seed"])
        got = gpu_sample(plan, targets, tb, t_end)
        assert_same(got, ref, oracle_lib, f"seed {seed}: { {k: v for k, v in c.items() if k not in ('rng', 'src', 'dst', 'ts')} }")
    adj.close()
    plan.close()
