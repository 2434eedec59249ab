"""Seeded synthetic edge streams and query batches.

This module serves both the CPU oracle's tests and the HIP path's tests/bench.  It
contains no sampling arithmetic: it only draws random numbers, sorts timestamps and
slices arrays.  The paper evaluates on Reddit, Netflix, GDELT, MAG and LDBC (section 6,
"Datasets"); none of them is available here, so the streams below borrow only their shape
facts: 10-11k edges per node down to ~10, power-law degrees (section 4.1), ingestion
batches of ~100k edges (section 6.2), fan-out 10 (section 6, "Models").

A stream is an edge list in arrival order: ``src[i] -> dst[i]`` at time ``ts[i]`` with
edge id ``i``; ``ts`` is globally non-decreasing, so every node's edges arrive in
chronological order as the paper's storage assumes (section 4.1).  The query batch of a
stream is one epoch of link-prediction sampling over it: query ``i`` asks for the temporal
neighbours of ``src[i]`` before ``ts[i]``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


@dataclass
class Stream:
    """One dynamic graph instance: edges in arrival order plus its ingestion batching."""
    num_nodes: int
    src: np.ndarray          # int32 [n]
    dst: np.ndarray          # int32 [n]
    ts: np.ndarray           # float32 [n], non-decreasing
    batch: int               # edges per ingestion batch (last one may be short)

    @property
    def n(self) -> int:
        return int(self.src.shape[0])

    def batches(self):
        for lo in range(0, self.n, self.batch):
            hi = min(lo + self.batch, self.n)
            yield lo, hi


@dataclass
class Workload:
    """A named configuration: one or more independent streams and the sampler settings."""
    name: str
    seed: int
    streams: List[Stream]
    fanout: int = 10
    tau: int = 48
    description: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def num_instances(self) -> int:
        return len(self.streams)

    @property
    def num_nodes(self) -> int:
        return self.streams[0].num_nodes

    @property
    def total_edges(self) -> int:
        return sum(s.n for s in self.streams)

    def queries(self, window_frac: Optional[float] = None):
        """Concatenated query arrays over all instances, in stream order.

        Returns ``(targets int32[Q], t_start float32[Q] or None, t_end float32[Q],
        inst_rowptr int64[I+1])``.  ``window_frac`` turns on the windowed variant
        ``t_start = t_end - window_frac * span`` (span = last - first timestamp of the
        instance).
        """
        targets = np.concatenate([s.src for s in self.streams]) if len(self.streams) > 1 else self.streams[0].src
        t_end = np.concatenate([s.ts for s in self.streams]) if len(self.streams) > 1 else self.streams[0].ts
        rowptr = np.zeros(len(self.streams) + 1, dtype=np.int64)
        np.cumsum([s.n for s in self.streams], out=rowptr[1:])
        t_start = None
        if window_frac is not None:
            parts = []
            for s in self.streams:
                span = np.float32(s.ts[-1] - s.ts[0]) if s.n else np.float32(0)
                parts.append((s.ts - np.float32(window_frac) * span).astype(np.float32))
            t_start = np.concatenate(parts) if len(parts) > 1 else parts[0]
        return targets, t_start, t_end, rowptr


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _sorted_times(rng: np.random.Generator, n: int, dist: str) -> np.ndarray:
    if dist == "uniform":
        v = rng.random(n, dtype=np.float32)
    elif dist == "normal":
        v = rng.standard_normal(n, dtype=np.float32)
    else:
        raise ValueError(dist)
    v.sort()          # values only: any sorting algorithm gives the same array
    return v


def uniform_stream(rng: np.random.Generator, n: int, num_nodes: int, batch: int,
                   ts_dist: str = "uniform") -> Stream:
    """Draw order is fixed: src, dst, timestamp values."""
    src = rng.integers(0, num_nodes, n, dtype=np.int32)
    dst = rng.integers(0, num_nodes, n, dtype=np.int32)
    ts = _sorted_times(rng, n, ts_dist)
    return Stream(num_nodes, src, dst, ts, batch)


def zipf_stream(rng: np.random.Generator, n: int, num_nodes: int, batch: int,
                s: float = 1.1, ts_dist: str = "normal") -> Stream:
    """Node ranks follow Zipf(s) over 1..num_nodes (inverse CDF on the cumulative k^-s);
    rank r maps to a node id through a seeded permutation so hubs are not the low ids."""
    w = np.arange(1, num_nodes + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    perm = rng.permutation(num_nodes).astype(np.int32)

    def draw():
        u = rng.random(n)
        r = np.searchsorted(cdf, u, side="left")
        np.minimum(r, num_nodes - 1, out=r)
        return perm[r]

    src = draw()
    dst = draw()
    ts = _sorted_times(rng, n, ts_dist)
    return Stream(num_nodes, src, dst, ts, batch)


# ---- the five configurations -------------------------------------------------------

def c1() -> Workload:
    rng = _rng(0)
    return Workload("C1", 0, [uniform_stream(rng, 1 << 10, 1 << 6, 1 << 7)], tau=48,
                    description="n=2^10, |V|=2^6, uniform ids, U[0,1) times")


def c2() -> Workload:
    rng = _rng(1)
    return Workload("C2", 1, [uniform_stream(rng, 1 << 20, 1 << 16, 1 << 17)], tau=48,
                    description="n=2^20, |V|=2^16, uniform ids, U[0,1) times")


def c3(log2_n: int = 24) -> Workload:
    rng = _rng(2)
    n = 1 << log2_n
    v = max(n >> 4, 2)
    return Workload("C3", 2, [zipf_stream(rng, n, v, 1 << 17, 1.1, "normal")], tau=8192,
                    description=f"n=2^{log2_n}, |V|=n/16, Zipf(1.1) ids, N(0,1) times")


def c4(instances: int = 256, log2_n: int = 16) -> Workload:
    rng = _rng(3)
    n = 1 << log2_n
    streams = [uniform_stream(rng, n, max(n >> 4, 2), max(n >> 3, 1), "normal") for _ in range(instances)]
    return Workload("C4", 3, streams, tau=48,
                    description=f"{instances} instances of n=2^{log2_n}, |V|=n/16, N(0,1) times")


def c5(log2_n: int = 28) -> Workload:
    rng = _rng(4)
    n = 1 << log2_n
    return Workload("C5", 4, [uniform_stream(rng, n, max(n >> 4, 2), 1 << 17)], tau=48,
                    description=f"n=2^{log2_n}, |V|=n/16, uniform ids, U[0,1) times")


def literal_range(cfg: str) -> Workload:
    """Side runs with node ids drawn over [0, n) as the generic config text says
    (mean out-degree 1): C1 and C2 only."""
    if cfg == "C1":
        rng = _rng(0)
        return Workload("C1-literal", 0, [uniform_stream(rng, 1 << 10, 1 << 10, 1 << 7)], tau=48)
    if cfg == "C2":
        rng = _rng(1)
        return Workload("C2-literal", 1, [uniform_stream(rng, 1 << 20, 1 << 20, 1 << 17)], tau=48)
    raise ValueError(cfg)


def by_name(name: str, **kw) -> Workload:
    table = {"C1": c1, "C2": c2, "C3": c3, "C4": c4, "C5": c5}
    return table[name.upper()](**kw)


# ---- small random cases for brute-force and edge-case tests --------------------------

def tiny_stream(seed: int, n: int, num_nodes: int, batch: int, ties: bool = True) -> Stream:
    """Small stream with many equal timestamps when ``ties`` is set (integer-valued times
    drawn from a narrow range), to exercise the tie rules."""
    rng = _rng(seed)
    src = rng.integers(0, num_nodes, n, dtype=np.int32)
    dst = rng.integers(0, num_nodes, n, dtype=np.int32)
    if ties:
        ts = np.sort(rng.integers(0, max(n // 3, 2), n)).astype(np.float32)
    else:
        ts = _sorted_times(rng, n, "uniform")
    return Stream(num_nodes, src, dst, ts, batch)


def random_queries(seed: int, stream: Stream, q: int, with_start: bool = True):
    """Arbitrary (not stream-derived) queries: random targets including a few out-of-range
    ids, end times spread around the stream's time span, optional start times."""
    rng = _rng(seed)
    targets = rng.integers(-2, stream.num_nodes + 2, q, dtype=np.int32)
    lo = float(stream.ts[0]) if stream.n else 0.0
    hi = float(stream.ts[-1]) if stream.n else 1.0
    pad = 0.1 * (hi - lo) + 1.0
    if stream.n and np.all(stream.ts == np.round(stream.ts)):
        t_end = rng.integers(int(lo) - 1, int(hi) + 3, q).astype(np.float32)
        width = rng.integers(0, int(hi - lo) + 3, q).astype(np.float32)
    else:
        t_end = (lo - pad + (hi - lo + 2 * pad) * rng.random(q)).astype(np.float32)
        width = ((hi - lo + pad) * rng.random(q)).astype(np.float32)
    t_start = (t_end - width).astype(np.float32) if with_start else None
    return targets, t_start, t_end
