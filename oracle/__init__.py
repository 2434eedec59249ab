"""TEST INFRASTRUCTURE: ctypes access to the plain-C CPU oracles.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It never imports the HIP package and the HIP package never
imports it.  Argument marshalling only; all arithmetic is in the two C files:

* ``tns_oracle.c``        layout-free definition of the sampling result (O1-O5)
* ``blockstore_oracle.c`` the paper's block store + Algorithm 1, step by step

``khop_oracle.py`` chains the one-hop oracle into the multi-hop sampling of section 4.2.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_BUILD = os.path.join(_HERE, "_build")
_SO = os.path.join(_BUILD, "liboracle.so")
_SRCS = [os.path.join(_HERE, "tns_oracle.c"), os.path.join(_HERE, "blockstore_oracle.c")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2 -fopenmp``); returns the library path."""
    os.makedirs(_BUILD, exist_ok=True)
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRCS)
    if stale:
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
                               "-o", tmp] + _SRCS + ["-lm"])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, i64p, f32p, u8p = (C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float),
                                 C.POINTER(C.c_uint8))
        L.oracle_adj_build.argtypes = [C.c_int64, C.c_int64, i32p, i32p, f32p, i32p, u8p, i64p, C.c_int64,
                                       C.POINTER(C.c_void_p)]
        L.oracle_adj_build.restype = C.c_int
        L.oracle_adj_free.argtypes = [C.c_void_p]
        L.oracle_adj_free.restype = None
        L.oracle_pick.argtypes = [C.c_uint64, C.c_int64, C.c_int32, C.c_int32, C.c_uint64]
        L.oracle_pick.restype = C.c_uint64
        L.oracle_threads_used.restype = C.c_int
        L.oracle_sample.argtypes = [C.c_void_p, C.c_int64, i32p, f32p, f32p, i64p, C.c_int32, C.c_int32,
                                    C.c_int32, C.c_uint64, i32p, i32p, f32p, i32p, C.c_int32]
        L.oracle_sample.restype = C.c_int
        L.oracle_compact.argtypes = [C.c_int64, C.c_int32, i32p, i32p, f32p, i32p, i64p, i32p, i32p, f32p]
        L.oracle_compact.restype = C.c_int
        L.bs_create.argtypes = [C.c_int64, C.c_int64, C.c_int]
        L.bs_create.restype = C.c_void_p
        L.bs_destroy.argtypes = [C.c_void_p]
        L.bs_destroy.restype = None
        L.bs_add_batch.argtypes = [C.c_void_p, C.c_int64, i32p, i32p, f32p, i32p]
        L.bs_add_batch.restype = C.c_int
        L.bs_delete_edge.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.bs_delete_edge.restype = C.c_int
        L.bs_sample.argtypes = [C.c_void_p, C.c_int64, i32p, f32p, f32p, i64p, C.c_int32, C.c_int32,
                                C.c_int32, C.c_uint64, i32p, i32p, f32p, i32p]
        L.bs_sample.restype = C.c_int
        L.bs_walk_counts.argtypes = [C.c_void_p, C.c_int64, i32p, f32p, f32p, C.c_int32, C.c_int32, C.c_int32, i64p]
        L.bs_walk_counts.restype = C.c_int
        L.bs_stats.argtypes = [C.c_void_p, C.POINTER(C.c_double), i64p, i64p, i64p, i64p, i64p]
        L.bs_stats.restype = C.c_int
        L.bs_export_blocks.argtypes = [C.c_void_p, i32p, i64p, i64p, f32p, f32p]
        L.bs_export_blocks.restype = C.c_int64
        L.bs_export_node.argtypes = [C.c_void_p, C.c_int32, C.c_int64, i32p, i32p, f32p]
        L.bs_export_node.restype = C.c_int64
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        names = {-1: "EINVAL", -2: "EORDER", -3: "ERANGE", -4: "ENOMEM"}
        super().__init__(f"{where}: {names.get(code, code)}")
        self.code = code


def _p(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ct))


def _arr(a, dtype):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


class Sampled:
    """Padded result (O4) of a query batch."""

    def __init__(self, q: int, f: int):
        self.nbr = np.empty((q, f), dtype=np.int32)
        self.eid = np.empty((q, f), dtype=np.int32)
        self.ts = np.empty((q, f), dtype=np.float32)
        self.count = np.empty(q, dtype=np.int32)


def pick(seed: int, q: int, f: int, j: int, c: int) -> int:
    return int(lib().oracle_pick(seed, q, f, j, c))


def compact(s: Sampled):
    """O5: (rowptr int64[Q+1], nbr, eid, ts) with the padding removed."""
    q, f = s.nbr.shape
    rowptr = np.empty(q + 1, dtype=np.int64)
    total = int(np.sum(s.count, dtype=np.int64))
    cn = np.empty(total, dtype=np.int32)
    ce = np.empty(total, dtype=np.int32)
    ct = np.empty(total, dtype=np.float32)
    rc = lib().oracle_compact(q, f, _p(s.nbr, C.c_int32), _p(s.eid, C.c_int32), _p(s.ts, C.c_float),
                              _p(s.count, C.c_int32), _p(rowptr, C.c_int64), _p(cn, C.c_int32),
                              _p(ce, C.c_int32), _p(ct, C.c_float))
    if rc:
        raise OracleError(rc, "oracle_compact")
    return rowptr, cn, ce, ct


class Adjacency:
    """O1: per-node chronological edge lists of one graph instance."""

    def __init__(self, num_nodes, src, dst, ts, eid=None, present=None, batch_rowptr=None):
        src, dst, ts = _arr(src, np.int32), _arr(dst, np.int32), _arr(ts, np.float32)
        eid, present = _arr(eid, np.int32), _arr(present, np.uint8)
        brp = _arr(batch_rowptr, np.int64)
        h = C.c_void_p()
        rc = lib().oracle_adj_build(num_nodes, src.shape[0], _p(src, C.c_int32), _p(dst, C.c_int32),
                                    _p(ts, C.c_float), _p(eid, C.c_int32), _p(present, C.c_uint8),
                                    _p(brp, C.c_int64), 0 if brp is None else brp.shape[0] - 1, C.byref(h))
        if rc:
            raise OracleError(rc, "oracle_adj_build")
        self._h = h
        self.num_nodes = num_nodes

    def sample(self, targets, t_start, t_end, fanout, policy=0, inclusive_end=0, seed=0, q_ids=None,
               threads=1) -> Sampled:
        targets, t_start, t_end = _arr(targets, np.int32), _arr(t_start, np.float32), _arr(t_end, np.float32)
        q_ids = _arr(q_ids, np.int64)
        q = targets.shape[0]
        out = Sampled(q, fanout)
        rc = lib().oracle_sample(self._h, q, _p(targets, C.c_int32), _p(t_start, C.c_float),
                                 _p(t_end, C.c_float), _p(q_ids, C.c_int64), fanout, policy, inclusive_end,
                                 seed, _p(out.nbr, C.c_int32), _p(out.eid, C.c_int32), _p(out.ts, C.c_float),
                                 _p(out.count, C.c_int32), threads)
        if rc:
            raise OracleError(rc, "oracle_sample")
        self.threads_used = int(lib().oracle_threads_used())
        return out

    def close(self):
        if self._h:
            lib().oracle_adj_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class BlockStore:
    """Structural oracle: the paper's block store and Algorithm 1 walked over it."""
    ADAPTIVE, STRAWMAN, FIXED = 0, 1, 2

    def __init__(self, num_nodes, tau, sizing=0):
        self._h = lib().bs_create(num_nodes, tau, sizing)
        if not self._h:
            raise OracleError(-1, "bs_create")
        self.num_nodes = num_nodes

    def add_batch(self, src, dst, ts, eid=None):
        src, dst, ts, eid = _arr(src, np.int32), _arr(dst, np.int32), _arr(ts, np.float32), _arr(eid, np.int32)
        rc = lib().bs_add_batch(self._h, src.shape[0], _p(src, C.c_int32), _p(dst, C.c_int32),
                                _p(ts, C.c_float), _p(eid, C.c_int32))
        if rc:
            raise OracleError(rc, "bs_add_batch")

    def add_stream(self, src, dst, ts, batch):
        n = len(src)
        for lo in range(0, n, batch):
            self.add_batch(src[lo:lo + batch], dst[lo:lo + batch], ts[lo:lo + batch])

    def delete_edge(self, node, eid) -> int:
        return int(lib().bs_delete_edge(self._h, node, eid))

    def sample(self, targets, t_start, t_end, fanout, policy=0, inclusive_end=0, seed=0, q_ids=None) -> Sampled:
        targets, t_start, t_end = _arr(targets, np.int32), _arr(t_start, np.float32), _arr(t_end, np.float32)
        q_ids = _arr(q_ids, np.int64)
        q = targets.shape[0]
        out = Sampled(q, fanout)
        rc = lib().bs_sample(self._h, q, _p(targets, C.c_int32), _p(t_start, C.c_float), _p(t_end, C.c_float),
                             _p(q_ids, C.c_int64), fanout, policy, inclusive_end, seed,
                             _p(out.nbr, C.c_int32), _p(out.eid, C.c_int32), _p(out.ts, C.c_float),
                             _p(out.count, C.c_int32))
        if rc:
            raise OracleError(rc, "bs_sample")
        return out

    def walk_counts(self, targets, t_start, t_end, fanout, policy=0, inclusive_end=0) -> dict:
        """What Algorithm 1's walk touches over a batch: node entries, block metadata records, timestamps compared
        by the bound searches, edges selected (the per-query quantities of a byte model, summed)."""
        targets, t_start, t_end = _arr(targets, np.int32), _arr(t_start, np.float32), _arr(t_end, np.float32)
        tot = np.zeros(4, np.int64)
        rc = lib().bs_walk_counts(self._h, targets.shape[0], _p(targets, C.c_int32), _p(t_start, C.c_float),
                                  _p(t_end, C.c_float), fanout, policy, inclusive_end, _p(tot, C.c_int64))
        if rc:
            raise OracleError(rc, "bs_walk_counts")
        return dict(nodes=int(tot[0]), blocks=int(tot[1]), probes=int(tot[2]), edges=int(tot[3]))

    def stats(self) -> dict:
        avg = C.c_double()
        v = [C.c_int64() for _ in range(5)]
        lib().bs_stats(self._h, C.byref(avg), *[C.byref(x) for x in v])
        return dict(avg_list_len=avg.value, max_list_len=v[0].value, num_blocks=v[1].value,
                    edge_slots=v[2].value, edges=v[3].value, wasted_slots=v[4].value)

    def blocks(self):
        nb = self.stats()["num_blocks"]
        node = np.empty(nb, np.int32)
        cap = np.empty(nb, np.int64)
        size = np.empty(nb, np.int64)
        tmin = np.empty(nb, np.float32)
        tmax = np.empty(nb, np.float32)
        w = lib().bs_export_blocks(self._h, _p(node, C.c_int32), _p(cap, C.c_int64), _p(size, C.c_int64),
                                   _p(tmin, C.c_float), _p(tmax, C.c_float))
        assert w == nb
        return dict(node=node, cap=cap, size=size, t_min=tmin, t_max=tmax)

    def node_edges(self, v, max_edges):
        nbr = np.empty(max_edges, np.int32)
        eid = np.empty(max_edges, np.int32)
        ts = np.empty(max_edges, np.float32)
        w = lib().bs_export_node(self._h, v, max_edges, _p(nbr, C.c_int32), _p(eid, C.c_int32), _p(ts, C.c_float))
        return nbr[:w], eid[:w], ts[:w]

    def close(self):
        if self._h:
            lib().bs_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
