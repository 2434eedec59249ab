"""ctypes binding of include/tns_cache.h (vectorised feature cache): same names, marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .binding import TnsError, _check, lib as _lib

TNS_CACHE_LRU, TNS_CACHE_LFU, TNS_CACHE_FIFO = 0, 1, 2
EXPORTS = ["tns_cache_create", "tns_cache_workspace", "tns_cache_fetch", "tns_cache_stats", "tns_cache_save",
           "tns_cache_restore", "tns_cache_destroy"]


class tns_cache_config(C.Structure):
    _fields_ = [("num_ids", C.c_int64), ("capacity", C.c_int64), ("dim", C.c_int32), ("policy", C.c_int32),
                ("lambda_", C.c_float), ("device", C.c_int32)]


_ready = False


def lib():
    global _ready
    L = _lib()
    if not _ready:
        vp, i32p, i64p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float)
        L.tns_cache_create.argtypes = [C.POINTER(tns_cache_config), C.POINTER(vp)]
        L.tns_cache_workspace.argtypes = [vp, C.c_int64, C.POINTER(C.c_size_t)]
        L.tns_cache_fetch.argtypes = [vp, C.c_int64, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.tns_cache_stats.argtypes = [vp, vp, i64p, i64p, i64p]
        L.tns_cache_save.argtypes = [vp, vp, i32p, i32p, f32p, i64p]
        L.tns_cache_restore.argtypes = [vp, vp, i32p, i32p, f32p, C.c_int64]
        L.tns_cache_destroy.argtypes = [vp]
        for n in EXPORTS:
            getattr(L, n).restype = C.c_int
        _ready = True
    return L


def tns_cache_create(num_ids: int, capacity: int, dim: int, policy: int = TNS_CACHE_LRU, lam: float = 0.2, device: int = 0):
    cfg = tns_cache_config(num_ids, capacity, dim, policy, lam, device)
    h = C.c_void_p()
    _check(lib().tns_cache_create(C.byref(cfg), C.byref(h)), "tns_cache_create")
    return h


def tns_cache_workspace(cache, B: int) -> int:
    n = C.c_size_t()
    _check(lib().tns_cache_workspace(cache, B, C.byref(n)), "tns_cache_workspace")
    return int(n.value)


def tns_cache_fetch(cache, B: int, d_ids: int, store: int, d_out: int, d_hit: int, d_workspace: int, workspace_bytes: int,
                    hip_stream: int = 0) -> None:
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_cache_fetch(cache, B, vp(d_ids), vp(store), vp(d_out), vp(d_hit), vp(d_workspace), workspace_bytes,
                                 vp(hip_stream)), "tns_cache_fetch")


def tns_cache_stats(cache, hip_stream: int = 0):
    v = [C.c_int64() for _ in range(3)]
    _check(lib().tns_cache_stats(cache, C.c_void_p(hip_stream or None), *[C.byref(x) for x in v]), "tns_cache_stats")
    return dict(hits=v[0].value, misses=v[1].value, replaced=v[2].value)


def tns_cache_save(cache, capacity: int, dim: int, hip_stream: int = 0):
    id_of = np.empty(capacity, np.int32)
    score = np.empty(capacity, np.int32)
    rows = np.empty((capacity, dim), np.float32)
    ring = C.c_int64()
    _check(lib().tns_cache_save(cache, C.c_void_p(hip_stream or None), id_of.ctypes.data_as(C.POINTER(C.c_int32)),
                                score.ctypes.data_as(C.POINTER(C.c_int32)), rows.ctypes.data_as(C.POINTER(C.c_float)),
                                C.byref(ring)), "tns_cache_save")
    return dict(id_of=id_of, score=score, rows=rows, ring=int(ring.value))


def tns_cache_restore(cache, saved: dict, hip_stream: int = 0) -> None:
    id_of = np.ascontiguousarray(saved["id_of"], np.int32)
    score = np.ascontiguousarray(saved["score"], np.int32)
    rows = np.ascontiguousarray(saved["rows"], np.float32)
    _check(lib().tns_cache_restore(cache, C.c_void_p(hip_stream or None), id_of.ctypes.data_as(C.POINTER(C.c_int32)),
                                   score.ctypes.data_as(C.POINTER(C.c_int32)), rows.ctypes.data_as(C.POINTER(C.c_float)),
                                   saved["ring"]), "tns_cache_restore")


def tns_cache_destroy(cache) -> None:
    _check(lib().tns_cache_destroy(cache), "tns_cache_destroy")


class Cache:
    """Owns a tns_cache; ``fetch`` allocates the output with torch and uses the current stream."""

    def __init__(self, num_ids, capacity, dim, policy=TNS_CACHE_LRU, lam=0.2, device=0):
        self.num_ids, self.capacity, self.dim, self.device = num_ids, capacity, dim, device
        self._h = tns_cache_create(num_ids, capacity, dim, policy, lam, device)
        self._ws = None

    def fetch(self, d_ids, d_store, out=None, hit=None):
        import torch
        B = int(d_ids.shape[0])
        dev = torch.device("cuda", self.device)
        if out is None:
            out = torch.empty((B, self.dim), dtype=torch.float32, device=dev)
        if hit is None:
            hit = torch.empty(B, dtype=torch.uint8, device=dev)
        need = tns_cache_workspace(self._h, B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=dev)
        with torch.cuda.device(self.device):
            tns_cache_fetch(self._h, B, d_ids.data_ptr(), d_store.data_ptr(), out.data_ptr(), hit.data_ptr(),
                            self._ws.data_ptr(), self._ws.numel(), torch.cuda.current_stream().cuda_stream)
        return out, hit

    def stats(self):
        return tns_cache_stats(self._h)

    def save(self):
        return tns_cache_save(self._h, self.capacity, self.dim)

    def restore(self, saved):
        tns_cache_restore(self._h, saved)

    def close(self):
        if getattr(self, "_h", None):
            tns_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
