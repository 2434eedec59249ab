"""Thin ctypes binding of the C ABI in include/tns.h: same names, argument marshalling only.

Every step of the sampling path runs in the HIP library; there is no Python or CPU
fallback.  If the library has not been built, importing the functions raises.
PyTorch is used by the convenience class only to own device memory and streams.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtns.so")

TNS_OK, TNS_EINVAL, TNS_EORDER, TNS_ERANGE, TNS_ENOMEM, TNS_EHIP, TNS_ESTATE, TNS_ESIZE = 0, -1, -2, -3, -4, -5, -6, -7
TNS_POLICY_RECENT, TNS_POLICY_UNIFORM = 0, 1
TNS_SIZING_ADAPTIVE, TNS_SIZING_STRAWMAN, TNS_SIZING_FIXED = 0, 1, 2
TNS_MAX_FANOUT = 64
TNS_FLAG_NO_XCD_REMAP = 1
TNS_FLAG_NO_NODE_SLAB = 2
TNS_FLAG_EDGES_ON_HOST = 4
TNS_FLAG_ALL_ON_HOST = 8
TNS_FLAG_DEVICE_INGEST = 16
TNS_FLAG_WIDE_POSITIONS = 32
TNS_FLAG_PREFIX_LAYOUT = 128
TNS_TEST_FLAG_LOST_TILE = 64      # csrc/tns_test_hooks.h: for the library's own tests, not in the public header

EXPORTS = ["tns_plan_create", "tns_set_sampler", "tns_add_edges", "tns_add_edges_device", "tns_delete_edges", "tns_delete_nodes", "tns_commit", "tns_workspace", "tns_run", "tns_run_status", "tns_run_static", "tns_hbm_probe_mix", "tns_workspace_khop", "tns_run_khop", "tns_compact", "tns_traffic_model", "tns_stats",
           "tns_node_blocks", "tns_hbm_probe", "tns_destroy", "tns_strerror", "tns_last_error"]


class tns_config(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_instances", C.c_int32), ("fanout", C.c_int32),
                ("policy", C.c_int32), ("block_threshold", C.c_int32), ("sizing", C.c_int32),
                ("inclusive_end", C.c_int32), ("seed", C.c_uint64), ("device", C.c_int32), ("flags", C.c_int32)]


class tns_stats_t(C.Structure):
    _fields_ = [("avg_list_len", C.c_double), ("max_list_len", C.c_int64), ("edge_data_bytes", C.c_int64),
                ("metadata_bytes", C.c_int64), ("wasted_slots", C.c_int64), ("num_blocks", C.c_int64),
                ("num_edges", C.c_int64)]


class tns_hop_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("nbr", "eid", "ts", "count", "rowptr", "cmp_nbr", "cmp_eid", "cmp_ts")]


class TnsError(RuntimeError):
    def __init__(self, status: int, where: str):
        L = lib()
        detail = L.tns_last_error().decode()
        super().__init__(f"{where}: {L.tns_strerror(status).decode()} ({status})" + (f": {detail}" if detail else ""))
        self.status = status


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no fallback path)")
        # One HIP runtime per process: PyTorch ships its own copy, and whichever copy is loaded first is the
        # one both sides must use.  Loading torch first keeps the library on the runtime that owns the
        # tensors and streams it is handed (without torch the library uses the system's runtime).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp, i32p, i64p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float)
        L.tns_plan_create.argtypes = [C.POINTER(tns_config), C.POINTER(vp)]
        L.tns_plan_create.restype = C.c_int
        L.tns_set_sampler.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_uint64]
        L.tns_set_sampler.restype = C.c_int
        L.tns_add_edges.argtypes = [vp, C.c_int32, i32p, i32p, f32p, i32p, C.c_int64]
        L.tns_add_edges.restype = C.c_int
        L.tns_add_edges_device.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_int64, vp]
        L.tns_add_edges_device.restype = C.c_int
        L.tns_delete_edges.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int64, i64p]
        L.tns_delete_edges.restype = C.c_int
        L.tns_delete_nodes.argtypes = [vp, C.c_int32, i32p, C.c_int64, C.c_int32]
        L.tns_delete_nodes.restype = C.c_int
        L.tns_commit.argtypes = [vp, vp]
        L.tns_commit.restype = C.c_int
        L.tns_workspace.argtypes = [vp, C.c_int64, C.POINTER(C.c_size_t)]
        L.tns_workspace.restype = C.c_int
        L.tns_run.argtypes = [vp, C.c_int64, vp, vp, vp, vp, C.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                              C.c_size_t, vp]
        L.tns_run.restype = C.c_int
        L.tns_run_status.argtypes = [vp, vp, vp, C.POINTER(C.c_int32)]
        L.tns_run_status.restype = C.c_int
        L.tns_run_static.argtypes = [vp, C.c_int64, vp, vp, vp, vp, C.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.tns_run_static.restype = C.c_int
        L.tns_workspace_khop.argtypes = [vp, C.c_int32, i32p, C.c_int64, C.POINTER(C.c_size_t)]
        L.tns_workspace_khop.restype = C.c_int
        L.tns_run_khop.argtypes = [vp, C.c_int32, i32p, C.c_float, C.c_int64, vp, vp, vp, vp, C.c_int64,
                                   C.POINTER(tns_hop_buffers), vp, C.c_size_t, vp]
        L.tns_run_khop.restype = C.c_int
        L.tns_compact.argtypes = [vp, C.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.tns_compact.restype = C.c_int
        L.tns_traffic_model.argtypes = [vp, C.c_int64, vp, vp, vp, vp, C.c_int64, vp, vp]
        L.tns_traffic_model.restype = C.c_int
        L.tns_stats.argtypes = [vp, C.c_int32, C.POINTER(tns_stats_t)]
        L.tns_stats.restype = C.c_int
        L.tns_node_blocks.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, i32p, i32p, f32p, f32p]
        L.tns_node_blocks.restype = C.c_int64
        L.tns_hbm_probe.argtypes = [C.c_int32, C.c_int32, vp, vp, C.c_size_t, vp]
        L.tns_hbm_probe.restype = C.c_int
        L.tns_hbm_probe_mix.argtypes = [C.c_int32, vp, C.c_size_t, vp, C.c_size_t, vp]
        L.tns_hbm_probe_mix.restype = C.c_int
        L.tns_destroy.argtypes = [vp]
        L.tns_destroy.restype = C.c_int
        L.tns_strerror.argtypes = [C.c_int]
        L.tns_strerror.restype = C.c_char_p
        L.tns_last_error.argtypes = []
        L.tns_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != TNS_OK:
        raise TnsError(status, where)


def _np(a, dtype):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=dtype)
    return arr, arr.ctypes.data_as(C.POINTER(np.ctypeslib.as_ctypes_type(dtype)))


# ---- the C ABI, one Python function per entry point -------------------------------------

def tns_plan_create(num_nodes: int, fanout: int, policy: int = TNS_POLICY_RECENT, block_threshold: int = 48,
                    num_instances: int = 1, sizing: int = TNS_SIZING_ADAPTIVE, inclusive_end: int = 0,
                    seed: int = 0, device: int = 0, flags: int = 0) -> C.c_void_p:
    cfg = tns_config(num_nodes, num_instances, fanout, policy, block_threshold, sizing, inclusive_end, seed,
                     device, flags)
    h = C.c_void_p()
    _check(lib().tns_plan_create(C.byref(cfg), C.byref(h)), "tns_plan_create")
    return h


def tns_set_sampler(plan, fanout: int, policy: int = TNS_POLICY_RECENT, inclusive_end: int = 0, seed: int = 0) -> None:
    _check(lib().tns_set_sampler(plan, fanout, policy, inclusive_end, seed), "tns_set_sampler")


def tns_add_edges(plan, instance: int, src, dst, ts, eid=None) -> None:
    src_a, src_p = _np(src, np.int32)
    dst_a, dst_p = _np(dst, np.int32)
    ts_a, ts_p = _np(ts, np.float32)
    eid_a, eid_p = _np(eid, np.int32)
    if not (len(src_a) == len(dst_a) == len(ts_a)) or (eid_a is not None and len(eid_a) != len(src_a)):
        raise ValueError("src, dst, ts (and eid) must have the same length")
    _check(lib().tns_add_edges(plan, instance, src_p, dst_p, ts_p, eid_p, len(src_a)), "tns_add_edges")


def tns_add_edges_device(plan, instance: int, d_src: int, d_dst: int, d_ts: int, d_eid: Optional[int], m: int,
                         stream: int) -> None:
    """Raw device pointers (ints) of the batch arrays; d_eid may be None."""
    _check(lib().tns_add_edges_device(plan, instance, d_src, d_dst, d_ts, d_eid, m, stream), "tns_add_edges_device")


def tns_delete_edges(plan, instance: int, src, eid) -> int:
    src_a, src_p = _np(src, np.int32)
    eid_a, eid_p = _np(eid, np.int32)
    if len(src_a) != len(eid_a):
        raise ValueError("src and eid must have the same length")
    n = C.c_int64()
    _check(lib().tns_delete_edges(plan, instance, src_p, eid_p, len(src_a), C.byref(n)), "tns_delete_edges")
    return int(n.value)


def tns_delete_nodes(plan, instance: int, nodes, deleted: bool = True) -> None:
    a, p = _np(nodes, np.int32)
    _check(lib().tns_delete_nodes(plan, instance, p, len(a), 1 if deleted else 0), "tns_delete_nodes")


def tns_commit(plan, hip_stream: int = 0) -> None:
    _check(lib().tns_commit(plan, C.c_void_p(hip_stream)), "tns_commit")


def tns_workspace(plan, Q: int) -> int:
    n = C.c_size_t()
    _check(lib().tns_workspace(plan, Q, C.byref(n)), "tns_workspace")
    return int(n.value)


def tns_run(plan, Q: int, d_targets: int, d_t_start: int, d_t_end: int, d_inst_rowptr: int, query_id_base: int,
            d_out_nbr: int, d_out_eid: int, d_out_ts: int, d_out_count: int, d_rowptr: int = 0, d_cmp_nbr: int = 0,
            d_cmp_eid: int = 0, d_cmp_ts: int = 0, d_workspace: int = 0, workspace_bytes: int = 0,
            hip_stream: int = 0) -> None:
    """All d_* arguments are raw device addresses (e.g. ``tensor.data_ptr()``), 0 for NULL."""
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_run(plan, Q, vp(d_targets), vp(d_t_start), vp(d_t_end), vp(d_inst_rowptr), query_id_base,
                         vp(d_out_nbr), vp(d_out_eid), vp(d_out_ts), vp(d_out_count), vp(d_rowptr), vp(d_cmp_nbr),
                         vp(d_cmp_eid), vp(d_cmp_ts), vp(d_workspace), workspace_bytes, vp(hip_stream)), "tns_run")


def tns_run_status(plan, d_workspace: int = 0, hip_stream: int = 0) -> bool:
    """True if a bounded wait of the padding removal ran out in the last step that used the workspace
    (0 = the static scratch of tns_run_static).  Waits for the stream."""
    out = C.c_int32()
    _check(lib().tns_run_status(plan, C.c_void_p(d_workspace or None), C.c_void_p(hip_stream or None), C.byref(out)),
           "tns_run_status")
    return bool(out.value)


def tns_run_static(plan, Q: int, d_targets: int, d_t_start: int, d_t_end: int, d_inst_rowptr: int, query_id_base: int,
                   d_out_nbr: int, d_out_eid: int, d_out_ts: int, d_out_count: int, d_rowptr: int, d_cmp_nbr: int,
                   d_cmp_eid: int, d_cmp_ts: int, hip_stream: int = 0) -> None:
    """tns_run with padding removal on the library's static scratch (no workspace argument)."""
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_run_static(plan, Q, vp(d_targets), vp(d_t_start), vp(d_t_end), vp(d_inst_rowptr), query_id_base,
                                vp(d_out_nbr), vp(d_out_eid), vp(d_out_ts), vp(d_out_count), vp(d_rowptr), vp(d_cmp_nbr),
                                vp(d_cmp_eid), vp(d_cmp_ts), vp(hip_stream)), "tns_run_static")


def tns_workspace_khop(plan, fanouts, Q: int) -> int:
    fo = (C.c_int32 * len(fanouts))(*fanouts)
    n = C.c_size_t()
    _check(lib().tns_workspace_khop(plan, len(fanouts), fo, Q, C.byref(n)), "tns_workspace_khop")
    return int(n.value)


def tns_run_khop(plan, fanouts, delta: float, Q: int, d_targets: int, d_t_start: int, d_t_end: int, d_inst_rowptr: int,
                 query_id_base: int, hops, d_workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    """hops: one dict per hop with the raw device addresses nbr, eid, ts, count, rowptr, cmp_nbr, cmp_eid, cmp_ts."""
    vp = lambda x: C.c_void_p(x or None)
    fo = (C.c_int32 * len(fanouts))(*fanouts)
    hb = (tns_hop_buffers * len(hops))()
    for i, h in enumerate(hops):
        for name, _ in tns_hop_buffers._fields_:
            setattr(hb[i], name, h[name] or None)
    _check(lib().tns_run_khop(plan, len(fanouts), fo, delta, Q, vp(d_targets), vp(d_t_start), vp(d_t_end),
                              vp(d_inst_rowptr), query_id_base, hb, vp(d_workspace), workspace_bytes, vp(hip_stream)),
           "tns_run_khop")


def tns_compact(plan, Q: int, d_out_nbr: int, d_out_eid: int, d_out_ts: int, d_out_count: int, d_rowptr: int,
                d_cmp_nbr: int, d_cmp_eid: int, d_cmp_ts: int, d_workspace: int, workspace_bytes: int,
                hip_stream: int = 0) -> None:
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_compact(plan, Q, vp(d_out_nbr), vp(d_out_eid), vp(d_out_ts), vp(d_out_count), vp(d_rowptr),
                             vp(d_cmp_nbr), vp(d_cmp_eid), vp(d_cmp_ts), vp(d_workspace), workspace_bytes,
                             vp(hip_stream)), "tns_compact")


def tns_traffic_model(plan, Q: int, d_targets: int, d_t_start: int, d_t_end: int, d_inst_rowptr: int,
                      query_id_base: int, d_counters: int, hip_stream: int = 0) -> None:
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_traffic_model(plan, Q, vp(d_targets), vp(d_t_start), vp(d_t_end), vp(d_inst_rowptr),
                                   query_id_base, vp(d_counters), vp(hip_stream)), "tns_traffic_model")


def tns_stats(plan, instance: int = -1) -> dict:
    st = tns_stats_t()
    _check(lib().tns_stats(plan, instance, C.byref(st)), "tns_stats")
    return {k: getattr(st, k) for k, _ in tns_stats_t._fields_}


def tns_node_blocks(plan, instance: int, node: int) -> dict:
    n = lib().tns_node_blocks(plan, instance, node, 0, None, None, None, None)
    if n < 0:
        raise TnsError(int(n), "tns_node_blocks")
    cap = np.empty(n, np.int32)
    size = np.empty(n, np.int32)
    tmin = np.empty(n, np.float32)
    tmax = np.empty(n, np.float32)
    i32p, f32p = C.POINTER(C.c_int32), C.POINTER(C.c_float)
    lib().tns_node_blocks(plan, instance, node, n, cap.ctypes.data_as(i32p), size.ctypes.data_as(i32p),
                          tmin.ctypes.data_as(f32p), tmax.ctypes.data_as(f32p))
    return dict(cap=cap, size=size, t_min=tmin, t_max=tmax)


def tns_hbm_probe(mode: int, nontemporal: bool, d_dst: int, d_src: int, nbytes: int, hip_stream: int = 0) -> None:
    """Streaming kernel of known traffic: mode 0 copy, 1 read, 2 write (raw device addresses)."""
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_hbm_probe(mode, 1 if nontemporal else 0, vp(d_dst), vp(d_src), nbytes, vp(hip_stream)), "tns_hbm_probe")


def tns_hbm_probe_mix(nontemporal: bool, d_dst: int, write_bytes: int, d_src: int, read_bytes: int, hip_stream: int = 0) -> None:
    """Streaming kernel that reads read_bytes and writes write_bytes, evenly interleaved (measurement aid)."""
    vp = lambda x: C.c_void_p(x or None)
    _check(lib().tns_hbm_probe_mix(1 if nontemporal else 0, vp(d_dst), write_bytes, vp(d_src), read_bytes, vp(hip_stream)),
           "tns_hbm_probe_mix")


def tns_destroy(plan) -> None:
    _check(lib().tns_destroy(plan), "tns_destroy")


# ---- convenience wrapper: owns the handle, allocates outputs as torch tensors -----------

class Plan:
    """Owns a tns_plan.  ``run`` allocates the output tensors on the plan's device with
    torch and passes raw pointers and the current torch stream to ``tns_run``."""

    def __init__(self, num_nodes: int, fanout: int, policy: int = TNS_POLICY_RECENT, block_threshold: int = 48,
                 num_instances: int = 1, sizing: int = TNS_SIZING_ADAPTIVE, inclusive_end: int = 0, seed: int = 0,
                 device: int = 0, flags: int = 0):
        self.num_nodes, self.fanout, self.num_instances, self.device = num_nodes, fanout, num_instances, device
        self.policy, self.flags = policy, flags
        self._h = tns_plan_create(num_nodes, fanout, policy, block_threshold, num_instances, sizing, inclusive_end,
                                  seed, device, flags)

    @property
    def handle(self):
        return self._h

    def set_sampler(self, fanout: int, policy: int = TNS_POLICY_RECENT, inclusive_end: int = 0, seed: int = 0):
        tns_set_sampler(self._h, fanout, policy, inclusive_end, seed)
        self.fanout, self.policy = fanout, policy

    def add_edges(self, src, dst, ts, eid=None, instance: int = 0):
        tns_add_edges(self._h, instance, src, dst, ts, eid)

    def add_edges_device(self, src, dst, ts, eid=None, instance: int = 0):
        """Batch given as torch tensors on the plan's device (int32, int32, float32[, int32]); needs a plan
        created with TNS_FLAG_DEVICE_INGEST."""
        import torch
        want = [(src, torch.int32), (dst, torch.int32), (ts, torch.float32)] + ([(eid, torch.int32)] if eid is not None else [])
        for t, dt in want:
            if t.dtype != dt or not t.is_cuda or t.device.index != self.device or not t.is_contiguous() or t.dim() != 1:
                raise ValueError("batch arrays must be contiguous 1-d tensors of the right dtype on the plan's device")
            if t.numel() != src.numel():
                raise ValueError("src, dst, ts (and eid) must have the same length")
        with torch.cuda.device(self.device):
            tns_add_edges_device(self._h, instance, src.data_ptr(), dst.data_ptr(), ts.data_ptr(),
                                 None if eid is None else eid.data_ptr(), src.numel(),
                                 torch.cuda.current_stream().cuda_stream)

    def add_stream(self, stream, instance: int = 0):
        """Ingest a workloads.Stream batch by batch, as the paper's continuous-learning setting does."""
        for lo, hi in stream.batches():
            tns_add_edges(self._h, instance, stream.src[lo:hi], stream.dst[lo:hi], stream.ts[lo:hi], None)

    def commit(self):
        import torch
        with torch.cuda.device(self.device):
            tns_commit(self._h, torch.cuda.current_stream().cuda_stream)

    def stats(self, instance: int = -1) -> dict:
        return tns_stats(self._h, instance)

    def node_blocks(self, node: int, instance: int = 0) -> dict:
        return tns_node_blocks(self._h, instance, node)

    def alloc_outputs(self, Q: int, compact: bool = True):
        import torch
        dev = torch.device("cuda", self.device)
        f = self.fanout
        out = dict(nbr=torch.empty(Q * f, dtype=torch.int32, device=dev),
                   eid=torch.empty(Q * f, dtype=torch.int32, device=dev),
                   ts=torch.empty(Q * f, dtype=torch.float32, device=dev),
                   count=torch.empty(Q, dtype=torch.int32, device=dev))
        if compact:
            out.update(rowptr=torch.empty(Q + 1, dtype=torch.int64, device=dev),
                       cmp_nbr=torch.empty(Q * f, dtype=torch.int32, device=dev),
                       cmp_eid=torch.empty(Q * f, dtype=torch.int32, device=dev),
                       cmp_ts=torch.empty(Q * f, dtype=torch.float32, device=dev),
                       workspace=torch.empty(tns_workspace(self._h, Q), dtype=torch.uint8, device=dev))
        return out

    def run(self, targets, t_start, t_end, inst_rowptr=None, out: Optional[dict] = None, compact: bool = True,
            query_id_base: int = 0) -> dict:
        """targets/t_start/t_end/inst_rowptr: torch tensors on the plan's device (t_start may be None)."""
        import torch
        Q = int(targets.shape[0])
        if out is None:
            out = self.alloc_outputs(Q, compact)
        p = lambda t: 0 if t is None else t.data_ptr()
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream().cuda_stream
            tns_run(self._h, Q, p(targets), p(t_start), p(t_end), p(inst_rowptr), query_id_base,
                    p(out.get("nbr")), p(out.get("eid")), p(out.get("ts")), p(out.get("count")),
                    p(out.get("rowptr")), p(out.get("cmp_nbr")), p(out.get("cmp_eid")), p(out.get("cmp_ts")),
                    p(out.get("workspace")), 0 if out.get("workspace") is None else out["workspace"].numel(), stream)
        return out

    def status(self, workspace=None) -> bool:
        """True if the padding removal of the last step on `workspace` (None: tns_run_static's scratch) timed out."""
        import torch
        with torch.cuda.device(self.device):
            return tns_run_status(self._h, 0 if workspace is None else workspace.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)

    def run_khop(self, fanouts, targets, t_start, t_end, inst_rowptr=None, delta: float = float("inf"),
                 query_id_base: int = 0):
        """Multi-hop sampling; returns one dict of output tensors per hop (sized for the most
        queries the hop can have) plus the workspace tensor."""
        import torch
        dev = torch.device("cuda", self.device)
        Q = int(targets.shape[0])
        hops, cap = [], Q
        for f in fanouts:
            hops.append(dict(nbr=torch.empty(cap * f, dtype=torch.int32, device=dev),
                             eid=torch.empty(cap * f, dtype=torch.int32, device=dev),
                             ts=torch.empty(cap * f, dtype=torch.float32, device=dev),
                             count=torch.empty(cap, dtype=torch.int32, device=dev),
                             rowptr=torch.empty(cap + 1, dtype=torch.int64, device=dev),
                             cmp_nbr=torch.empty(cap * f, dtype=torch.int32, device=dev),
                             cmp_eid=torch.empty(cap * f, dtype=torch.int32, device=dev),
                             cmp_ts=torch.empty(cap * f, dtype=torch.float32, device=dev), cap=cap, fanout=f))
            cap *= f
        ws = torch.empty(tns_workspace_khop(self._h, fanouts, Q), dtype=torch.uint8, device=dev)
        p = lambda t: 0 if t is None else t.data_ptr()
        ptrs = [{k: p(v) for k, v in h.items() if k not in ("cap", "fanout")} for h in hops]
        with torch.cuda.device(self.device):
            tns_run_khop(self._h, list(fanouts), delta, Q, p(targets), p(t_start), p(t_end), p(inst_rowptr),
                         query_id_base, ptrs, ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        return hops, ws

    def close(self):
        if getattr(self, "_h", None):
            tns_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
