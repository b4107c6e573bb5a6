"""Thin ctypes binding of libtangram.so (see include/tg.h).

Only argument marshalling happens here: numpy arrays become host pointers, torch CUDA tensors
provide device memory and the current HIP stream.  Every step of the scheduling path runs in
the library's kernels; there is no CPU fallback - a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

OK = 0
E_INVALID_ARG = -1
E_RANGE = -2
INF = np.iinfo(np.int64).max


class TgError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class ProblemDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "N", "M", "K", "n_classes", "n_tasks", "depth")] + [
        ("order_policy", C.c_int32)] + [(n, C.c_void_p) for n in (
            "k_list", "type_k", "speedup_q16", "node_type", "node_cap", "node_free", "node_backlog_us",
            "node_chunks", "node_busy_off", "node_busy_rel_us", "act_type", "act_model", "act_t_ori_us",
            "act_age_us", "act_kmask", "act_param", "act_pin_node", "act_task", "node_aux_free", "act_aux",
            "act_service", "node_resident", "restore_us", "node_core_free", "act_quota_mask")] + [(n, C.c_int32) for n in
                                                                        ("n_services", "numa_cores", "gpu_pooled", "queue_prefix", "nodes_shared", "reserved_")]


class AssignOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("node", "units", "act_us", "defer_reason", "summary", "node_used",
                                          "task_sum_us", "node_obj", "core_set")]


class TraceDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("S", "A", "M", "K", "n_classes", "depth", "max_ticks")] + [
        ("flags", C.c_uint32), ("tick_us", C.c_int64)] + [(n, C.c_void_p) for n in (
            "k_list", "type_k", "speedup_q16", "node_type", "node_cap", "quota_rate", "quota_tok0_micro",
            "arrival_us", "act_type", "act_model", "act_t_ori_us", "act_kmask", "act_param", "act_pin_node",
            "act_service", "restore_us")] + [("n_services", C.c_int32), ("cache_slots", C.c_int32),
                                             ("act_quota_mask", C.c_void_p), ("node_aux", C.c_void_p),
                                             ("act_aux", C.c_void_p), ("numa_cores", C.c_int32), ("order_policy", C.c_int32)]


class ReplayOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("start_us", "finish_us", "units", "node", "mean_act_us", "p99_act_us",
                                          "n_started", "n_ticks", "core_set")]


SUMMARY_DTYPE = np.dtype([("sum_act_us", "<i8"), ("n_selected", "<i4"), ("n_prefix", "<i4"), ("n_evicted", "<i4"),
                          ("n_infeasible", "<i4"), ("units_used", "<i8", 3), ("units_free", "<i8", 3),
                          ("mean_act_us", "<f8"), ("util", "<f8", 3)])

_DT = dict(k_list=np.int32, type_k=np.int32, speedup_q16=np.uint32, node_type=np.uint8, node_cap=np.int32,
           node_free=np.int32, node_backlog_us=np.int64, node_chunks=np.uint8, node_busy_off=np.int32,
           node_busy_rel_us=np.int64, act_type=np.uint8, act_model=np.uint8, act_t_ori_us=np.int64,
           act_age_us=np.int64, act_kmask=np.uint32, act_param=np.uint32, act_pin_node=np.int32,
           act_task=np.int32, quota_rate=np.int32, quota_tok0_micro=np.int64, arrival_us=np.int64,
           node_aux_free=np.int32, act_aux=np.int32, act_service=np.int32, node_resident=np.uint64, restore_us=np.int64,
           node_core_free=np.uint64, act_quota_mask=np.uint64, node_aux=np.int32)

EXPORTS = ("tg_build_problem", "tg_free_problem", "tg_num_candidates", "tg_assign_workspace_bytes",
           "tg_score_candidates", "tg_assign", "tg_assign_static", "tg_step", "tg_step_on", "tg_build_trace", "tg_free_trace", "tg_replay_workspace_bytes",
           "tg_replay_trace", "tg_replay_trace_part", "tg_replay_capacity", "tg_strerror")


def library_path():
    return _build.LIB


def load():
    """Load libtangram.so (building it first only if no built library is there)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build_library()
        L = C.CDLL(path)
        vp = C.c_void_p
        L.tg_build_problem.argtypes = [vp, vp, C.POINTER(vp)]
        L.tg_free_problem.argtypes = [vp]
        L.tg_free_problem.restype = None
        L.tg_num_candidates.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.tg_assign_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        L.tg_score_candidates.argtypes = [vp, vp, vp]
        L.tg_assign.argtypes = [vp, vp, vp, vp, C.c_size_t, vp]
        L.tg_assign_static.argtypes = [vp, vp, vp, vp]
        L.tg_step.argtypes = [vp, vp, vp, vp, C.c_size_t, vp]
        L.tg_step_on.argtypes = [vp, vp, vp, vp, C.c_size_t, vp, vp]
        L.tg_build_trace.argtypes = [vp, vp, C.POINTER(vp)]
        L.tg_free_trace.argtypes = [vp]
        L.tg_free_trace.restype = None
        L.tg_replay_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        L.tg_replay_trace.argtypes = [vp, vp, vp, C.c_size_t, vp]
        L.tg_replay_trace_part.argtypes = [vp, vp, vp, C.c_size_t, C.c_int, C.c_int, vp]
        L.tg_replay_capacity.argtypes = [vp, vp]
        L.tg_strerror.argtypes = [C.c_int]
        L.tg_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def strerror(code):
    return load().tg_strerror(int(code)).decode()


def _check(code, what):
    if code != OK:
        raise TgError(code, what)


def _fill(struct, d, names, keep):
    for n in names:
        v = d.get(n)
        if v is None:
            setattr(struct, n, None)
            continue
        a = np.ascontiguousarray(v, dtype=_DT[n])
        keep.append(a)
        setattr(struct, n, a.ctypes.data)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)


class Problem:
    """B cluster snapshots packed on the device (tg_build_problem)."""

    def __init__(self, p: dict):
        L = load()
        d = ProblemDesc()
        for n in ("B", "N", "M", "K", "n_classes", "n_tasks", "depth"):
            setattr(d, n, int(p[n]))
        d.order_policy = int(p.get("order_policy", 0))
        keep = []
        _fill(d, p, [f[0] for f in ProblemDesc._fields_[8:-6]], keep)
        d.n_services = len(p["restore_us"]) if p.get("restore_us") is not None else 0
        d.numa_cores = int(p.get("numa_cores", 0))
        d.gpu_pooled = int(p.get("gpu_pooled", 0))
        d.queue_prefix = int(p.get("queue_prefix", 0))
        d.nodes_shared = int(p.get("nodes_shared", 0))
        self.has_cores = p.get("node_core_free") is not None
        h = C.c_void_p()
        _check(L.tg_build_problem(C.byref(d), _stream(), C.byref(h)), "tg_build_problem")
        self._h = h
        self.B, self.N, self.M, self.n_tasks = int(p["B"]), int(p["N"]), int(p["M"]), int(p["n_tasks"])
        cnt, nbytes = C.c_int64(), C.c_int64()
        _check(L.tg_num_candidates(h, C.byref(cnt), C.byref(nbytes)), "tg_num_candidates")
        self.num_candidates = int(cnt.value)
        ws = C.c_size_t()
        _check(L.tg_assign_workspace_bytes(h, C.byref(ws)), "tg_assign_workspace_bytes")
        self.assign_ws_bytes = int(ws.value)

    def free(self):
        if getattr(self, "_h", None):
            load().tg_free_problem(self._h)
            self._h = None

    __del__ = free

    def alloc_cost(self):
        import torch
        return torch.empty(max(self.num_candidates, 2), dtype=torch.int64, device="cuda")

    def score(self, out=None):
        """tg_score_candidates into ``out`` (a CUDA int64 tensor) or a new tensor."""
        if out is None:
            out = self.alloc_cost()
        _check(load().tg_score_candidates(self._h, _ptr(out), _stream()), "tg_score_candidates")
        return out

    def alloc_assign(self):
        import torch
        dev = "cuda"
        B, N, M = self.B, self.N, self.M
        bufs = dict(
            node=torch.empty(B * N, dtype=torch.int32, device=dev),
            units=torch.empty(B * N, dtype=torch.int32, device=dev),
            act_us=torch.empty(B * N, dtype=torch.int64, device=dev),
            defer_reason=torch.empty(B * N, dtype=torch.uint8, device=dev),
            summary=torch.empty(B * SUMMARY_DTYPE.itemsize, dtype=torch.uint8, device=dev),
            node_used=torch.empty(B * M, dtype=torch.int32, device=dev),
            task_sum_us=torch.empty(B * self.n_tasks, dtype=torch.int64, device=dev),
            node_obj=torch.empty(B * M, dtype=torch.int64, device=dev),
            ws=torch.empty(max(self.assign_ws_bytes, 256), dtype=torch.uint8, device=dev),
        )
        if self.has_cores:
            bufs["core_set"] = torch.empty(B * N * 4, dtype=torch.int64, device=dev)   # bit patterns of uint64 words
        return bufs

    def assign(self, cost=None, bufs=None):
        """tg_assign; returns the dict of CUDA output tensors (summary as raw bytes)."""
        if bufs is None:
            bufs = self.alloc_assign()
        o = AssignOut()
        for n, _ in AssignOut._fields_:
            setattr(o, n, bufs[n].data_ptr() if bufs.get(n) is not None else None)
        _check(load().tg_assign(self._h, _ptr(cost), C.byref(o), _ptr(bufs["ws"]), bufs["ws"].numel(), _stream()),
               "tg_assign")
        return bufs

    def assign_static(self, cost, bufs):
        """tg_assign_static: tg_assign on the library's static workspace (``bufs`` needs no "ws")."""
        o = AssignOut()
        for n, _ in AssignOut._fields_:
            setattr(o, n, bufs[n].data_ptr() if bufs.get(n) is not None else None)
        _check(load().tg_assign_static(self._h, _ptr(cost), C.byref(o), _stream()), "tg_assign_static")
        return bufs

    def step(self, cost, bufs, score_stream=None):
        """tg_step: the score tensor into ``cost`` and the assignment into ``bufs`` in one call; with ``score_stream``
        (a torch.cuda.Stream other than the current one) tg_step_on: the score kernels run on that stream."""
        o = AssignOut()
        for n, _ in AssignOut._fields_:
            setattr(o, n, bufs[n].data_ptr() if bufs.get(n) is not None else None)
        if score_stream is None:
            _check(load().tg_step(self._h, _ptr(cost), C.byref(o), _ptr(bufs["ws"]), bufs["ws"].numel(), _stream()), "tg_step")
        else:
            _check(load().tg_step_on(self._h, _ptr(cost), C.byref(o), _ptr(bufs["ws"]), bufs["ws"].numel(), _stream(),
                                     C.c_void_p(score_stream.cuda_stream)), "tg_step_on")
        return cost, bufs


def summary_to_numpy(summary_bytes):
    return np.frombuffer(summary_bytes.cpu().numpy().tobytes(), dtype=SUMMARY_DTYPE)


REPLAY_CAPS = ("wait_cpu", "wait_gpu", "wait_api", "running", "cand_cpu_elastic", "cand_gpu_elastic", "cand_node",
               "cand_step", "pinned_wait_step", "busy_units", "heap_entries", "chunk_states", "dp_cells", "nodes_cpu",
               "nodes_gpu", "nodes_api")


def _trace_desc(t: dict):
    d = TraceDesc()
    for n in ("S", "A", "M", "K", "n_classes", "depth", "max_ticks"):
        setattr(d, n, int(t[n]))
    d.flags = ((1 if int(t.get("queue_prefix", 0)) else 0) | (2 if int(t.get("gpu_pooled", 0)) else 0)   # TG_TRACE_QUEUE_PREFIX, _GPU_POOLED
               | (4 if int(t.get("cache_per_gpu", 0)) else 0))                                           # _CACHE_PER_GPU
    d.tick_us = int(t["tick_us"])
    keep = []
    _fill(d, t, [f[0] for f in TraceDesc._fields_[9:-7]] + ["act_quota_mask", "node_aux", "act_aux"], keep)
    d.numa_cores = int(t.get("numa_cores", 0))
    d.order_policy = int(t.get("order_policy", 0))
    d.n_services = len(t["restore_us"]) if t.get("restore_us") is not None else 0
    d.cache_slots = int(t.get("cache_slots", 64))
    return d, keep


def replay_capacity(t: dict):
    """tg_replay_capacity: {name: largest value the replay's buffers hold}; host only, no device needed."""
    d, keep = _trace_desc(t)
    cap = np.zeros(len(REPLAY_CAPS), np.int64)
    _check(load().tg_replay_capacity(C.byref(d), cap.ctypes.data), "tg_replay_capacity")
    return dict(zip(REPLAY_CAPS, cap.tolist()))


class Trace:
    """S arrival traces packed on the device (tg_build_trace)."""

    def __init__(self, t: dict):
        L = load()
        d, keep = _trace_desc(t)
        h = C.c_void_p()
        _check(L.tg_build_trace(C.byref(d), _stream(), C.byref(h)), "tg_build_trace")
        self._h = h
        self.S, self.A, self.M = int(t["S"]), int(t["A"]), int(t["M"])
        self.has_cores = int(t.get("numa_cores", 0)) > 0
        ws = C.c_size_t()
        _check(L.tg_replay_workspace_bytes(h, C.byref(ws)), "tg_replay_workspace_bytes")
        self.ws_bytes = int(ws.value)

    def free(self):
        if getattr(self, "_h", None):
            load().tg_free_trace(self._h)
            self._h = None

    __del__ = free

    def alloc(self):
        import torch
        dev = "cuda"
        n = self.S * self.A
        cores = dict(core_set=torch.empty(n * 4, dtype=torch.int64, device=dev)) if self.has_cores else {}
        return dict(
            **cores,
            start_us=torch.empty(n, dtype=torch.int64, device=dev), finish_us=torch.empty(n, dtype=torch.int64, device=dev),
            units=torch.empty(n, dtype=torch.int32, device=dev), node=torch.empty(n, dtype=torch.int32, device=dev),
            mean_act_us=torch.empty(self.S, dtype=torch.float64, device=dev),
            p99_act_us=torch.empty(self.S, dtype=torch.int64, device=dev),
            n_started=torch.empty(self.S, dtype=torch.int32, device=dev),
            n_ticks=torch.empty(self.S, dtype=torch.int32, device=dev),
            ws=torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=dev))

    def replay(self, bufs=None):
        if bufs is None:
            bufs = self.alloc()
        o = ReplayOut()
        for n, _ in ReplayOut._fields_:
            setattr(o, n, bufs[n].data_ptr() if bufs.get(n) is not None else None)
        _check(load().tg_replay_trace(self._h, C.byref(o), _ptr(bufs["ws"]), bufs["ws"].numel(), _stream()),
               "tg_replay_trace")
        return bufs

    def replay_part(self, bufs, restart, n_ticks):
        """tg_replay_trace_part: ``n_ticks`` more ticks on ``bufs`` (from time 0 with ``restart``)."""
        o = ReplayOut()
        for n, _ in ReplayOut._fields_:
            setattr(o, n, bufs[n].data_ptr() if bufs.get(n) is not None else None)
        _check(load().tg_replay_trace_part(self._h, C.byref(o), _ptr(bufs["ws"]), bufs["ws"].numel(), int(bool(restart)), int(n_ticks),
                                           _stream()), "tg_replay_trace_part")
        return bufs
