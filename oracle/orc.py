"""ctypes loader for the CPU oracle (test infrastructure; never imported by the product package).

``build()`` compiles ``tangram_oracle.cpp`` with g++ into ``liborc.so`` next to it; the
wrappers take the numpy problem / trace dicts of ``gen`` and return numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tangram_oracle.cpp")
_LIB = os.path.join(_HERE, "liborc.so")
_BF_SRC = os.path.join(_HERE, "bruteforce.cpp")
_BF_LIB = os.path.join(_HERE, "libbrute.so")
_lib = None
_bf = None

INF = np.iinfo(np.int64).max


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", _LIB, _SRC])
    if force or not os.path.exists(_BF_LIB) or os.path.getmtime(_BF_LIB) < os.path.getmtime(_BF_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", _BF_LIB, _BF_SRC])
    return _LIB


def brute():
    """Exhaustive-search library (bruteforce.cpp): bf_value, bf_best."""
    global _bf
    if _bf is None:
        build()
        L = C.CDLL(_BF_LIB)
        L.bf_value.restype = C.c_int64
        L.bf_value.argtypes = [C.c_int] * 4 + [C.c_void_p] * 6
        L.bf_best.restype = C.c_int64
        L.bf_best.argtypes = [C.c_int] * 4 + [C.c_void_p] * 4 + [C.c_int] + [C.c_void_p] * 2
        _bf = L
    return _bf


class Problem(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "N", "M", "K", "n_classes", "n_tasks", "depth", "order_policy")] + [
        (n, C.c_void_p) for n in (
            "k_list", "type_k", "speedup_q16", "node_type", "node_cap", "node_free", "node_backlog_us",
            "node_chunks", "node_busy_off", "node_busy_rel_us", "act_type", "act_model", "act_t_ori_us",
            "act_age_us", "act_kmask", "act_param", "act_pin_node", "act_task", "node_aux_free", "act_aux",
            "act_service", "node_resident", "restore_us", "act_quota_mask", "node_core_free")] + [("numa_cores", C.c_int32), ("gpu_pooled", C.c_int32), ("queue_prefix", C.c_int32)]


class Summary(C.Structure):
    _fields_ = [("sum_act_us", C.c_int64), ("n_assigned", C.c_int32), ("n_prefix", C.c_int32),
                ("n_evicted", C.c_int32), ("n_infeasible", C.c_int32), ("units_used", C.c_int64 * 3),
                ("units_free", C.c_int64 * 3), ("mean_act_us", C.c_double), ("util", C.c_double * 3)]


SUMMARY_DTYPE = np.dtype([("sum_act_us", "<i8"), ("n_assigned", "<i4"), ("n_prefix", "<i4"), ("n_evicted", "<i4"),
                          ("n_infeasible", "<i4"), ("units_used", "<i8", 3), ("units_free", "<i8", 3),
                          ("mean_act_us", "<f8"), ("util", "<f8", 3)])


class Trace(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("S", "A", "M", "K", "n_classes", "depth", "max_ticks", "cache_slots")] + [
        ("tick_us", C.c_int64)] + [(n, C.c_void_p) for n in (
            "k_list", "type_k", "speedup_q16", "node_type", "node_cap", "quota_rate", "quota_tok0_micro",
            "arrival_us", "act_type", "act_model", "act_t_ori_us", "act_kmask", "act_param", "act_pin_node",
            "act_service", "restore_us", "act_quota_mask")] + [("queue_prefix", C.c_int32)] + [
        ("node_aux", C.c_void_p), ("act_aux", C.c_void_p), ("numa_cores", C.c_int32), ("order_policy", C.c_int32),
        ("gpu_pooled", C.c_int32), ("cache_per_gpu", C.c_int32)]


_DT = dict(k_list=np.int32, type_k=np.int32, speedup_q16=np.uint32, node_type=np.uint8, node_cap=np.int32,
           node_free=np.int32, node_backlog_us=np.int64, node_chunks=np.uint8, node_busy_off=np.int32,
           node_busy_rel_us=np.int64, act_type=np.uint8, act_model=np.uint8, act_t_ori_us=np.int64,
           act_age_us=np.int64, act_kmask=np.uint32, act_param=np.uint32, act_pin_node=np.int32,
           act_task=np.int32, quota_rate=np.int32, quota_tok0_micro=np.int64, arrival_us=np.int64,
           node_aux_free=np.int32, act_aux=np.int32, act_service=np.int32, node_resident=np.uint64, restore_us=np.int64,
           node_core_free=np.uint64, act_quota_mask=np.uint64, node_aux=np.int32)


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_duration.restype = C.c_int64
        L.orc_duration.argtypes = [C.c_int, C.c_int64, C.c_uint32, C.c_int, C.c_uint32]
        L.orc_num_candidates.restype = C.c_int64
        L.orc_num_candidates.argtypes = [C.c_void_p]
        L.orc_score.restype = None
        L.orc_score.argtypes = [C.c_void_p, C.c_void_p]
        L.orc_assign.restype = None
        L.orc_assign.argtypes = [C.c_void_p] * 11
        L.orc_take_cores.restype = C.c_int
        L.orc_take_cores.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.orc_dp_units.restype = C.c_int64
        L.orc_dp_units.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_dp_chunks.restype = C.c_int64
        L.orc_dp_chunks.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_estimate.restype = C.c_int64
        L.orc_estimate.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        L.orc_chunk_take.restype = C.c_int
        L.orc_chunk_take.argtypes = [C.c_void_p, C.c_int]
        L.orc_chunk_encode_roundtrip.restype = C.c_int
        L.orc_chunk_encode_roundtrip.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.orc_mask_chunks.restype = C.c_int
        L.orc_mask_chunks.argtypes = [C.c_int, C.c_void_p]
        L.orc_mask_alloc.restype = C.c_int
        L.orc_mask_alloc.argtypes = [C.POINTER(C.c_int), C.c_int]
        L.orc_replay.restype = None
        L.orc_replay.argtypes = [C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 9
        L.orc_replay_extents.restype = None
        L.orc_replay_extents.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        _lib = L
    return _lib


def _fill(struct, d, names, keep):
    for n in names:
        v = d.get(n)
        if v is None:
            setattr(struct, n, None)
            continue
        a = np.ascontiguousarray(v, dtype=_DT[n])
        keep.append(a)
        setattr(struct, n, a.ctypes.data)


def _problem(p):
    keep = []
    s = Problem()
    for n in ("B", "N", "M", "K", "n_classes", "n_tasks", "depth"):
        setattr(s, n, int(p[n]))
    s.order_policy = int(p.get("order_policy", 0))      # 0: first come first served, 1: least estimated ACT first
    _fill(s, p, [f[0] for f in Problem._fields_[8:-3]], keep)
    s.numa_cores = int(p.get("numa_cores", 0))          # cores per NUMA domain (with node_core_free)
    s.gpu_pooled = int(p.get("gpu_pooled", 0))          # 1: the GPU nodes of a snapshot are one pool of chunks
    s.queue_prefix = int(p.get("queue_prefix", 0))      # 1: one admitted prefix of the whole queue instead of one per pool
    return s, keep


def _trace(t):
    keep = []
    s = Trace()
    for n in ("S", "A", "M", "K", "n_classes", "depth", "max_ticks"):
        setattr(s, n, int(t[n]))
    s.tick_us = int(t["tick_us"])
    s.cache_slots = int(t.get("cache_slots", 64))
    s.queue_prefix = int(t.get("queue_prefix", 0))       # 1: every step admits one prefix of the whole waiting queue
    s.numa_cores = int(t.get("numa_cores", 0))           # > 0: CPU actions get named cores (NUMA domains of that many)
    s.order_policy = int(t.get("order_policy", 0))       # 1: every step visits the queue by least estimated ACT
    s.gpu_pooled = int(t.get("gpu_pooled", 0))           # 1: every step sees the GPU nodes as one pool of chunks
    s.cache_per_gpu = int(t.get("cache_per_gpu", 0))     # 1: every GPU of a GPU node keeps its own cache of services
    _fill(s, t, [f[0] for f in Trace._fields_[9:-7]] + ["node_aux", "act_aux"], keep)
    return s, keep


def duration(model, T, param, k, speedup=0):
    return int(lib().orc_duration(int(model), int(T), int(param), int(k), int(speedup)))


def num_candidates(p):
    s, keep = _problem(p)
    return int(lib().orc_num_candidates(C.addressof(s)))


def score(p):
    s, keep = _problem(p)
    n = int(lib().orc_num_candidates(C.addressof(s)))
    cost = np.empty(n, np.int64)
    lib().orc_score(C.addressof(s), cost.ctypes.data)
    return cost


def assign(p):
    s, keep = _problem(p)
    B, N, M = int(p["B"]), int(p["N"]), int(p["M"])
    out = dict(node=np.empty(B * N, np.int32), units=np.empty(B * N, np.int32), act_us=np.empty(B * N, np.int64),
               reason=np.empty(B * N, np.uint8), summary=np.zeros(B, SUMMARY_DTYPE),
               node_used=np.empty(B * M, np.int32), task_sum=np.empty(B * int(p["n_tasks"]), np.int64),
               node_obj=np.empty(B * M, np.int64), home=np.empty(B * N, np.int32))
    if p.get("node_core_free") is not None:
        out["core_set"] = np.zeros(B * N * 4, np.uint64)
    assert SUMMARY_DTYPE.itemsize == C.sizeof(Summary)
    lib().orc_assign(C.addressof(s), *[out[k].ctypes.data for k in
                                       ("node", "units", "act_us", "reason", "summary", "node_used", "task_sum", "node_obj", "home")],
                     out["core_set"].ctypes.data if "core_set" in out else None)
    return out


def take_cores(free, numa_cores, k):
    """One allocation on a 0/1 map of free cores; returns (core ids, map afterwards)."""
    f = np.ascontiguousarray(free, np.uint8).copy()
    got = np.zeros(max(int(k), 1), np.int32)
    n = lib().orc_take_cores(f.ctypes.data, len(f), int(numa_cores), int(k), got.ctypes.data)
    return [int(x) for x in got[:n]], f


def dp_units(dur, k_list, U):
    dur = np.ascontiguousarray(dur, np.int64)
    m, K = dur.shape
    kl = np.ascontiguousarray(k_list, np.int32)
    k_out = np.zeros(m, np.int32)
    v = lib().orc_dp_units(m, dur.ctypes.data, kl.ctypes.data, K, int(U), k_out.ctypes.data)
    return int(v), k_out


def dp_chunks(dur, k_list, chunks):
    dur = np.ascontiguousarray(dur, np.int64)
    m, K = dur.shape
    kl = np.ascontiguousarray(k_list, np.int32)
    ch = np.ascontiguousarray(chunks, np.uint8)
    k_out = np.zeros(m, np.int32)
    v = lib().orc_dp_chunks(m, dur.ctypes.data, kl.ctypes.data, K, ch.ctypes.data, k_out.ctypes.data)
    return int(v), k_out


def estimate(heap, ac_dur, k_list, depth):
    heap = np.ascontiguousarray(heap, np.int64)
    kl = np.ascontiguousarray(k_list, np.int32)
    ac_dur = np.ascontiguousarray(ac_dur, np.int64).reshape(-1, len(kl))
    return int(lib().orc_estimate(heap.ctypes.data, len(heap), ac_dur.shape[0], ac_dur.ctypes.data,
                                  kl.ctypes.data, len(kl), int(depth)))


def chunk_take(chunks, k):
    ch = np.array(chunks, np.uint8)
    ok = lib().orc_chunk_take(ch.ctypes.data, int(k))
    return bool(ok), tuple(int(x) for x in ch)


def chunk_roundtrip(bound, j):
    b = np.array(bound, np.uint8)
    out = np.zeros(4, np.uint8)
    e = lib().orc_chunk_encode_roundtrip(b.ctypes.data, int(j), out.ctypes.data)
    return int(e), tuple(int(x) for x in out)


def mask_chunks(mask):
    out = np.zeros(4, np.uint8)
    lib().orc_mask_chunks(int(mask), out.ctypes.data)
    return tuple(int(x) for x in out)


def mask_alloc(mask, k):
    m = C.c_int(int(mask))
    s = lib().orc_mask_alloc(C.byref(m), int(k))
    return int(s), int(m.value)


def replay(t, s_lo=0, s_hi=None):
    s, keep = _trace(t)
    S, A = int(t["S"]), int(t["A"])
    s_hi = S if s_hi is None else s_hi
    out = dict(start_us=np.full(S * A, -1, np.int64), finish_us=np.full(S * A, -1, np.int64),
               units=np.zeros(S * A, np.int32), node=np.full(S * A, -1, np.int32), mean_act=np.zeros(S),
               p99_act=np.full(S, -1, np.int64), n_started=np.zeros(S, np.int32), n_ticks=np.zeros(S, np.int32))
    if int(t.get("numa_cores", 0)) > 0:
        out["core_set"] = np.zeros(S * A * 4, np.uint64)
    lib().orc_replay(C.addressof(s), int(s_lo), int(s_hi), *[out[k].ctypes.data for k in
                     ("start_us", "finish_us", "units", "node", "mean_act", "p99_act", "n_started", "n_ticks")],
                     out["core_set"].ctypes.data if "core_set" in out else None)
    return out


EXTENTS = ("wait_cpu", "wait_gpu", "wait_api", "running", "cand_cpu_elastic", "cand_gpu_elastic", "cand_node",
           "cand_step", "pinned_wait_step", "busy_units", "heap_entries", "chunk_states", "dp_cells", "nodes_cpu",
           "nodes_gpu", "nodes_api")


def replay_extents(t, s_lo=0, s_hi=None):
    """Largest sizes the steps of each replayed scenario worked on: {name: [S] int64} (orc_replay_extents)."""
    s, keep = _trace(t)
    S = int(t["S"])
    s_hi = S if s_hi is None else s_hi
    ext = np.zeros((S, len(EXTENTS)), np.int64)
    lib().orc_replay_extents(C.addressof(s), int(s_lo), int(s_hi), ext.ctypes.data)
    return {n: ext[:, x].copy() for x, n in enumerate(EXTENTS)}
