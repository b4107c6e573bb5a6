"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
include/tg.h declares, and rejects bad descriptions with the documented error codes before
anything touches the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tg():
    from paper_2603_13019_amd import tg as _tg
    _tg.load()
    return _tg


def test_header_symbols_are_exported(tg):
    hdr = open(os.path.join(ROOT, "include", "tg.h")).read()
    declared = set(re.findall(r"\b(tg_[a-z_]+)\s*\(", hdr))
    assert declared == set(tg.EXPORTS)
    lib = tg.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror(tg):
    assert tg.strerror(0) == "ok"
    for code in range(-7, 0):
        assert tg.strerror(code) not in ("ok", "unknown error")
    assert tg.strerror(-99) == "unknown error"


def test_field_offsets_match_the_compiled_header(tg, tmp_path):
    """Every field of the four structs sits where a C compiler puts it: a small program that includes
    include/tg.h prints offsetof() of the fields by name, the binding's ctypes structures must agree."""
    import subprocess
    structs = {"tg_problem_desc": tg.ProblemDesc, "tg_assign_out": tg.AssignOut, "tg_trace_desc": tg.TraceDesc,
               "tg_replay_out": tg.ReplayOut}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "tg.h"', 'int main(void) {']
    for cname, st in structs.items():
        lines.append(f'  printf("{cname} %zu\\n", sizeof({cname}));')
        for fname, _ in st._fields_:
            lines.append(f'  printf("{cname}.{fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  printf("tg_summary %zu\\n", sizeof(tg_summary));', '  return 0;', '}']
    src = tmp_path / "offsets.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "offsets"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = dict(l.split() for l in subprocess.check_output([str(exe)], text=True).splitlines())
    for cname, st in structs.items():
        assert int(got[cname]) == C.sizeof(st), cname
        for fname, _ in st._fields_:
            assert int(got[f"{cname}.{fname}"]) == getattr(st, fname).offset, f"{cname}.{fname}"
    assert int(got["tg_summary"]) == tg.SUMMARY_DTYPE.itemsize


def test_struct_layouts_match_header(tg):
    assert C.sizeof(tg.ProblemDesc) == 8 * 4 + 25 * 8 + 6 * 4
    assert C.sizeof(tg.AssignOut) == 9 * 8
    assert C.sizeof(tg.TraceDesc) == 8 * 4 + 8 + 16 * 8 + 2 * 4 + 3 * 8 + 2 * 4
    assert C.sizeof(tg.ReplayOut) == 9 * 8
    assert tg.SUMMARY_DTYPE.itemsize == 8 + 16 + 24 + 24 + 8 + 24


def _build_rc(tg, p):
    d = tg.ProblemDesc()
    for n in ("B", "N", "M", "K", "n_classes", "n_tasks", "depth"):
        setattr(d, n, int(p[n]))
    d.order_policy = int(p.get("order_policy", 0))
    keep = []
    tg._fill(d, p, [f[0] for f in tg.ProblemDesc._fields_[8:-6]], keep)
    d.n_services = int(p.get("n_services", len(p["restore_us"]) if p.get("restore_us") is not None else 0))
    d.numa_cores = int(p.get("numa_cores", 0))
    d.gpu_pooled = int(p.get("gpu_pooled", 0))
    d.queue_prefix = int(p.get("queue_prefix", 0))
    d.nodes_shared = int(p.get("nodes_shared", 0))
    d.reserved_ = int(p.get("reserved_", 0))
    h = C.c_void_p()
    rc = tg.load().tg_build_problem(C.byref(d), None, C.byref(h))
    assert rc != 0 and not h.value
    return rc


BAD = {
    "k_list_not_ascending": (lambda p: p["k_list"].__setitem__(1, 1), -1),
    "unit_above_limit": (lambda p: p["k_list"].__setitem__(3, 65), -1),
    "order_policy": (lambda p: p.__setitem__("order_policy", 2), -1),
    "nodes_shared_flag": (lambda p: p.__setitem__("nodes_shared", 2), -1),
    "reserved_field": (lambda p: p.__setitem__("reserved_", 1), -1),
    "depth": (lambda p: p.__setitem__("depth", 9), -1),
    "free_above_cap": (lambda p: p["node_free"].__setitem__(0, 33), -1),
    "node_kind": (lambda p: p["node_type"].__setitem__(0, 7), -1),
    "model": (lambda p: p["act_model"].__setitem__(5, 3), -1),
    "missing_array": (lambda p: p.__setitem__("act_kmask", None), -1),
    "t_ori_zero": (lambda p: p["act_t_ori_us"].__setitem__(3, 0), -2),
    "t_ori_too_large": (lambda p: p["act_t_ori_us"].__setitem__(3, 1 << 36), -2),
    "backlog_negative": (lambda p: p["node_backlog_us"].__setitem__(1, -1), -2),
    "age_too_large": (lambda p: p["act_age_us"].__setitem__(1, 1 << 40), -2),
    "cpu_node_too_large": (lambda p: p["node_cap"].__setitem__(0, 257), -2),
    "amdahl_fraction": (lambda p: p["act_param"].__setitem__(2, 1_000_001), -3),
    "speedup_decreasing": (lambda p: p["speedup_q16"].__setitem__(1, 65536 // 2), -3),
    "speedup_superlinear": (lambda p: p["speedup_q16"].__setitem__(1, 65536 * 2 + 1), -3),
    "task_out_of_range": (lambda p: p["act_task"].__setitem__(0, 5), -1),
}


@pytest.mark.parametrize("name", list(BAD))
def test_build_rejects(tg, name):
    p = gen.make_config(1)
    p = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    mutate, want = BAD[name]
    mutate(p)
    assert _build_rc(tg, p) == want


def test_build_rejects_gpu_specifics(tg):
    p = gen.make_random_problem(2, B=1, N=10, n_cpu=1, n_gpu=1, n_api=1, shuffle_nodes=False, busy=False)
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    q["node_chunks"][1 * 4 + 0] += 1                       # chunk counts no longer add up to node_free
    assert _build_rc(tg, q) == -1
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    q["k_list"] = np.array([1, 2, 3, 8], np.int32)         # GPU options must be 1, 2, 4, 8
    assert _build_rc(tg, q) == -1
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    api = np.flatnonzero(q["act_type"] == gen.TYPE_API)
    if api.size:
        q["act_model"][api[0]] = 1                         # API actions cannot be elastic
        assert _build_rc(tg, q) == -1


def test_trace_services_are_validated(tg):
    t = gen.make_trace(S=2, A=50, seed=3, contended=True)
    n = t["S"] * t["A"]
    gpu = t["act_type"] == gen.TYPE_GPU
    sv = np.where(gpu, 0, -1).astype(np.int32)
    ok = dict(act_service=sv, restore_us=np.array([5, 6], np.int64), cache_slots=2)
    assert _trace_rc(tg, dict(t, act_service=sv)) == -1                      # both arrays or neither
    assert _trace_rc(tg, dict(t, restore_us=ok["restore_us"])) == -1
    assert _trace_rc(tg, dict(t, **ok, n_services=0)) == -1
    assert _trace_rc(tg, dict(t, **dict(ok, cache_slots=0))) == -1
    assert _trace_rc(tg, dict(t, **dict(ok, cache_slots=65))) == -1
    assert _trace_rc(tg, dict(t, **dict(ok, act_service=np.where(gpu, 2, -1).astype(np.int32)))) == -1   # id out of range
    cpu_calls = sv.copy()
    cpu_calls[np.flatnonzero(~gpu)[0]] = 1
    assert _trace_rc(tg, dict(t, **dict(ok, act_service=cpu_calls))) == -1   # only GPU actions call services
    assert _trace_rc(tg, dict(t, **dict(ok, restore_us=np.array([5, 1 << 36], np.int64)))) == -2


def test_trace_quota_masks_are_validated(tg):
    t = gen.make_trace(S=1, A=60, seed=8, cluster=(1, 8, 1, 3), type_probs=(0.3, 0.2, 0.5), max_ticks=100)
    gen.with_extra_quotas(t, frac=1.0, seed=1)
    api = np.flatnonzero(t["node_type"] == gen.TYPE_API)
    i = int(np.flatnonzero(t["act_quota_mask"] != 0)[0])
    own = int(np.flatnonzero(api == t["act_pin_node"][i])[0])
    m = t["act_quota_mask"].copy(); m[i] |= np.uint64(1 << own)
    assert _trace_rc(tg, dict(t, act_quota_mask=m)) == -1      # the action's own quota
    m = t["act_quota_mask"].copy(); m[i] |= np.uint64(1 << 3)
    assert _trace_rc(tg, dict(t, act_quota_mask=m)) == -1      # a quota the scenario does not have
    c = int(np.flatnonzero(t["act_type"] == gen.TYPE_CPU)[0])
    m = t["act_quota_mask"].copy(); m[c] = np.uint64(1)
    assert _trace_rc(tg, dict(t, act_quota_mask=m)) == -1      # only API actions draw on quotas


def test_second_resource_arrays_come_in_pairs(tg):
    p = gen.make_random_problem(10, B=1, N=30)
    q = dict(p, act_aux=np.zeros(30, np.int32))
    assert _build_rc(tg, q) == -1                              # demand without what the nodes have
    q = dict(p, node_aux_free=np.zeros(p["M"], np.int32))
    assert _build_rc(tg, q) == -1
    q = dict(p, act_aux=np.full(30, -1, np.int32), node_aux_free=np.zeros(p["M"], np.int32))
    assert _build_rc(tg, q) == -1                              # negative demand


def test_service_arrays_are_validated(tg):
    p = gen.make_random_problem(11, B=1, N=30)
    M = p["M"]
    full = dict(act_service=np.zeros(30, np.int32), node_resident=np.zeros(M, np.uint64), restore_us=np.array([5, 6], np.int64))
    for missing in full:
        q = dict(p, **{k: v for k, v in full.items() if k != missing})
        assert _build_rc(tg, dict(q, n_services=2)) == -1      # all three arrays or none
    assert _build_rc(tg, dict(p, **full, n_services=0)) == -1
    assert _build_rc(tg, dict(p, **full, n_services=65)) == -1
    q = dict(p, **full); q["act_service"] = np.full(30, 2, np.int32)
    assert _build_rc(tg, q) == -1                              # service id out of range
    q = dict(p, **full); q["node_resident"] = np.full(M, 4, np.uint64)
    assert _build_rc(tg, q) == -1                              # resident bit of a service that does not exist
    q = dict(p, **full); q["restore_us"] = np.array([5, 1 << 36], np.int64)
    assert _build_rc(tg, q) == -2


def test_core_maps_are_validated(tg):
    p = gen.make_random_problem(12, B=1, N=30, n_cpu=2, n_gpu=1, n_api=1, cpu_cap_hi=40)
    gen.with_core_maps(p, 8, 0)
    for numa in (0, 2, 12, 128):
        assert _build_rc(tg, dict(p, numa_cores=numa)) == -1   # 4, 8, 16, 32 or 64 cores per domain
    assert _build_rc(tg, dict(p, node_core_free=None)) == -1   # a domain size without the maps
    j = int(np.flatnonzero((p["node_type"] == gen.TYPE_CPU) & (p["node_free"] > 0))[0])
    maps = p["node_core_free"].copy().reshape(-1, 4)
    low = int(maps[j][0]) & -int(maps[j][0])
    maps[j][0] = np.uint64(int(maps[j][0]) ^ low)
    assert _build_rc(tg, dict(p, node_core_free=maps.reshape(-1))) == -1      # fewer free cores than node_free
    maps[j][0] = np.uint64(int(maps[j][0]) | low)
    cap = int(p["node_cap"][j])
    moved = maps.copy()
    moved[j][0] = np.uint64(int(moved[j][0]) ^ low)
    moved[j][cap // 64] = np.uint64(int(moved[j][cap // 64]) | 1 << (cap % 64))
    assert _build_rc(tg, dict(p, node_core_free=moved.reshape(-1))) == -1     # a core the node does not have


def test_quota_masks_are_validated(tg):
    p = gen.make_random_problem(13, B=1, N=60, n_cpu=1, n_gpu=1, n_api=3, type_probs=(0.3, 0.2, 0.5))
    gen.with_extra_quotas(p, frac=1.0, seed=0)
    api = np.flatnonzero(p["node_type"] == gen.TYPE_API)
    i = int(np.flatnonzero(p["act_quota_mask"] != 0)[0])
    own = int(np.flatnonzero(api == p["act_pin_node"][i])[0])
    m = p["act_quota_mask"].copy(); m[i] |= np.uint64(1 << own)
    assert _build_rc(tg, dict(p, act_quota_mask=m)) == -1       # the action's own quota
    m = p["act_quota_mask"].copy(); m[i] |= np.uint64(1 << 3)
    assert _build_rc(tg, dict(p, act_quota_mask=m)) == -1       # a quota the snapshot does not have
    c = int(np.flatnonzero(p["act_type"] == gen.TYPE_CPU)[0])
    m = p["act_quota_mask"].copy(); m[c] = np.uint64(1)
    assert _build_rc(tg, dict(p, act_quota_mask=m)) == -1       # only API actions draw on quotas


def test_pooled_gpus_are_validated(tg):
    p = gen.make_random_problem(14, B=1, N=40, n_cpu=1, n_gpu=3, n_api=0, pin_frac=0.0, shuffle_nodes=False)
    g = np.flatnonzero(p["node_type"] == gen.TYPE_GPU)
    p["node_backlog_us"][g] = 0
    p["gpu_pooled"] = 1
    assert _build_rc(tg, dict(p, gpu_pooled=2)) == -1
    assert _build_rc(tg, dict(p, gpu_pooled=0, queue_prefix=2)) == -1
    assert _build_rc(tg, dict(p, gpu_pooled=0, queue_prefix=-1)) == -1
    q = dict(p); q["node_backlog_us"] = p["node_backlog_us"].copy(); q["node_backlog_us"][g[1]] = 5
    assert _build_rc(tg, q) == -1                               # a pool has one backlog
    q = dict(p); q["act_pin_node"] = p["act_pin_node"].copy()
    q["act_pin_node"][int(np.flatnonzero(p["act_type"] == gen.TYPE_GPU)[0])] = int(g[0])
    assert _build_rc(tg, q) == -1                               # no GPU action pinned to a node of the pool
    q = dict(p); q["node_cap"] = p["node_cap"].copy(); q["node_cap"][g[2]] = 16
    assert _build_rc(tg, q) == -1                               # nodes of 8 GPUs
    q = dict(p, act_service=np.full(40, -1, np.int32), node_resident=np.zeros(p["M"], np.uint64),
             restore_us=np.array([5], np.int64))
    assert _build_rc(tg, q) == -1                               # services need per-node residency
    big = gen.make_random_problem(15, B=1, N=40, n_cpu=0, n_gpu=9, n_api=0, pin_frac=0.0, bad_frac=0.0)
    big["node_backlog_us"][:] = 0
    assert _build_rc(tg, dict(big, gpu_pooled=1)) == -2         # more than 64 GPUs in one pool


def test_null_arguments(tg):
    L = tg.load()
    assert L.tg_step(None, None, None, None, 0, None) == -1
    assert L.tg_build_problem(None, None, None) == -1
    assert L.tg_num_candidates(None, None, None) == -1
    assert L.tg_assign_workspace_bytes(None, None) == -1
    assert L.tg_score_candidates(None, None, None) == -1
    assert L.tg_assign(None, None, None, None, 0, None) == -1
    assert L.tg_build_trace(None, None, None) == -1
    assert L.tg_replay_workspace_bytes(None, None) == -1
    assert L.tg_replay_trace(None, None, None, 0, None) == -1
    L.tg_free_problem(None)
    L.tg_free_trace(None)


def _trace_rc(tg, t):
    d = tg.TraceDesc()
    for n in ("S", "A", "M", "K", "n_classes", "depth", "max_ticks"):
        setattr(d, n, int(t[n]))
    d.flags = int(t.get("flags", 0))
    d.tick_us = int(t["tick_us"])
    keep = []
    tg._fill(d, t, [f[0] for f in tg.TraceDesc._fields_[9:-7]] + ["act_quota_mask", "node_aux", "act_aux"], keep)
    d.numa_cores = int(t.get("numa_cores", 0))
    d.order_policy = int(t.get("order_policy", 0))
    d.n_services = int(t.get("n_services", len(t["restore_us"]) if t.get("restore_us") is not None else 0))
    d.cache_slots = int(t.get("cache_slots", 64))
    h = C.c_void_p()
    rc = tg.load().tg_build_trace(C.byref(d), None, C.byref(h))
    assert rc != 0 and not h.value
    return rc


BAD_TRACE = {
    "arrivals_not_sorted": (lambda t: t["arrival_us"].__setitem__(5, 0), -1),
    "gpu_node_not_8": (lambda t: t["node_cap"].__setitem__(int(np.flatnonzero(t["node_type"] == gen.TYPE_GPU)[0]), 4), -1),
    "tick_zero": (lambda t: t.__setitem__("tick_us", 0), -1),
    "unknown_flag": (lambda t: t.__setitem__("flags", 8), -1),
    "pooled_gpus_with_a_pinned_gpu_action": (lambda t: (t.__setitem__("flags", 2), t["act_type"].__setitem__(7, 1), t["act_kmask"].__setitem__(7, 1),
                                                        t["act_model"].__setitem__(7, 0),
                                                        t["act_pin_node"].__setitem__(7, int(np.flatnonzero(t["node_type"] == gen.TYPE_GPU)[0]))), -1),
    "pooled_gpus_with_services": (lambda t: (t.__setitem__("flags", 2), gen.trace_with_services(t, 1, 4, 2)), -1),
    "pooled_gpus_with_a_second_resource": (lambda t: (t.__setitem__("flags", 2), gen.trace_with_aux(t, 1, False)), -1),
    "numa_domain_not_a_power_of_two": (lambda t: t.__setitem__("numa_cores", 12), -1),
    "numa_domain_too_small": (lambda t: t.__setitem__("numa_cores", 2), -1),
    "second_resource_half_given": (lambda t: t.__setitem__("node_aux", np.ones(t["S"] * t["M"], np.int32)), -1),
    "second_resource_negative": (lambda t: (t.__setitem__("node_aux", np.ones(t["S"] * t["M"], np.int32)),
                                            t.__setitem__("act_aux", np.full(t["S"] * t["A"], -1, np.int32))), -1),
    "unknown_flag_next_to_a_known_one": (lambda t: t.__setitem__("flags", 9), -1),
    "unknown_visiting_order": (lambda t: t.__setitem__("order_policy", 2), -1),
    "tokens_above_bucket": (lambda t: t["quota_tok0_micro"].__setitem__(int(np.flatnonzero(t["node_type"] == gen.TYPE_API)[0]), 10**12), -1),
    "t_ori_range": (lambda t: t["act_t_ori_us"].__setitem__(0, 0), -2),
    "class_out_of_range": (lambda t: (t["act_model"].__setitem__(0, 2), t["act_param"].__setitem__(0, 99), t["act_type"].__setitem__(0, 1)), -3),
}


@pytest.mark.parametrize("name", list(BAD_TRACE))
def test_build_trace_rejects(tg, name):
    t = gen.make_trace(S=2, A=50, seed=3, contended=True)
    t = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in t.items()}
    t["arrival_us"][5] = max(int(t["arrival_us"][5]), 1)
    mutate, want = BAD_TRACE[name]
    mutate(t)
    assert _trace_rc(tg, t) == want
