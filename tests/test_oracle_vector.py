"""Pins for the oracle's second, co-constrained resource (Sec. 4.1: an action's cost is a vector;
Sec. 5.2: a node needs the cores for the action and the memory for the trajectory when the
trajectory's first action is placed): a closed form, and the whole admission / node-choice loop
re-run by an independent Python simulator with exact rational durations (which also pins the
loop without the second resource)."""
from fractions import Fraction

import numpy as np
import pytest

import gen
import pyref

INF = pyref.INF


def _dur(p, g, q):
    K = p["K"]
    sp = int(p["speedup_q16"][int(p["act_param"][g]) * K + q]) if p["act_model"][g] == 2 else 0
    return pyref.duration(int(p["act_model"][g]), int(p["act_t_ori_us"][g]), int(p["act_param"][g]),
                          int(p["k_list"][q]), sp)


def _options(p, g):
    t = int(p["act_type"][g])
    qs = [q for q in range(int(p["type_k"][t])) if p["act_kmask"][g] >> q & 1]
    return qs[:1] if p["act_model"][g] == 0 else qs


def restore_delay(p, g, n):
    """Sec. 5.3: a service that is not resident on the node is restored before the action runs."""
    if p.get("act_service") is None or p["act_service"][g] < 0:
        return 0
    s = int(p["act_service"][g])
    return 0 if int(p["node_resident"][n]) >> s & 1 else int(p["restore_us"][s])


def _place(p, b):
    """Admission and node choice of one snapshot without GPU nodes: returns (home, reason) with
    reason 0 admitted, 1 deferred behind a misfit, 3 never feasible."""
    N, M = p["N"], p["M"]
    nt = p["node_type"][b * M:(b + 1) * M]
    cap = p["node_cap"][b * M:(b + 1) * M]
    rem = p["node_free"][b * M:(b + 1) * M].astype(np.int64).copy()
    back = p["node_backlog_us"][b * M:(b + 1) * M]
    aux_rem = (p["node_aux_free"][b * M:(b + 1) * M].astype(np.int64).copy() if p.get("node_aux_free") is not None
               else np.full(M, 1 << 40))
    home, reason = np.full(N, -1), np.zeros(N, int)
    api = [j for j in range(M) if nt[j] == gen.TYPE_API][:64]
    closed, type_closed = set(), set()
    whole_queue = bool(p.get("queue_prefix", 0))                # one prefix of the whole queue instead of one per pool
    for i in range(N):
        g = b * N + i
        t, pin = int(p["act_type"][g]), int(p["act_pin_node"][g])
        ops = _options(p, g)
        nodes = [pin] if pin >= 0 else list(range(M))
        feasible = bool(ops) and any(0 <= j < M and nt[j] == t and p["k_list"][ops[0]] <= cap[j] for j in nodes)
        if not feasible:
            reason[i] = 3
            continue
        if t in type_closed or (pin >= 0 and pin in closed) or (whole_queue and (closed or type_closed)):
            reason[i] = 1
            continue
        kmin = int(p["k_list"][ops[0]])
        aux = int(p["act_aux"][g]) if p.get("act_aux") is not None and pin < 0 else 0
        more = [api[r] for r in range(len(api)) if int(p["act_quota_mask"][g]) >> r & 1] if p.get("act_quota_mask") is not None else []
        best = None
        for j in nodes:
            if nt[j] != t or j in closed or rem[j] < kmin or aux > aux_rem[j] or any(rem[x] < 1 for x in more):
                continue
            q = max(q for q in ops if p["k_list"][q] <= cap[j] and p["k_list"][q] <= rem[j])
            e = (int(back[j]) + restore_delay(p, g, b * M + j) + _dur(p, g, q), j)
            best = e if best is None or e < best else best
        if best is None:
            reason[i] = 1
            (closed.add(pin) if pin >= 0 else type_closed.add(t))
            continue
        j = best[1]
        home[i] = j
        rem[j] -= kmin
        aux_rem[j] -= aux
        for x in more:
            rem[x] -= 1
    return home, reason


def _with_aux(p, seed, scarce):
    rng = np.random.default_rng(seed)
    p["act_aux"] = rng.integers(0, 40, p["B"] * p["N"]).astype(np.int32)
    hi = 120 if scarce else 4000
    p["node_aux_free"] = rng.integers(0, hi, p["B"] * p["M"]).astype(np.int32)
    return p


@pytest.mark.parametrize("seed", range(16))
def test_admission_loop_rerun_in_python(orc, seed):
    p = gen.make_random_problem(300 + seed, B=3, N=60 + 10 * seed, n_cpu=2 + seed % 4, n_gpu=0, n_api=seed % 3,
                                busy=False, cpu_cap_hi=16 + 8 * (seed % 3), pin_frac=0.3)
    p["type_k"][gen.TYPE_GPU] = 0
    a = (p["act_type"] == gen.TYPE_CPU)
    p["act_kmask"][a] |= 1
    if seed % 4:                                                # every fourth case: no second resource at all
        _with_aux(p, seed, scarce=seed % 2 == 0)
    o = orc.assign(p)
    N = p["N"]
    for b in range(p["B"]):
        home, reason = _place(p, b)
        np.testing.assert_array_equal(o["home"][b * N:(b + 1) * N], home, err_msg=f"snapshot {b} home")
        got = o["reason"][b * N:(b + 1) * N]
        np.testing.assert_array_equal(got == 3, reason == 3)
        np.testing.assert_array_equal(got == 1, reason == 1)
    if seed % 4:
        q = dict(p); q["act_aux"] = None; q["node_aux_free"] = None
        assert (orc.assign(q)["home"] != o["home"]).any() or seed % 2, "a scarce second resource should change the placement"


def test_second_resource_closes_the_prefix_on_one_node(orc):
    """One node with plenty of cores, one unit per action, nothing elastic, nothing pinned: actions are
    admitted while their running total of the second resource fits; the first that does not closes the pool."""
    N = 12
    p = gen.subset_problem(gen.make_config(1), 0, N, n_cpu_nodes=1, cap=16)
    p["act_model"][:] = 0
    p["act_pin_node"][:] = -1
    need = np.array([5, 7, 1, 9, 3, 3, 8, 2, 6, 4, 1, 1], np.int32)
    p["act_aux"] = need
    for have in (0, 4, 5, 13, 22, 25, 100):
        p["node_aux_free"] = np.array([have], np.int32)
        o = orc.assign(p)
        n_fit = int((np.cumsum(need) <= have).sum())
        assert list(o["reason"]) == [0] * n_fit + [1] * (N - n_fit)
    p["act_pin_node"][:] = 0                                    # trajectories already on the node: not charged again
    p["node_aux_free"] = np.array([0], np.int32)
    assert (orc.assign(p)["reason"] == 0).all()


@pytest.mark.parametrize("seed", range(8))
def test_second_resource_is_never_oversubscribed(orc, seed):
    p = _with_aux(gen.make_random_problem(340 + seed, B=3, N=200, n_cpu=3, n_gpu=2, n_api=1, cpu_cap_hi=48), seed, scarce=True)
    o = orc.assign(p)
    N, M = p["N"], p["M"]
    for b in range(p["B"]):
        used = np.zeros(M, np.int64)
        for i in range(N):
            g = b * N + i
            if o["home"][g] >= 0 and p["act_pin_node"][g] < 0:
                used[o["home"][g]] += p["act_aux"][g]
        assert (used <= p["node_aux_free"][b * M:(b + 1) * M]).all()
