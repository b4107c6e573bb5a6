"""Pins for the oracle's second visiting order (Sec. 4.2: the algorithm works with other
ordering algorithms; ORDER_COST = ascending least estimated ACT over an action's candidates,
ties in FCFS rank).  The keys are recomputed here from Eq. 1 / Eq. 2 with exact rationals, the
problem is relabelled so that FCFS order *is* the cost order, and the FCFS oracle (pinned
elsewhere) must then agree with the cost-ordered oracle action by action; plus two closed forms."""
import numpy as np
import pytest

import gen
import pyref

INF = pyref.INF
PER_ACTION = ("act_type", "act_model", "act_t_ori_us", "act_age_us", "act_kmask", "act_param", "act_pin_node", "act_task",
              "act_aux", "act_service")


def _dur(p, g, q):
    K = p["K"]
    sp = int(p["speedup_q16"][int(p["act_param"][g]) * K + q]) if p["act_model"][g] == 2 else 0
    return pyref.duration(int(p["act_model"][g]), int(p["act_t_ori_us"][g]), int(p["act_param"][g]),
                          int(p["k_list"][q]), sp)


def _keys(p):
    """Least finite entry of every action's row of the score tensor (Eq. 2), INF if it has none."""
    B, N, M = p["B"], p["N"], p["M"]
    key = np.full(B * N, INF, dtype=object)
    for b in range(B):
        for i in range(N):
            g = b * N + i
            t = int(p["act_type"][g])
            qs = [q for q in range(int(p["type_k"][t])) if p["act_kmask"][g] >> q & 1]
            if p["act_model"][g] == 0:
                qs = qs[:1]                                    # a non-elastic action only has its minimum
            pin = int(p["act_pin_node"][g])
            for j in range(M):
                n = b * M + j
                if p["node_type"][n] != t or (pin >= 0 and pin != j):
                    continue
                extra = 0                                   # Sec. 5.3: restore a service that is not resident on the node
                if p.get("act_service") is not None and p["act_service"][g] >= 0:
                    sv = int(p["act_service"][g])
                    extra = 0 if int(p["node_resident"][n]) >> sv & 1 else int(p["restore_us"][sv])
                for q in qs:
                    if p["k_list"][q] <= p["node_cap"][n]:
                        key[g] = min(key[g], int(p["node_backlog_us"][n]) + extra + _dur(p, g, q))
    return key


def _relabel(p, perm):
    """perm[b][r] = old index of the action that gets rank r in snapshot b."""
    q = dict(p)
    N = p["N"]
    idx = np.concatenate([b * N + np.asarray(perm[b]) for b in range(p["B"])])
    for k in PER_ACTION:
        if p.get(k) is not None:
            q[k] = np.ascontiguousarray(p[k][idx])
    return q, idx


@pytest.mark.parametrize("seed", range(12))
def test_cost_order_is_fcfs_on_the_relabelled_problem(orc, seed):
    p = gen.make_random_problem(100 + seed, B=3, N=50 + 5 * seed, n_cpu=2 + seed % 2, n_gpu=seed % 3, n_api=seed % 2,
                                depth=1 + seed % 2, busy=seed % 2 == 0, cpu_cap_hi=20 + 4 * (seed % 3))
    key = _keys(p)
    N = p["N"]
    perm = [sorted(range(N), key=lambda i, b=b: (key[b * N + i], i)) for b in range(p["B"])]
    assert any(pm != list(range(N)) for pm in perm), "the case should reorder something"
    q, idx = _relabel(p, perm)
    want = orc.assign(q)                                       # FCFS on the relabelled problem
    got = orc.assign(dict(p, order_policy=1))                  # cost order on the original
    for k in ("node", "units", "act_us", "reason"):
        np.testing.assert_array_equal(got[k][idx], want[k], err_msg=k)
    np.testing.assert_array_equal(got["node_obj"], want["node_obj"])
    np.testing.assert_array_equal(got["node_used"], want["node_used"])
    for k in ("sum_act_us", "n_assigned", "n_prefix", "n_evicted", "n_infeasible"):
        np.testing.assert_array_equal(got["summary"][k], want["summary"][k], err_msg=k)
    fcfs = orc.assign(p)
    assert any((fcfs[k] != got[k]).any() for k in ("node", "units", "reason")), "the order should matter here"


def test_cost_order_admits_the_shortest_on_one_node(orc):
    """One node, one unit per action, nothing elastic: the admitted set is the `free` shortest
    actions, each finishing after backlog + its duration (closed form); FCFS admits the first."""
    N = 12
    p = gen.subset_problem(gen.make_config(1), 0, N, n_cpu_nodes=1, cap=16)
    p["act_model"][:] = 0
    p["node_backlog_us"][:] = 7_000
    T = p["act_t_ori_us"].astype(np.int64)
    assert len(set(T.tolist())) == N
    for free in (0, 1, 4, 11, 12, 16):
        p["node_free"][:] = free
        o = orc.assign(dict(p, order_policy=1))
        short = np.argsort(T, kind="stable")[:min(free, N)]
        sel = np.zeros(N, bool)
        sel[short] = True
        np.testing.assert_array_equal(o["reason"] == 0, sel)
        np.testing.assert_array_equal(o["act_us"][sel], p["act_age_us"][sel] + 7_000 + T[sel])
        assert int(o["summary"]["sum_act_us"][0]) == int((p["act_age_us"][sel] + 7_000 + T[sel]).sum())
        f = orc.assign(p)
        np.testing.assert_array_equal(f["reason"] == 0, np.arange(N) < min(free, N))
        if 0 < free < N:                                       # the shortest `free` can only lower the sum of durations
            assert T[sel].sum() <= T[:free].sum()


def test_cost_order_with_equal_keys_is_fcfs(orc):
    p = gen.make_random_problem(8, B=2, N=120, n_cpu=4, n_gpu=2, n_api=0, bad_frac=0.0, pin_frac=0.0)
    p["act_t_ori_us"][:] = 1_000_000
    p["act_model"][:] = 1
    p["act_param"][:] = 900_000
    p["act_kmask"][:] = np.where(p["act_type"] == gen.TYPE_GPU, 0b0111, 0b1111)
    p["node_backlog_us"][:] = 0
    a, b = orc.assign(p), orc.assign(dict(p, order_policy=1))
    for k in ("node", "units", "act_us", "reason", "node_obj"):
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)
