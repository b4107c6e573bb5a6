"""Pins for the oracle's whole-queue prefix (Alg. 1 as printed: the admitted candidates are the
longest prefix of the waiting queue that the resources accommodate, so the first action that
does not fit stops the admission for every kind of resource).  A closed form on two resources,
the admission loop re-run by the independent Python simulator, the step against the per-pool
step on a problem whose tail was made inert by hand, the cost order through relabelling, and
invariants of the visiting order."""
import numpy as np
import pytest

import gen
from test_oracle_order import _keys, _relabel
from test_oracle_pooled import _pooled_problem
from test_oracle_service import _with_services
from test_oracle_vector import _place, _with_aux


def _first_blocked(reason):
    w = np.flatnonzero(reason == 1)
    return int(w[0]) if len(w) else len(reason)


def test_two_resources_one_prefix_closed_form(orc):
    """One CPU node with `free` cores and one quota with `tok` tokens, one unit per action, nothing
    elastic: per pool the first `free` CPU actions and the first `tok` API actions are admitted; with one
    prefix over the whole queue the admission ends at the first action whose own running count runs over."""
    rng = np.random.default_rng(5)
    N = 40
    p = gen.make_random_problem(77, B=1, N=N, n_cpu=1, n_gpu=0, n_api=1, bad_frac=0.0, pin_frac=0.0, busy=False)
    is_api = rng.random(N) < 0.4
    p["act_type"][:] = np.where(is_api, gen.TYPE_API, gen.TYPE_CPU)
    p["act_model"][:] = 0
    p["act_kmask"][:] = 1
    p["act_pin_node"][:] = np.where(is_api, int(np.flatnonzero(p["node_type"] == gen.TYPE_API)[0]), -1)
    cpu, api = int(np.flatnonzero(p["node_type"] == gen.TYPE_CPU)[0]), int(np.flatnonzero(p["node_type"] == gen.TYPE_API)[0])
    p["node_cap"][cpu] = 64
    p["node_cap"][api] = 64
    n_cpu_before, n_api_before = np.cumsum(~is_api), np.cumsum(is_api)          # inclusive running counts
    for free, tok in ((0, 5), (3, 0), (4, 6), (10, 2), (30, 30), (7, 7)):
        p["node_free"][cpu], p["node_free"][api] = free, tok
        per_pool = np.where(is_api, n_api_before <= tok, n_cpu_before <= free)
        o = orc.assign(p)
        np.testing.assert_array_equal(o["reason"] == 0, per_pool)
        n = _first_blocked(np.where(per_pool, 0, 1))
        w = orc.assign(dict(p, queue_prefix=1))
        np.testing.assert_array_equal(w["reason"], np.where(np.arange(N) < n, 0, 1))
        np.testing.assert_array_equal(w["node"][:n], o["node"][:n])
        np.testing.assert_array_equal(w["act_us"][:n], o["act_us"][:n])
        assert int(w["summary"]["n_assigned"][0]) == n and int(w["summary"]["n_prefix"][0]) == N - n


@pytest.mark.parametrize("seed", range(12))
def test_admission_loop_rerun_in_python(orc, seed):
    p = gen.make_random_problem(900 + seed, B=3, N=60 + 10 * seed, n_cpu=2 + seed % 4, n_gpu=0, n_api=1 + seed % 3,
                                busy=False, cpu_cap_hi=24 + 8 * (seed % 3), pin_frac=0.3)
    p["type_k"][gen.TYPE_GPU] = 0
    p["act_kmask"][p["act_type"] == gen.TYPE_CPU] |= 1
    if seed % 3 == 1:
        _with_aux(p, seed, scarce=False)
    if seed % 3 == 2:
        gen.with_extra_quotas(p, 0.5, seed)
    p["queue_prefix"] = 1
    o = orc.assign(p)
    N = p["N"]
    blocked_somewhere = False
    for b in range(p["B"]):
        home, reason = _place(p, b)
        np.testing.assert_array_equal(o["home"][b * N:(b + 1) * N], home, err_msg=f"snapshot {b} home")
        got = o["reason"][b * N:(b + 1) * N]
        np.testing.assert_array_equal(got == 3, reason == 3)
        np.testing.assert_array_equal(got == 1, reason == 1)
        n = _first_blocked(reason)
        blocked_somewhere |= n < N
        assert ((reason[n:] == 1) | (reason[n:] == 3)).all()
    assert blocked_somewhere
    assert (orc.assign(dict(p, queue_prefix=0))["home"] != o["home"]).any(), "the whole-queue prefix should bind here"


def _inert_tail(p, first):
    """The problem with every action at or behind first[b] made unschedulable by hand (no allowed
    option): such actions take part in nothing."""
    q = dict(p)
    q["act_kmask"] = p["act_kmask"].copy()
    N = p["N"]
    for b in range(p["B"]):
        q["act_kmask"][b * N + first[b]:(b + 1) * N] = 0
    return q


@pytest.mark.parametrize("seed", range(10))
def test_step_equals_per_pool_step_without_the_tail(orc, seed):
    """Up to the first action that does not fit nothing is closed, so both rules admit the same actions
    to the same nodes; behind it the whole-queue rule admits nobody.  With nothing pinned the waiting
    tail enters no node's estimate, so the whole step must equal the per-pool step on a problem whose
    tail cannot be scheduled at all.  Every second case pins actions but has nothing elastic (then no
    node runs the eviction loop and the waiting tail does not matter either)."""
    pins = seed % 2 == 1
    p = gen.make_random_problem(940 + seed, B=4, N=150 + 20 * seed, n_cpu=2 + seed % 3, n_gpu=1 + seed % 3, n_api=seed % 3,
                                busy=seed % 3 == 0, cpu_cap_hi=32, pin_frac=0.3 if pins else 0.0,
                                bad_frac=0.0 if not pins else 0.02)
    if pins:
        p["act_model"][:] = 0
    if seed % 4 == 2:
        _with_services(p, seed)
    plain = orc.assign(p)
    N, M = p["N"], p["M"]
    first = [_first_blocked(plain["reason"][b * N:(b + 1) * N]) for b in range(p["B"])]
    assert any(f < N for f in first)
    w = orc.assign(dict(p, queue_prefix=1))
    ref = orc.assign(_inert_tail(p, first))
    for b in range(p["B"]):
        s, f = slice(b * N, b * N + first[b]), first[b]
        for k in ("node", "units", "act_us", "reason"):
            np.testing.assert_array_equal(w[k][s], ref[k][s], err_msg=f"{k} snapshot {b}")
        tail = w["reason"][b * N + f:(b + 1) * N]
        assert ((tail == 1) | (tail == 3)).all()
        np.testing.assert_array_equal(tail == 3, plain["reason"][b * N + f:(b + 1) * N] == 3)
        assert (w["node"][b * N + f:(b + 1) * N] == -1).all() and (w["units"][b * N + f:(b + 1) * N] == 0).all()
    np.testing.assert_array_equal(w["node_obj"], ref["node_obj"])
    np.testing.assert_array_equal(w["node_used"], ref["node_used"])
    for k in ("sum_act_us", "n_assigned", "n_evicted"):
        np.testing.assert_array_equal(w["summary"][k], ref["summary"][k], err_msg=k)


@pytest.mark.parametrize("seed", range(8))
def test_cost_order_is_fcfs_on_the_relabelled_problem(orc, seed):
    """Under the cost order the one prefix is a prefix of the whole queue sorted by (key, FCFS rank)."""
    p = gen.make_random_problem(970 + seed, B=3, N=60 + 5 * seed, n_cpu=2 + seed % 2, n_gpu=seed % 3, n_api=1 + seed % 2,
                                depth=1 + seed % 2, busy=seed % 2 == 0, cpu_cap_hi=20 + 4 * (seed % 3))
    p["queue_prefix"] = 1
    key = _keys(p)
    N = p["N"]
    perm = [sorted(range(N), key=lambda i, b=b: (key[b * N + i], i)) for b in range(p["B"])]
    q, idx = _relabel(p, perm)
    want = orc.assign(q)
    got = orc.assign(dict(p, order_policy=1))
    for k in ("node", "units", "act_us", "reason"):
        np.testing.assert_array_equal(got[k][idx], want[k], err_msg=k)
    np.testing.assert_array_equal(got["node_obj"], want["node_obj"])
    np.testing.assert_array_equal(got["node_used"], want["node_used"])
    per_pool = orc.assign(dict(p, order_policy=1, queue_prefix=0))
    assert (per_pool["reason"] != got["reason"]).any()


def test_ample_capacity_changes_nothing(orc):
    p = gen.make_random_problem(990, B=3, N=40, n_cpu=6, n_gpu=8, n_api=2, cpu_cap_hi=128, bad_frac=0.02, pin_frac=0.0,
                                type_probs=(0.75, 0.1, 0.15))
    p["node_free"][:] = p["node_cap"]
    if p.get("node_chunks") is not None:
        p["node_chunks"] = None
    p["node_busy_off"], p["node_busy_rel_us"] = None, None
    api = p["node_type"] == gen.TYPE_API
    p["node_cap"][api] = 1000
    p["node_free"][api] = 1000
    a = orc.assign(p)
    assert not (a["reason"] == 1).any()
    for order in (0, 1):
        x, y = orc.assign(dict(p, order_policy=order)), orc.assign(dict(p, order_policy=order, queue_prefix=1))
        for k in ("node", "units", "act_us", "reason", "node_obj", "node_used"):
            np.testing.assert_array_equal(x[k], y[k], err_msg=k)


@pytest.mark.parametrize("seed", range(10))
def test_nobody_is_admitted_behind_a_waiting_action(orc, seed):
    """Every feature switched on at random: in visiting order no admitted action (selected or evicted
    from its node's tail) follows one that waits because of the prefix rule."""
    if seed % 2:
        p = _pooled_problem(1000 + seed, 2 + seed % 3, N=200)
    else:
        p = gen.make_random_problem(1000 + seed, B=4, N=200, n_cpu=3, n_gpu=2, n_api=2, cpu_cap_hi=48, pin_frac=0.25)
        if seed % 4 == 0:
            _with_services(p, seed)
    p["queue_prefix"] = 1
    for order in (0, 1):
        o = orc.assign(dict(p, order_policy=order))
        key = _keys(p) if order else None
        N = p["N"]
        for b in range(p["B"]):
            visit = sorted(range(N), key=lambda i: (key[b * N + i], i)) if order else range(N)
            r = o["reason"][b * N:(b + 1) * N][list(visit)]
            n = _first_blocked(r)
            assert not np.isin(r[n:], (0, 2)).any()
            assert not (r[:n] == 1).any()


def head_problem(seed=5):
    """One node with 8 free cores; the head scales badly (10 s on one core, 9.9 s on eight); behind it an API action
    finds no token, which ends the whole-queue prefix, so seven one-second actions pinned to the node wait."""
    p = gen.make_random_problem(seed, B=1, N=9, n_cpu=1, n_gpu=0, n_api=1, bad_frac=0.0, pin_frac=0.0, busy=False, k_list=(1, 2, 4, 8))
    p["type_k"][gen.TYPE_GPU] = 0
    cpu = int(np.flatnonzero(p["node_type"] == gen.TYPE_CPU)[0])
    api = int(np.flatnonzero(p["node_type"] == gen.TYPE_API)[0])
    p["node_cap"][cpu] = p["node_free"][cpu] = 8
    p["node_cap"][api], p["node_free"][api] = 4, 0
    p["node_backlog_us"][:] = 0
    p["act_age_us"][:] = 0
    p["act_type"][:] = gen.TYPE_CPU
    p["act_type"][1] = gen.TYPE_API
    p["act_pin_node"][:] = cpu
    p["act_pin_node"][1] = api
    p["act_model"][:] = 0
    p["act_kmask"][:] = 1
    p["act_t_ori_us"][:] = 1_000_000
    p["act_model"][0], p["act_kmask"][0], p["act_t_ori_us"][0] = 1, 0b1111, 10_000_000
    p["act_param"][0] = 11_429                                  # parallel fraction in ppm: 10 s -> 9.9 s on eight cores
    p["queue_prefix"], p["depth"] = 1, 2
    return p, cpu


@pytest.mark.parametrize("seed", [5, 7])                        # the CPU node is node 1 / node 0 of the snapshot
def test_the_head_of_a_node_is_never_evicted(orc, seed):
    """Alg. 1's eviction loop stops at one candidate even where keeping nobody would look better (every step must make
    progress).  DPArrange gives the head all eight cores: 9.9 + 7 * 10.9 = 86.2 s with the seven waiting behind it.
    Keeping nobody would estimate the head on one core next to the seven, 10 + 7 * 1 = 17 s - less, and still the head
    stays."""
    p, cpu = head_problem(seed)
    assert cpu == (1 if seed == 5 else 0)
    d8 = orc.duration(1, 10_000_000, 11_429, 8)
    assert 9_899_000 < d8 < 9_901_000
    o = orc.assign(p)
    assert list(o["reason"]) == [0] + [1] * 8
    assert o["units"][0] == 8 and o["act_us"][0] == d8
    assert o["node_obj"][cpu] == d8 + 7 * (d8 + 1_000_000)
    assert 10_000_000 + 7 * 1_000_000 < o["node_obj"][cpu]
