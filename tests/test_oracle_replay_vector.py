"""Pins for the second resource (Sec. 4.1: the cost of an action is a vector; Sec. 5.2: memory next to cores) in the
trace replay: an action that is free to choose its node holds its demand from start to finish, pinned actions hold
none.  An integer tick simulation on one node, cases in which the resource cannot bind, and the running totals re-derived
from the oracle's own start and finish times."""
import numpy as np
import pytest

import gen


def _with_aux(t, seed, cap_lo, cap_hi, need_hi=40):
    rng = np.random.default_rng(seed + 77)
    t["act_aux"] = rng.integers(0, need_hi, t["S"] * t["A"]).astype(np.int32)
    t["node_aux"] = rng.integers(cap_lo, cap_hi, t["S"] * t["M"]).astype(np.int32)
    return t


@pytest.mark.parametrize("seed", range(5))
def test_one_node_against_an_integer_simulation(orc, seed):
    """One node with more cores than actions, one core per action, nothing elastic, nothing pinned: per tick the queue
    is admitted in order while the running total of the second resource fits; the first misfit closes it."""
    A = 120
    t = gen.make_trace(S=2, A=A, seed=130 + seed, cluster=(1, 200, 0, 0), type_probs=(1, 0, 0), rate_per_s=60.0,
                       horizon_s=2.0, max_ticks=100_000, pin_frac=0.0, cpu_median=900_000)
    t["act_model"][:] = 0
    t["act_kmask"][:] = 1
    _with_aux(t, seed, 60, 120)
    o = orc.replay(t)
    tick = int(t["tick_us"])
    waited = False
    for s in range(2):
        arr, T, need = t["arrival_us"][s * A:(s + 1) * A], t["act_t_ori_us"][s * A:(s + 1) * A], t["act_aux"][s * A:(s + 1) * A]
        rem = int(t["node_aux"][s])
        start = np.full(A, -1, np.int64)
        running, waiting, nxt, n = [], [], 0, 0
        while (start < 0).any() and n < 100_000:
            now = n * tick
            rem += sum(a for f, a in running if f <= now)
            running = [(f, a) for f, a in running if f > now]
            while nxt < A and arr[nxt] <= now:
                waiting.append(nxt)
                nxt += 1
            while waiting and need[waiting[0]] <= rem:
                i = waiting.pop(0)
                start[i] = now
                rem -= int(need[i])
                running.append((now + int(T[i]), int(need[i])))
            waited |= bool(waiting)
            n += 1
        np.testing.assert_array_equal(o["start_us"][s * A:(s + 1) * A], start, err_msg=f"scenario {s}")
    assert waited, "the second resource should make somebody wait"


def test_cases_in_which_it_cannot_bind(orc):
    t = gen.make_trace(S=2, A=300, seed=140, contended=True, rate_per_s=80.0, horizon_s=4.0, max_ticks=20000)
    base = orc.replay(t)
    roomy = orc.replay(_with_aux(dict(t), 1, 10**6, 10**6 + 1))
    for k in base:
        np.testing.assert_array_equal(base[k], roomy[k], err_msg=k)
    # everybody pinned: trajectories whose share was taken before the trace began - nothing is charged, even with none left
    M = t["M"]
    q = dict(t)
    q["act_pin_node"] = t["act_pin_node"].copy()
    for s in range(2):
        for ty in (gen.TYPE_CPU, gen.TYPE_GPU):
            nodes = np.flatnonzero(t["node_type"][s * M:(s + 1) * M] == ty)
            a = np.flatnonzero((t["act_type"][s * 300:(s + 1) * 300] == ty) & (q["act_pin_node"][s * 300:(s + 1) * 300] < 0)) + s * 300
            q["act_pin_node"][a] = nodes[a % len(nodes)]
    pinned = orc.replay(q)
    none_left = orc.replay(dict(_with_aux(dict(q), 2, 0, 1)))
    for k in pinned:
        np.testing.assert_array_equal(pinned[k], none_left[k], err_msg=k)


@pytest.mark.parametrize("seed", range(6))
def test_running_totals_from_the_oracles_own_times(orc, seed):
    """At every start the demands of the unpinned actions running on the node, the new one included, fit the node;
    and a scarce resource delays somebody."""
    A = 400
    t = gen.make_trace(S=2, A=A, seed=150 + seed, cluster=(3, 16, 2, 2), rate_per_s=90.0, horizon_s=4.5, max_ticks=50_000,
                       pin_frac=(0.0, 0.4)[seed % 2])
    plain = orc.replay(t)
    _with_aux(t, seed, 30, 90)
    o = orc.replay(t)
    M = t["M"]
    for s in range(2):
        sl = slice(s * A, (s + 1) * A)
        st, fin, nd = o["start_us"][sl], o["finish_us"][sl], o["node"][sl]
        held = np.where((t["act_pin_node"][sl] < 0) & (t["act_type"][sl] != gen.TYPE_API), t["act_aux"][sl], 0)
        for i in np.flatnonzero(st >= 0):
            together = (nd == nd[i]) & (st >= 0) & (st <= st[i]) & (fin > st[i])
            assert held[together].sum() <= t["node_aux"][s * M + nd[i]], (s, i)
    assert (plain["start_us"] != o["start_us"]).any()
