"""Pins for the whole-queue prefix (Alg. 1 as printed) in the trace replay: cores and tokens against an
independent integer simulation under both prefix rules, start times that follow the arrival order when
nothing is elastic, and an uncontended cluster on which the rule cannot bind."""
import numpy as np
import pytest

import gen


def _unit_trace(S, A, seed, cores, rate_per_s):
    """One CPU node and one quota; every action takes one unit and is not elastic."""
    t = gen.make_trace(S=S, A=A, seed=seed, cluster=(1, cores, 0, 1), type_probs=(0.6, 0, 0.4), rate_per_s=rate_per_s,
                       horizon_s=A / rate_per_s, max_ticks=100_000, cpu_median=400_000)
    t["act_model"][:] = 0
    t["act_kmask"][:] = 1
    return t


def _simulate(t, s, whole_queue):
    A, M, tick = t["A"], t["M"], int(t["tick_us"])
    nt = t["node_type"][s * M:(s + 1) * M]
    cpu, api = int(np.flatnonzero(nt == gen.TYPE_CPU)[0]), int(np.flatnonzero(nt == gen.TYPE_API)[0])
    free = int(t["node_cap"][s * M + cpu])
    cap_u, rate = int(t["node_cap"][s * M + api]) * 10**6, int(t["quota_rate"][s * M + api])
    tok = int(t["quota_tok0_micro"][s * M + api])
    arr = t["arrival_us"][s * A:(s + 1) * A]
    kind = t["act_type"][s * A:(s + 1) * A]
    T = t["act_t_ori_us"][s * A:(s + 1) * A]
    start = np.full(A, -1, np.int64)
    running = []                                                # finish times of the cores in use
    waiting, nxt, n = [], 0, 0
    while (start < 0).any() and n < t["max_ticks"]:
        now = n * tick
        free += sum(1 for f in running if f <= now)
        running = [f for f in running if f > now]
        if n > 0:
            tok = min(cap_u, tok + rate * tick)
        while nxt < A and arr[nxt] <= now:
            waiting.append(nxt)
            nxt += 1
        closed, still = set(), []
        for w, i in enumerate(waiting):
            k = int(kind[i])
            fits = free >= 1 if k == gen.TYPE_CPU else tok >= 10**6
            if k in closed or (whole_queue and closed) or not fits:
                closed.add(k)
                still.append(i)
                continue
            start[i] = now
            if k == gen.TYPE_CPU:
                free -= 1
                running.append(now + int(T[i]))
            else:
                tok -= 10**6
        waiting = still
        n += 1
    return start


@pytest.mark.parametrize("seed", range(6))
def test_cores_and_tokens_against_an_integer_simulation(orc, seed):
    t = _unit_trace(2, 250, 60 + seed, cores=2 + seed % 3, rate_per_s=12.0 + 4 * seed)
    M = t["M"]
    api = t["node_type"] == gen.TYPE_API
    t["quota_rate"][api] = 2 + seed                            # tokens per second: scarce
    t["node_cap"][api] = 3
    t["quota_tok0_micro"][api] = 2_000_000
    differ = False
    for whole_queue in (0, 1):
        o = orc.replay(dict(t, queue_prefix=whole_queue))
        for s in range(2):
            want = _simulate(t, s, bool(whole_queue))
            np.testing.assert_array_equal(o["start_us"][s * 250:(s + 1) * 250], want, err_msg=f"scenario {s} rule {whole_queue}")
        if whole_queue == 0:
            per_pool = o["start_us"].copy()
        else:
            differ = (per_pool != o["start_us"]).any()
    assert differ, "cores and tokens should block each other under the whole-queue rule"


@pytest.mark.parametrize("seed", range(6))
def test_starts_follow_the_arrival_order_when_nothing_is_elastic(orc, seed):
    """Without elastic actions nobody is evicted, so every admitted action starts: an action that starts at a tick
    has nobody before it in the queue still waiting, i.e. start times do not decrease with the arrival rank."""
    t = gen.make_trace(S=3, A=500, seed=80 + seed, cluster=(2, 8, 1, 2), rate_per_s=60.0, horizon_s=500 / 60.0,
                       max_ticks=100_000, cpu_median=500_000)
    t["act_model"][:] = 0
    o = orc.replay(dict(t, queue_prefix=1))
    p = orc.replay(t)
    violated = False
    for s in range(3):
        st = o["start_us"][s * 500:(s + 1) * 500]
        st = st[st >= 0]
        assert len(st) > 400
        assert (np.diff(st) >= 0).all()
        pst = p["start_us"][s * 500:(s + 1) * 500]
        pst = pst[pst >= 0]
        violated |= bool((np.diff(pst) < 0).any())
    assert violated, "with one prefix per pool some action should overtake a waiting one of another kind"


def test_uncontended_cluster_changes_nothing(orc):
    t = gen.make_trace(S=2, A=300, seed=90, cluster=(8, 128, 8, 2), rate_per_s=20.0, horizon_s=15.0, max_ticks=4000)
    api = t["node_type"] == gen.TYPE_API
    t["quota_rate"][api] = 1000
    t["node_cap"][api] = 1000
    t["quota_tok0_micro"][api] = 10**9
    t["act_pin_node"][t["act_type"] != gen.TYPE_API] = -1
    a, b = orc.replay(t), orc.replay(dict(t, queue_prefix=1))
    for k in a:
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)
    assert (a["start_us"] >= 0).all()
