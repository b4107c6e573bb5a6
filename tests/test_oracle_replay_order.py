"""CPU pins of the trace replay under the second visiting order (least estimated ACT first, Sec. 4.2's remark that the
step also runs on top of other orderings): closed forms from single-machine scheduling, the tick loop around the step,
and the cases in which the order cannot matter."""
import numpy as np
import pytest

import gen
from test_oracle_replay import check_every_tick_is_one_step


def _one_core_trace(durations_ticks, tick=100_000, arrivals=None):
    """One CPU node with one core, non-elastic one-core actions of the given lengths (in ticks)."""
    A = len(durations_ticks)
    t = gen.make_trace(S=1, A=A, seed=1, cluster=(1, 1, 0, 0), type_probs=(1, 0, 0), pin_frac=0.0, max_ticks=10**6, tick_us=tick)
    t["arrival_us"] = np.zeros(A, np.int64) if arrivals is None else np.asarray(arrivals, np.int64)
    t["act_model"] = np.zeros(A, np.uint8)                          # no elasticity: one option, the smallest allowed
    t["act_kmask"] = np.ones(A, np.uint32)
    t["act_t_ori_us"] = (np.asarray(durations_ticks, np.int64) * tick)
    t["act_pin_node"] = np.full(A, -1, np.int32)
    return t


def test_one_core_everything_queued_at_once_is_shortest_processing_time_first(orc):
    """All jobs present at time 0 on one machine: the cost order runs them by ascending length (equal lengths in arrival
    order), each starting when the one before it ends - the textbook SPT schedule; FCFS runs them as they came."""
    d = np.array([5, 3, 9, 1, 3, 7, 2, 9, 4, 1])
    t = _one_core_trace(d)
    o = orc.replay(dict(t, order_policy=1))
    spt = np.lexsort((np.arange(len(d)), d))                        # by length, then arrival
    want = np.zeros(len(d), np.int64)
    want[spt] = np.concatenate([[0], np.cumsum(d[spt])[:-1]]) * t["tick_us"]
    np.testing.assert_array_equal(o["start_us"], want)
    f = orc.replay(t)
    np.testing.assert_array_equal(f["start_us"], np.concatenate([[0], np.cumsum(d)[:-1]]) * t["tick_us"])
    # SPT minimises the mean completion time on one machine
    assert o["mean_act"][0] < f["mean_act"][0]
    assert o["mean_act"][0] == (want + d * t["tick_us"]).mean()


def test_one_core_with_arrivals_over_time_picks_the_shortest_waiting_job_at_every_completion(orc):
    """Non-preemptive SPT with release times, simulated independently: whenever the core falls free (on the tick grid) the
    shortest job that has arrived starts; ties by arrival."""
    rng = np.random.default_rng(3)
    A, tick = 60, 100_000
    d = rng.integers(1, 8, A)
    arr = np.sort(rng.integers(0, 150, A)) * tick + rng.integers(0, tick, A)
    arr.sort()
    t = _one_core_trace(d, tick, arr)
    o = orc.replay(dict(t, order_policy=1))
    start = np.full(A, -1, np.int64)
    free_at, now = 0, 0
    while (start < 0).any():
        here = [i for i in range(A) if start[i] < 0 and arr[i] <= now]
        if here and free_at <= now:
            i = min(here, key=lambda x: (d[x], x))
            start[i] = now
            free_at = now + d[i] * tick
        now += tick
    np.testing.assert_array_equal(o["start_us"], start)
    assert (orc.replay(t)["start_us"] != start).any()               # FCFS differs on this trace


@pytest.mark.parametrize("seed", range(4))
def test_every_tick_is_one_step_in_cost_order(orc, seed):
    """The tick loop around the step under the cost order: every tick re-run as one step (whose own cost order is pinned in
    test_oracle_order.py) on the snapshot rebuilt from the replay's reported times."""
    A = 240
    t = gen.make_trace(S=1, A=A, seed=320 + seed, cluster=(2 + seed % 2, 8 + 4 * (seed % 3), 0, 2), type_probs=(0.8, 0, 0.2),
                       rate_per_s=70.0, horizon_s=A / 70.0, max_ticks=50_000, pin_frac=(0.0, 0.3)[seed % 2], cpu_median=700_000)
    t["depth"] = 1 + seed % 3
    t["quota_rate"][t["node_type"] == gen.TYPE_API] = 3 + seed
    t["order_policy"] = 1
    o, _ = check_every_tick_is_one_step(orc, t)
    assert (o["start_us"] != orc.replay(dict(t, order_policy=0))["start_us"]).any(), "the order should matter on this trace"


def test_order_cannot_matter_when_a_step_never_sees_two_actions(orc):
    t = gen.make_trace(S=3, A=300, seed=8, rate_per_s=20.0, horizon_s=15.0, max_ticks=2000, type_probs=(0.7, 0.3, 0))   # the large default cluster
    t["arrival_us"] = np.tile(np.arange(300, dtype=np.int64) * 3 * t["tick_us"] + 17, 3)   # one arrival every third tick
    a, b = orc.replay(t), orc.replay(dict(t, order_policy=1))
    assert (a["start_us"] == -(-t["arrival_us"] // t["tick_us"]) * t["tick_us"]).all()      # everybody starts at once
    for k in a:
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)


def test_gpu_chunks_are_handed_out_in_visiting_order(orc):
    """Two GPU actions start in the same tick on one node: the shorter one is visited first under the cost order and so takes
    the lower chunk address.  Seen through what fits next: after a 4-GPU action and a 2-GPU action start together on a free
    8-GPU node, whichever came second sits at GPUs 4-5 (or 4-7) - and conservation holds either way."""
    t = gen.make_trace(S=1, A=40, seed=11, cluster=(0, 0, 1, 0), type_probs=(0, 1, 0), rate_per_s=40.0, horizon_s=1.0, max_ticks=10**5,
                       pin_frac=0.0)
    for order in (0, 1):
        o = orc.replay(dict(t, order_policy=order))
        assert (o["start_us"] >= 0).all()
        ev = sorted([(int(s), +int(u)) for s, u in zip(o["start_us"], o["units"])] +
                    [(-(-int(f) // t["tick_us"]) * t["tick_us"], -int(u)) for f, u in zip(o["finish_us"], o["units"])],
                    key=lambda e: (e[0], e[1]))
        used = 0
        for _, d in ev:
            used += d
            assert 0 <= used <= 8


# --- the second visiting order next to the service cache: the keys move with what is resident (Sec. 4.2, 5.3) ----------

def _whole_node_trace(T_ticks, services, restore_ticks, slots, arrivals_ticks, tick=100_000, per_gpu=0):
    """One 8-GPU node; every action takes all 8 GPUs without elasticity: one machine whose set-up time for a job
    depends on what its cache holds."""
    A = len(T_ticks)
    t = gen.make_trace(S=1, A=A, seed=1, cluster=(0, 0, 1, 0), type_probs=(0, 1, 0), pin_frac=0.0, max_ticks=10**6, tick_us=tick)
    k8 = [int(k) for k in t["k_list"]].index(8)
    t["arrival_us"] = np.asarray(arrivals_ticks, np.int64) * tick
    t["act_model"] = np.zeros(A, np.uint8)
    t["act_kmask"] = np.full(A, 1 << k8, np.uint32)
    t["act_t_ori_us"] = np.asarray(T_ticks, np.int64) * tick
    t["act_pin_node"] = np.full(A, -1, np.int32)
    t["act_service"] = np.asarray(services, np.int32)
    t["restore_us"] = np.asarray(restore_ticks, np.int64) * tick
    t["cache_slots"] = slots
    t["cache_per_gpu"] = per_gpu
    t["order_policy"] = 1
    return t


def _one_machine_with_cache(T, sv, restore, slots, arr):
    """Independent simulation on the tick grid: whenever the machine is free, the arrived job with the least
    (run time + restore time unless its service is cached) starts, earlier arrival on ties; LRU cache."""
    A = len(T)
    start, fin = [-1] * A, [-1] * A
    cache, seq, free_at, now = {}, 0, 0, 0
    while min(start) < 0:
        here = [i for i in range(A) if start[i] < 0 and arr[i] <= now]
        if here and free_at <= now:
            cost = lambda i: T[i] + (restore[sv[i]] if sv[i] >= 0 and sv[i] not in cache else 0)
            i = min(here, key=lambda x: (cost(x), x))
            start[i], fin[i] = now, now + cost(i)
            free_at = fin[i]
            if sv[i] >= 0:
                if sv[i] not in cache and len(cache) >= slots:
                    del cache[min(cache, key=lambda y: (cache[y], y))]
                seq += 1
                cache[sv[i]] = seq
        now += 1
    return start, fin


@pytest.mark.parametrize("seed", range(12))
def test_cost_order_with_services_follows_the_cache(orc, seed):
    rng = np.random.default_rng(900 + seed)
    A = 40
    T = rng.integers(1, 6, A).tolist()
    n_sv = int(rng.integers(2, 5))
    sv = rng.integers(-1, n_sv, A).tolist()
    restore = rng.integers(1, 9, n_sv).tolist()
    slots = int(rng.integers(1, 3))
    arr = sorted(rng.integers(0, 60 if seed % 2 else 1, A).tolist())       # odd seeds: arrivals over time; even: all at once
    want_start, want_fin = _one_machine_with_cache(T, sv, restore, slots, arr)
    for per_gpu in (0, 1):                                                  # whole-node actions: both caches are the same
        t = _whole_node_trace(T, sv, restore, slots, arr, per_gpu=per_gpu)
        o = orc.replay(t)
        np.testing.assert_array_equal(o["start_us"], np.asarray(want_start, np.int64) * t["tick_us"])
        np.testing.assert_array_equal(o["finish_us"], np.asarray(want_fin, np.int64) * t["tick_us"])
    fcfs = orc.replay(dict(t, order_policy=0))
    assert (fcfs["start_us"] != o["start_us"]).any()
    # the cache changes the order, not only the durations: the static keys (run time alone) give another schedule
    static = np.lexsort((np.arange(A), np.asarray(T)))
    by_key = np.argsort(o["start_us"], kind="stable")
    if seed % 2 == 0:
        assert (by_key != static).any()


def test_cost_order_with_free_restores_is_the_plain_cost_order(orc):
    t = gen.make_trace(S=2, A=500, seed=98, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000)
    t["order_policy"] = 1
    base = orc.replay(t)
    gen.trace_with_services(t, 3, n_services=5, slots=1)
    t["restore_us"][:] = 0
    o = orc.replay(t)
    for k in ("start_us", "finish_us", "units", "node"):
        np.testing.assert_array_equal(o[k], base[k])
