"""Pins for the service cache of the oracle's replay (Sec. 5.3): every node keeps up to
`cache_slots` services resident, least recently used out first; an action whose service was not
resident when its tick began is delayed by the restore time.  Closed forms for hit / miss
patterns, and the cache re-run in Python from the oracle's own start times and nodes."""
import numpy as np
import pytest

import gen
import pyref


def _gpu_trace(n, services, restore, slots, gap_s=10, T=1_000_000):
    """One 8-GPU node; action i arrives at i*gap_s (nothing overlaps), runs non-elastically on one GPU."""
    t = gen.make_trace(S=1, A=n, seed=1, cluster=(0, 0, 1, 0), type_probs=(0, 1, 0), rate_per_s=1.0, horizon_s=1.0,
                       max_ticks=n * gap_s * 10 + 1000, pin_frac=0.0)
    t["arrival_us"] = (np.arange(n, dtype=np.int64) * gap_s * 1_000_000)
    t["act_model"][:] = 0
    t["act_kmask"][:] = 1
    t["act_t_ori_us"][:] = T
    t["act_pin_node"][:] = -1
    t["act_service"] = np.asarray(services, np.int32)
    t["restore_us"] = np.asarray(restore, np.int64)
    t["cache_slots"] = slots
    return t


@pytest.mark.parametrize("slots,pattern,misses", [
    (1, [0, 1, 0, 1, 0, 1], [1, 1, 1, 1, 1, 1]),               # one slot, two services: every call restores
    (2, [0, 1, 0, 1, 0, 1], [1, 1, 0, 0, 0, 0]),               # both fit: only the first calls restore
    (2, [0, 1, 2, 0, 1, 2], [1, 1, 1, 1, 1, 1]),               # three services cycling through two slots: LRU always misses
    (2, [0, 1, 0, 2, 0, 1], [1, 1, 0, 1, 0, 1]),               # 1 is the least recently used when 2 comes, then 1 misses again
    (3, [0, 1, 2, 0, 1, 2], [1, 1, 1, 0, 0, 0]),
    (1, [0, 0, -1, 0, 1, 1], [1, 0, 0, 0, 1, 0]),              # an action without a service touches nothing
])
def test_hit_and_miss_patterns(orc, slots, pattern, misses):
    restore = [300_000, 700_000, 1_100_000]
    t = _gpu_trace(len(pattern), pattern, restore, slots)
    o = orc.replay(t)
    np.testing.assert_array_equal(o["start_us"], t["arrival_us"])
    want = [1_000_000 + (restore[s] if m else 0) for s, m in zip(pattern, misses)]
    np.testing.assert_array_equal(o["finish_us"] - o["start_us"], want)


def _dur(t, g, k):
    q = list(t["k_list"]).index(k)
    K = t["K"]
    sp = int(t["speedup_q16"][int(t["act_param"][g]) * K + q]) if t["act_model"][g] == 2 else 0
    return pyref.duration(int(t["act_model"][g]), int(t["act_t_ori_us"][g]), int(t["act_param"][g]), int(k), sp)


def _with_services(t, seed, n_services, slots):
    rng = np.random.default_rng(seed)
    sv = rng.integers(-1, n_services, t["S"] * t["A"]).astype(np.int32)
    sv[t["act_type"] != gen.TYPE_GPU] = -1                     # services live on GPU nodes
    t["act_service"] = sv
    t["restore_us"] = (rng.integers(1, 9, n_services) * 150_000).astype(np.int64)
    t["cache_slots"] = slots
    return t


@pytest.mark.parametrize("seed", range(8))
def test_cache_rerun_from_the_oracles_starts(orc, seed):
    t = gen.make_trace(S=3, A=500, seed=70 + seed, cluster=(1, 16, 2 + seed % 2, 1), type_probs=(0.2, 0.7, 0.1),
                       rate_per_s=40.0, horizon_s=12.0, max_ticks=60000, pin_frac=0.3)
    _with_services(t, seed, n_services=(2, 5, 9)[seed % 3], slots=1 + seed % 3)
    o = orc.replay(t)
    S, A, M = t["S"], t["A"], t["M"]
    for s in range(S):
        resident = [0] * M
        used = {}
        seq = [0] * M
        started = [i for i in range(A) if o["start_us"][s * A + i] >= 0]
        misses = 0
        for start in sorted(set(int(o["start_us"][s * A + i]) for i in started)):
            snap = list(resident)                              # what the step of this tick saw
            for i in (i for i in started if o["start_us"][s * A + i] == start):   # index order = first come first served
                g = s * A + i
                j, sv = int(o["node"][g]), int(t["act_service"][g])
                delay = 0
                if sv >= 0:
                    if not snap[j] >> sv & 1:
                        delay = int(t["restore_us"][sv])
                        misses += 1
                    if not resident[j] >> sv & 1 and bin(resident[j]).count("1") >= t["cache_slots"]:
                        victim = min((x for x in range(64) if resident[j] >> x & 1), key=lambda x: (used[(j, x)], x))
                        resident[j] &= ~(1 << victim)
                    resident[j] |= 1 << sv
                    seq[j] += 1
                    used[(j, sv)] = seq[j]
                assert o["finish_us"][g] == start + delay + _dur(t, g, int(o["units"][g])), (s, i)
        assert misses > 0


def test_no_service_calls_is_the_plain_replay(orc):
    t = gen.make_trace(S=2, A=400, seed=90, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000)
    base = orc.replay(t)
    t["act_service"] = np.full(t["S"] * t["A"], -1, np.int32)
    t["restore_us"] = np.array([123456], np.int64)
    t["cache_slots"] = 1
    o = orc.replay(t)
    for k in ("start_us", "finish_us", "units", "node"):
        np.testing.assert_array_equal(o[k], base[k])


def test_with_room_for_everything_a_service_is_restored_once_per_node(orc):
    t = gen.make_trace(S=2, A=600, seed=91, cluster=(0, 0, 2, 0), type_probs=(0, 1, 0), rate_per_s=30.0, horizon_s=20.0,
                       max_ticks=60000, pin_frac=0.0)
    _with_services(t, 3, n_services=4, slots=64)
    o = orc.replay(t)
    A = t["A"]
    for s in range(t["S"]):
        late = {}
        for i in sorted(range(A), key=lambda i: (int(o["start_us"][s * A + i]), i)):
            g = s * A + i
            sv = int(t["act_service"][g])
            if sv < 0 or o["start_us"][g] < 0:
                continue
            delayed = o["finish_us"][g] - o["start_us"][g] > _dur(t, g, int(o["units"][g]))
            key = (int(o["node"][g]), sv)
            if delayed:                                        # only in the tick of the first use on that node
                late.setdefault(key, int(o["start_us"][g]))
                assert late[key] == int(o["start_us"][g])
            else:
                assert key in late and late[key] < int(o["start_us"][g])
