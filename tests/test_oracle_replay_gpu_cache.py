"""Pins for the oracle's replay with a cache on every GPU (Sec. 5.3, `cache_per_gpu`): every GPU keeps up to
`cache_slots` services, least recently used out first; an action finds its service resident when every GPU of the
block it is given caches it; among the free chunks of the level the allocation takes from, one that caches the
service comes first.  Closed forms on one 8-GPU node, the whole run re-derived in Python (buddy allocation and
caches on sets of GPUs) from the oracle's own starts, and the cases in which the per-GPU cache is the per-node one."""
import numpy as np
import pytest

import gen
from test_oracle_replay_service import _dur, _with_services

SEC = 1_000_000


def _node_trace(rows, restore, slots, per_gpu=1):
    """One 8-GPU node.  rows: (arrival second, GPUs, run time in seconds, service or -1), non-elastic."""
    n = len(rows)
    t = gen.make_trace(S=1, A=n, seed=1, cluster=(0, 0, 1, 0), type_probs=(0, 1, 0), rate_per_s=1.0, horizon_s=1.0,
                       max_ticks=100000, pin_frac=0.0)
    k_list = [int(k) for k in t["k_list"]]
    t["arrival_us"] = np.asarray([r[0] * SEC for r in rows], np.int64)
    t["act_model"][:] = 0
    t["act_kmask"] = np.asarray([1 << k_list.index(r[1]) for r in rows], np.uint32)
    t["act_t_ori_us"] = np.asarray([r[2] * SEC for r in rows], np.int64)
    t["act_pin_node"][:] = -1
    t["act_service"] = np.asarray([r[3] for r in rows], np.int32)
    t["restore_us"] = np.asarray(restore, np.int64)
    t["cache_slots"] = slots
    t["cache_per_gpu"] = per_gpu
    return t


def _delays(orc, t):
    o = orc.replay(t)
    np.testing.assert_array_equal(o["start_us"], t["arrival_us"])          # nobody waits in these cases
    return [int(x) for x in o["finish_us"] - o["start_us"] - t["act_t_ori_us"]]


R = [300_000, 700_000]       # restore times of services 0 and 1


def test_one_after_the_other_lands_on_the_first_gpu(orc):
    """Nothing overlaps: every action takes GPU 0, so two services on one slot evict each other as on a node."""
    rows = [(10 * i, 1, 1, i % 2) for i in range(6)]
    assert _delays(orc, _node_trace(rows, R, 1)) == [R[0], R[1]] * 3
    rows = [(10 * i, 1, 1, 0) for i in range(4)]
    assert _delays(orc, _node_trace(rows, R, 1)) == [R[0], 0, 0, 0]


def test_side_by_side_both_stay_cached(orc):
    """0 on GPU 0 and 1 on GPU 1 at the same time: later each finds its own GPU again - on a node with one slot
    they would evict each other."""
    rows = [(0, 1, 100, 0), (10, 1, 100, 1), (200, 1, 100, 0), (210, 1, 100, 1)]
    assert _delays(orc, _node_trace(rows, R, 1)) == [R[0], R[1], 0, 0]
    assert _delays(orc, _node_trace(rows, R, 1, per_gpu=0)) == [R[0], R[1], R[0], R[1]]


def test_the_chunk_that_caches_the_service_comes_first(orc):
    """GPUs 0 and 2 busy, 1 and 3 free chunks of one GPU; 3 caches service 1: it is taken before GPU 1."""
    rows = [(0, 1, 1000, -1),      # GPU 0, stays
            (1, 1, 5, 0),          # GPU 1: service 0
            (2, 1, 1000, -1),      # GPU 2, stays
            (3, 1, 5, 1),          # GPU 3: service 1
            (100, 1, 50, 1),       # free chunks of one GPU: 1 and 3; 3 caches it
            (110, 1, 50, 0)]       # GPU 1 is the only free chunk of one GPU and caches it
    assert _delays(orc, _node_trace(rows, R, 1)) == [0, R[0], 0, R[1], 0, 0]
    # the other way round: service 0 asks first and finds GPU 1, the lowest one, anyway
    rows[4], rows[5] = (100, 1, 50, 0), (110, 1, 50, 1)
    assert _delays(orc, _node_trace(rows, R, 1)) == [0, R[0], 0, R[1], 0, 0]


def test_the_level_comes_before_the_cache(orc):
    """The service is cached on GPU 4, inside a free chunk of four; a free chunk of one GPU exists: that one is taken."""
    rows = [(0, 4, 20, -1),        # GPUs 0-3
            (1, 1, 5, 0),          # GPU 4 (split off the chunk 4-7): service 0
            (100, 1, 1000, -1),    # everything free again: GPU 0
            (101, 1, 5, 0)]        # free: 1 | 2-3 | 4-7 -> GPU 1, which does not cache it
    assert _delays(orc, _node_trace(rows, R, 1)) == [0, R[0], 0, R[0]]


def test_the_block_inside_a_larger_chunk(orc):
    """The whole node is one free chunk and GPU 4 caches the service: GPU 4 is the block taken."""
    rows = [(0, 4, 20, -1), (1, 1, 5, 0),
            (100, 1, 50, 0),       # all free: GPU 4 again
            (101, 1, 50, 0),       # GPU 4 busy: free 5 | 6-7 | 0-3 -> GPU 5, a miss
            (200, 1, 50, 0),       # all free: the first block that caches it is GPU 4
            (201, 1, 50, 0),       # GPU 5 caches it too and is the free chunk of one GPU
            (202, 1, 50, 0)]       # 6-7: GPU 6, a miss
    assert _delays(orc, _node_trace(rows, R, 1)) == [0, R[0], 0, R[0], 0, 0, R[0]]


def test_every_gpu_of_the_block_must_cache_it(orc):
    rows = [(0, 1, 5, 0),          # GPU 0
            (100, 2, 5, 0),        # GPUs 0-1: GPU 1 does not cache it
            (200, 2, 5, 0),        # now both do
            (300, 4, 5, 0),        # 0-3: 2 and 3 do not
            (400, 4, 5, 0), (500, 8, 5, 0), (600, 8, 5, 0), (700, 1, 5, 0)]
    assert _delays(orc, _node_trace(rows, R, 2)) == [R[0], R[0], 0, R[0], 0, R[0], 0, 0]


def test_least_recently_used_per_gpu(orc):
    """Two slots on GPU 0, three services in turn always miss; the order of use decides the victim."""
    rows = [(10 * i, 1, 1, sv) for i, sv in enumerate([0, 1, 2, 0, 1, 2])]
    assert _delays(orc, _node_trace(rows, [R[0], R[1], 900_000], 2)) == [R[0], R[1], 900_000, R[0], R[1], 900_000]
    rows = [(10 * i, 1, 1, sv) for i, sv in enumerate([0, 1, 0, 2, 0, 1])]
    assert _delays(orc, _node_trace(rows, [R[0], R[1], 900_000], 2)) == [R[0], R[1], 0, 900_000, 0, R[1]]


# --- the whole run again, in Python, from the oracle's own starts ------------------------------------------------

def _free_chunks(free, start=0, size=8):
    """Maximal aligned free blocks of a node whose free GPUs are the set ``free``, ascending."""
    if all(g in free for g in range(start, start + size)):
        return [(start, size)]
    if size == 1:
        return []
    return _free_chunks(free, start, size // 2) + _free_chunks(free, start + size // 2, size // 2)


def _take(free, need, sv, cache):
    chunks = _free_chunks(free)
    size = min(sz for _, sz in chunks if sz >= need)
    level = [st for st, sz in chunks if sz == size]
    blocks = [b for st in level for b in range(st, st + size, need)]
    cached = [b for b in blocks if sv >= 0 and all(sv in cache[g] for g in range(b, b + need))]
    first = cached[0] if cached else level[0]
    return first, bool(cached)


@pytest.mark.parametrize("seed", range(10))
def test_rerun_from_the_oracles_starts(orc, seed):
    t = gen.make_trace(S=2, A=500, seed=270 + seed, cluster=(1, 16, 1 + seed % 3, 1), type_probs=(0.2, 0.7, 0.1),
                       rate_per_s=(40.0, 80.0)[seed % 2], horizon_s=12.0, max_ticks=60000, pin_frac=0.3)
    _with_services(t, seed, n_services=(2, 5, 9)[seed % 3], slots=1 + seed % 3)
    t["cache_per_gpu"] = 1
    o = orc.replay(t)
    S, A, M = t["S"], t["A"], t["M"]
    hits = misses = preferred = 0
    for s in range(S):
        gpu_nodes = [j for j in range(M) if t["node_type"][s * M + j] == gen.TYPE_GPU]
        free = {j: set(range(int(t["node_cap"][s * M + j]))) for j in gpu_nodes}
        cache = {j: [dict() for _ in range(8)] for j in gpu_nodes}          # per GPU: service -> number of its last use
        seq = {j: 0 for j in gpu_nodes}
        running = []
        started = [i for i in range(A) if o["start_us"][s * A + i] >= 0 and t["act_type"][s * A + i] == gen.TYPE_GPU]
        for start in sorted(set(int(o["start_us"][s * A + i]) for i in started)):
            for fin, j, gpus in [r for r in running if r[0] <= start]:
                free[j] |= gpus
            running = [r for r in running if r[0] > start]
            for i in (i for i in started if o["start_us"][s * A + i] == start):      # index order = first come first served
                g = s * A + i
                j, k, sv = int(o["node"][g]), int(o["units"][g]), int(t["act_service"][g])
                first, hit = _take(free[j], k, sv, cache[j])
                if sv >= 0:
                    lowest, _ = _take(free[j], k, -1, cache[j])
                    preferred += hit and first != lowest
                    hits += hit
                    misses += not hit
                    seq[j] += 1
                    for x in range(first, first + k):
                        c = cache[j][x]
                        if sv not in c and len(c) >= t["cache_slots"]:
                            del c[min(c, key=lambda y: (c[y], y))]
                        c[sv] = seq[j]
                delay = int(t["restore_us"][sv]) if sv >= 0 and not hit else 0
                assert o["finish_us"][g] == start + delay + _dur(t, g, k), (s, i)
                gpus = set(range(first, first + k))
                assert gpus <= free[j]
                free[j] -= gpus
                running.append((int(o["finish_us"][g]), j, gpus))
    assert hits > 0 and misses > 0
    if seed in (0, 1, 4):
        assert preferred > 0                                   # the preference really changed a block


# --- where the cache per GPU is the cache per node --------------------------------------------------------------

def test_whole_node_actions_see_the_cache_of_the_node(orc):
    """Every GPU action takes all 8 GPUs: the 8 caches of a node are always equal, and equal to the node's."""
    t = gen.make_trace(S=3, A=400, seed=95, cluster=(1, 16, 3, 0), type_probs=(0.2, 0.8, 0), rate_per_s=20.0, horizon_s=20.0,
                       max_ticks=100000, pin_frac=0.3)
    k8 = [int(k) for k in t["k_list"]].index(8)
    gpu = t["act_type"] == gen.TYPE_GPU
    t["act_kmask"] = np.where(gpu, 1 << k8, t["act_kmask"]).astype(np.uint32)
    t["act_model"] = np.where(gpu, 0, t["act_model"]).astype(np.uint8)
    _with_services(t, 5, n_services=6, slots=2)
    per_node = orc.replay(t)
    assert (per_node["finish_us"][gpu] > 0).any()
    t["cache_per_gpu"] = 1
    per_gpu = orc.replay(t)
    for k in ("start_us", "finish_us", "units", "node"):
        np.testing.assert_array_equal(per_gpu[k], per_node[k])


def test_free_restores_change_nothing(orc):
    t = gen.make_trace(S=2, A=500, seed=96, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000)
    base = orc.replay(t)
    _with_services(t, 2, n_services=5, slots=1)
    t["restore_us"][:] = 0
    t["cache_per_gpu"] = 1
    o = orc.replay(t)
    for k in ("start_us", "finish_us", "units", "node"):
        np.testing.assert_array_equal(o[k], base[k])


def test_without_services_the_flag_changes_nothing(orc):
    t = gen.make_trace(S=2, A=400, seed=97, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000)
    base = orc.replay(t)
    t["cache_per_gpu"] = 1
    o = orc.replay(t)
    for k in ("start_us", "finish_us", "units", "node"):
        np.testing.assert_array_equal(o[k], base[k])
