"""CPU pins of the trace replay with the GPU nodes of a scenario scheduled as one pool of chunks (Sec. 5.3, Alg. 4):
the tick loop around the pooled step, with the chunks of every node re-run on addresses by an independent allocator."""
import numpy as np
import pytest

import gen
from pyref import Buddy


def _gpu_trace(S, A, seed, n_gpu, rate, horizon_s, n_cpu=0):
    probs = (0.4, 0.6, 0) if n_cpu else (0, 1, 0)
    t = gen.make_trace(S=S, A=A, seed=seed, cluster=(n_cpu, 16, n_gpu, 0), type_probs=probs, rate_per_s=rate, horizon_s=horizon_s,
                       max_ticks=200_000, pin_frac=0.3)
    t["act_pin_node"] = np.where(t["act_type"] == gen.TYPE_GPU, -1, t["act_pin_node"]).astype(np.int32)   # a pool has no pins
    return t


def test_one_gpu_node_is_its_own_pool(orc):
    t = _gpu_trace(3, 300, 5, 1, 40.0, 6.0, n_cpu=2)
    a, b = orc.replay(t), orc.replay(dict(t, gpu_pooled=1))
    for k in a:
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)


@pytest.mark.parametrize("seed", range(5))
def test_every_tick_is_one_pooled_step_on_addresses_rebuilt_from_the_replays_own_times(orc, seed):
    """At every tick the free GPUs of every node are rebuilt here on addresses - an independent buddy allocator per node,
    fed with the starts (in arrival order, on the node the replay reported) and the finishes the replay reported - and one
    pooled step (pinned on its own in test_oracle_pooled.py) on that snapshot must select exactly the actions the replay
    started at that tick, on the same nodes with the same GPUs.  Every reported start must also find its chunk."""
    n_gpu, A = 2 + seed % 3, 220
    t = _gpu_trace(1, A, 500 + seed, n_gpu, 60.0 + 30 * seed, A / 80.0)
    t["depth"] = 1 + seed % 3
    t["gpu_pooled"] = 1
    o = orc.replay(t)
    M, tick = t["M"], int(t["tick_us"])
    start, fin, units, node, arr = o["start_us"], o["finish_us"], o["units"], o["node"], t["arrival_us"]
    assert (start >= 0).all()
    alloc = [Buddy() for _ in range(M)]
    held = {}                                                       # action -> (node, first GPU)
    waited = spread = False
    for n in range(int(o["n_ticks"][0])):
        now = n * tick
        for i in [i for i in held if fin[i] <= now]:
            j, s0 = held.pop(i)
            alloc[j].free(s0, int(units[i]))
        waiting = np.flatnonzero((arr <= now) & (start >= now))
        if len(waiting) == 0:
            continue
        running = sorted(held)
        free = np.array([bin(b.mask).count("1") for b in alloc], np.int32)
        chunks = np.array([c for b in alloc for c in b.counts()], np.uint8)
        busy = [[] for _ in range(M)]
        for i in running:
            busy[node[i]] += [int(fin[i]) - now] * int(units[i])
        p = dict(B=1, N=len(waiting), M=M, K=t["K"], n_classes=t["n_classes"], n_tasks=1, depth=t["depth"], gpu_pooled=1,
                 k_list=t["k_list"], type_k=t["type_k"], speedup_q16=t["speedup_q16"],
                 node_type=t["node_type"], node_cap=t["node_cap"], node_free=free, node_backlog_us=np.zeros(M, np.int64),
                 node_chunks=chunks, node_busy_off=np.concatenate([[0], np.cumsum([len(b) for b in busy])]).astype(np.int32),
                 node_busy_rel_us=np.array([x for b in busy for x in b] or [0], np.int64),
                 act_age_us=(now - arr[waiting]).astype(np.int64), act_task=None,
                 **{k: t[k][waiting] for k in ("act_type", "act_model", "act_t_ori_us", "act_kmask", "act_param", "act_pin_node")})
        s = orc.assign(p)
        go = start[waiting] == now
        np.testing.assert_array_equal(s["reason"] == 0, go, err_msg=f"tick {n}")
        np.testing.assert_array_equal(s["node"][go], node[waiting][go], err_msg=f"tick {n}")
        np.testing.assert_array_equal(s["units"][go], units[waiting][go], err_msg=f"tick {n}")
        np.testing.assert_array_equal(s["act_us"][go], (fin - arr)[waiting][go], err_msg=f"tick {n}")
        waited |= bool((~go).any())
        for i in waiting[go]:                                       # arrival order = visiting order
            s0 = alloc[node[i]].alloc(int(units[i]))
            assert s0 is not None, f"action {i} found no chunk of {units[i]} GPUs on node {node[i]} at tick {n}"
            held[int(i)] = (int(node[i]), s0)
        spread |= len(set(node[waiting][go])) > 1
    assert waited and spread


def test_pooling_changes_the_schedule_of_a_contended_cluster(orc):
    t = _gpu_trace(2, 400, 9, 3, 150.0, 3.0)
    a, b = orc.replay(t), orc.replay(dict(t, gpu_pooled=1))
    assert (a["start_us"] != b["start_us"]).any() or (a["units"] != b["units"]).any()
    for o in (a, b):                                                # GPUs in use never exceed a node's eight
        for s in range(2):
            sl = slice(s * 400, (s + 1) * 400)
            for j in range(t["M"]):
                m = o["node"][sl] == j
                rel = -(-o["finish_us"][sl][m] // t["tick_us"]) * t["tick_us"]
                ev = np.concatenate([o["start_us"][sl][m], rel])
                dl = np.concatenate([o["units"][sl][m], -o["units"][sl][m]]).astype(np.int64)
                order = np.lexsort((dl, ev))
                assert np.cumsum(dl[order]).max(initial=0) <= 8
