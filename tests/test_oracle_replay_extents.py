"""CPU pins of the observer of the oracle's replay (orc_replay_extents: the largest sizes the steps of a scenario worked
on).  Everything that can be re-derived from the replay's own outputs - who waited when, who ran where - is re-derived
here; the rest is bounded from both sides."""
import numpy as np
import pytest

import gen


def _per_tick(t, o, s):
    """For scenario s, per tick with somebody waiting: (waiting ids, running ids, ids started now)."""
    A, tick = t["A"], int(t["tick_us"])
    sl = slice(s * A, (s + 1) * A)
    arr, start, fin = t["arrival_us"][sl], o["start_us"][sl], o["finish_us"][sl]
    never = start < 0
    for n in range(int(o["n_ticks"][s])):
        now = n * tick
        waiting = np.flatnonzero((arr <= now) & (never | (start >= now)))
        if len(waiting) == 0:
            continue
        running = np.flatnonzero(~never & (start < now) & (fin > now))
        yield now, waiting, running, waiting[start[waiting] == now]


@pytest.mark.parametrize("case", ["contended", "default", "pooled", "tick_limit"])
def test_extents_against_the_replays_own_outputs(orc, case):
    if case == "contended":
        t = gen.make_trace(S=3, A=500, seed=61, contended=True, rate_per_s=150.0, horizon_s=3.0, max_ticks=40000)
    elif case == "default":
        t = gen.make_trace(S=2, A=800, seed=62, rate_per_s=200.0, horizon_s=4.0)
    elif case == "pooled":
        t = gen.trace_with_pooled_gpus(gen.make_trace(S=2, A=400, seed=63, cluster=(2, 16, 3, 1), rate_per_s=150.0, horizon_s=3.0,
                                                       max_ticks=40000))
    else:
        t = gen.make_trace(S=2, A=500, seed=64, contended=True, rate_per_s=500.0, horizon_s=1.0, max_ticks=40)
    o, e = orc.replay(t), orc.replay_extents(t)
    S, A, M = t["S"], t["A"], t["M"]
    for s in range(S):
        nt = t["node_type"][s * M:(s + 1) * M]
        cap = t["node_cap"][s * M:(s + 1) * M]
        ty = t["act_type"][s * A:(s + 1) * A]
        units, node = o["units"][s * A:(s + 1) * A], o["node"][s * A:(s + 1) * A]
        assert [e["nodes_cpu"][s], e["nodes_gpu"][s], e["nodes_api"][s]] == [(nt == k).sum() for k in range(3)]
        wait = np.zeros(3, np.int64)
        run = started_step = started_node = heap = busy = 0
        for now, waiting, running, go in _per_tick(t, o, s):
            wait = np.maximum(wait, np.bincount(ty[waiting], minlength=3))
            run = max(run, int((ty[running] != gen.TYPE_API).sum()))      # quotas hold nothing while an action runs
            started_step = max(started_step, len(go))
            if len(go):
                started_node = max(started_node, int(np.bincount(node[go]).max()))
                for j in np.unique(node[go]):                              # nodes that certainly had candidates
                    if nt[j] == gen.TYPE_API:
                        continue
                    pool = t.get("gpu_pooled") and nt[j] == gen.TYPE_GPU
                    on = running[(nt[node[running]] == gen.TYPE_GPU) if pool else (node[running] == j)]
                    b = int(units[on].sum())
                    busy = max(busy, b)
                    heap = max(heap, int(cap[nt == gen.TYPE_GPU].sum()) if pool else int(cap[j]))   # free + busy = everything the resource has
        assert [e["wait_cpu"][s], e["wait_gpu"][s], e["wait_api"][s]] == list(wait)
        assert e["running"][s] == run
        # candidates: at least the actions a step started (the evicted ones are candidates too), never more than waited
        assert started_step <= e["cand_step"][s] <= wait.sum()
        assert started_node <= e["cand_node"][s] <= e["cand_step"][s]
        assert e["cand_cpu_elastic"][s] <= e["cand_node"][s] and e["cand_gpu_elastic"][s] <= e["cand_node"][s]
        assert e["pinned_wait_step"][s] <= wait.sum()
        # heaps: the nodes seen above are among those the observer saw; a resource's heap is as large as the resource
        assert busy <= e["busy_units"][s] <= e["heap_entries"][s]
        biggest = max([int(c) for c, k in zip(cap, nt) if k != gen.TYPE_API] + ([int(cap[nt == gen.TYPE_GPU].sum())] if t.get("gpu_pooled") else []))
        assert heap <= e["heap_entries"][s] <= biggest
        assert e["dp_cells"][s] <= max([int(c) for c, k in zip(cap, nt) if k == gen.TYPE_CPU] + [0]) + 1
        n_gpu = int((nt == gen.TYPE_GPU).sum())
        most = {0: 1, 1: 40, 2: 100, 3: 196}[n_gpu if t.get("gpu_pooled") else min(n_gpu, 1)]
        assert e["chunk_states"][s] <= most
        if e["cand_gpu_elastic"][s]:
            assert e["chunk_states"][s] >= 2 * 2 * 2 * 2                   # at least the four radices of an almost empty state
    if case == "contended":
        assert e["cand_step"].max() > 1 and e["pinned_wait_step"].max() > 0 and e["busy_units"].max() >= 24
        assert (e["heap_entries"] == 32).all() and (e["dp_cells"] > 1).all()
    if case == "pooled":
        assert (e["heap_entries"] == 24).all()                              # three nodes of 8 GPUs: one heap
        assert (e["chunk_states"] >= 2 * 2 * 2 * 4).all()                   # the first GPU step sees three free 8-chunks in one state


def test_a_full_node_with_a_queue_in_closed_form(orc):
    """One 4-core node, ten one-core non-elastic jobs of 3 ticks at time 0: four start, six wait; every later step sees
    at most the cores that fell free as candidates, a heap of 4 entries and up to 4 busy units."""
    A = 10
    t = gen.make_trace(S=1, A=A, seed=1, cluster=(1, 4, 0, 0), type_probs=(1, 0, 0), pin_frac=0.0, max_ticks=1000)
    t["arrival_us"] = np.zeros(A, np.int64)
    t["act_model"] = np.zeros(A, np.uint8); t["act_kmask"] = np.ones(A, np.uint32)
    t["act_t_ori_us"] = np.full(A, 3 * t["tick_us"], np.int64)
    t["act_pin_node"] = np.full(A, -1, np.int32)
    e = orc.replay_extents(t)
    want = dict(wait_cpu=10, wait_gpu=0, wait_api=0, running=4, cand_cpu_elastic=0, cand_gpu_elastic=0, cand_node=4, cand_step=4,
                pinned_wait_step=0, busy_units=0, heap_entries=4, chunk_states=0, dp_cells=0, nodes_cpu=1, nodes_gpu=0, nodes_api=0)
    assert {k: int(v[0]) for k, v in e.items()} == want
    # pinned to the node, the six that wait are its waiting list; elastic, the tables are in use
    t["act_pin_node"] = np.zeros(A, np.int32)
    t["act_model"] = np.ones(A, np.uint8); t["act_param"] = np.full(A, 500_000, np.uint32); t["act_kmask"] = np.full(A, 3, np.uint32)
    e = {k: int(v[0]) for k, v in orc.replay_extents(t).items()}
    assert e["pinned_wait_step"] == 6 and e["cand_cpu_elastic"] == 4 and e["dp_cells"] == 5 and e["heap_entries"] == 4
