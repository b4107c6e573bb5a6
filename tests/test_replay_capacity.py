"""Host-side bounds model of the replay kernel's buffers (no GPU).

tg_replay_capacity reports, from the same layout code the launcher uses, how large every list and
table of a step may grow before an index of the replay kernel would leave its block of local memory
or its slice of the workspace.  The oracle's replay observes, tick by tick, how large those same
quantities actually get on a trace (orc_replay_extents).  Every observed maximum must stay within
the capacity, on the random sweep of small traces, on the contended clusters under both admission
rules, and on the shapes that once overran a block (a quota with more candidates than any node has
units; pools wider than a wavefront).
"""
import numpy as np
import pytest

import gen
from paper_2603_13019_amd import tg


def _check(t, orc, what):
    cap = tg.replay_capacity(t)
    seen = orc.replay_extents(t)
    assert set(cap) == set(seen)
    for name, c in cap.items():
        worst = int(seen[name].max())
        assert worst <= c, f"{what}: {name} reaches {worst}, the kernel's buffers hold {c}"
    return cap, seen


def test_random_sweep_stays_inside_every_buffer(orc):
    """The 60 traces of the GPU sweep and 1940 more drawn the same way."""
    hit = {}
    for seed in range(500, 2500):
        t = gen.random_trace(seed)
        cap, seen = _check(t, orc, f"seed {seed}")
        for name in cap:
            hit[name] = max(hit.get(name, 0.0), int(seen[name].max()) / max(cap[name], 1))
    # the sweep is not vacuous: node tables are sized exactly, heaps and rows of the units table fill up
    for name in ("nodes_cpu", "nodes_gpu", "nodes_api"):
        assert hit[name] == 1.0
    assert hit["heap_entries"] > 0.9 and hit["dp_cells"] > 0.9 and hit["chunk_states"] > 0.5, hit


CONTENDED = {
    "contended_small": dict(S=6, A=400, seed=21, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000),
    "contended_burst": dict(S=4, A=700, seed=22, contended=True, rate_per_s=400.0, horizon_s=2.0, max_ticks=30000),
    "depth_and_ties": dict(S=4, A=500, seed=31, contended=True, rate_per_s=120.0, horizon_s=4.0, max_ticks=30000),
    "workload5_contended": dict(S=3, A=10_000, seed=5, contended=True, max_ticks=200_000),
    "workload5": dict(S=2, A=10_000, seed=4),
}


@pytest.mark.parametrize("queue_prefix", [1, 0])
@pytest.mark.parametrize("name", list(CONTENDED))
def test_contended_clusters_under_both_admission_rules(orc, name, queue_prefix):
    t = dict(gen.make_trace(**CONTENDED[name]), queue_prefix=queue_prefix)
    cap, seen = _check(t, orc, name)
    if "contended" in name:
        # a saturated 32-core node: its heap holds one entry per core while a queue waits
        assert int(seen["heap_entries"].max()) == 32 and int(seen["wait_cpu"].max()) > 16
        assert int(seen["busy_units"].max()) >= 24


def test_contended_whole_queue_prefix_with_quotas_services_aux_and_cores(orc):
    for seed in range(8):
        t = gen.make_trace(S=3, A=500, seed=700 + seed, cluster=(2, 16, 2, 3), rate_per_s=120.0, horizon_s=4.0, max_ticks=30000,
                           pin_frac=0.5)
        gen.with_extra_quotas(t, frac=0.5, seed=seed)
        gen.trace_with_services(t, seed, n_services=5, slots=2)
        gen.trace_with_aux(t, seed, scarce=bool(seed & 1))
        t["numa_cores"] = 8
        t["queue_prefix"] = 1
        t["depth"] = 1 + seed % 4
        _check(t, orc, f"seed {seed}")


def test_quota_with_more_candidates_than_any_node_has_units(orc):
    """A quota's candidates are bounded by its tokens, not by the units of the CPU and GPU nodes the per-node
    tables are sized for: they may pass the rows of those tables (the kernel then stages none of their rows),
    but never the list slice."""
    t = gen.make_trace(S=3, A=320, seed=71, cluster=(1, 4, 0, 1), type_probs=(0.06, 0, 0.94), rate_per_s=50.0, horizon_s=6.4,
                       max_ticks=4000)
    t["node_cap"] = np.where(t["node_type"] == gen.TYPE_API, 300, t["node_cap"]).astype(np.int32)
    t["quota_tok0_micro"] = np.where(t["node_type"] == gen.TYPE_API, 300_000_000, 0).astype(np.int64)
    cap, seen = _check(t, orc, "quota")
    assert int(seen["cand_node"].max()) > cap["cand_cpu_elastic"]
    assert int(seen["cand_cpu_elastic"].max()) <= 4


def test_wide_pools(orc):
    for cluster, probs in (((70, 4, 6, 0), (0.4, 0.6, 0)), ((90, 8, 3, 0), (0.8, 0.2, 0)), ((150, 16, 2, 0), (0.9, 0.1, 0)),
                           ((0, 0, 70, 0), (0, 1, 0))):
        t = gen.make_trace(S=2, A=900, seed=72, cluster=cluster, type_probs=probs, rate_per_s=300.0, horizon_s=3.0, max_ticks=30000)
        cap, seen = _check(t, orc, str(cluster))
        assert cap["nodes_cpu"] == max(cluster[0], 1) and cap["nodes_gpu"] == max(cluster[2], 1)


def test_largest_nodes(orc):
    """256-core nodes, the largest the builder takes: heap of 256 entries, 257 cells per row."""
    t = gen.make_trace(S=2, A=3000, seed=9, cluster=(2, 256, 1, 0), type_probs=(0.9, 0.1, 0), rate_per_s=600.0, horizon_s=4.0,
                       max_ticks=60000, cpu_median=4_000_000)
    cap, seen = _check(t, orc, "256 cores")
    assert cap["heap_entries"] == 256 and cap["dp_cells"] >= 257
    assert int(seen["heap_entries"].max()) == 256


def test_capacity_rejects_what_the_builder_rejects():
    t = gen.make_trace(S=1, A=10, seed=1, contended=True)
    bad = dict(t, node_cap=np.where(t["node_type"] == gen.TYPE_CPU, 257, t["node_cap"]).astype(np.int32))
    with pytest.raises(tg.TgError) as e:
        tg.replay_capacity(bad)
    assert e.value.code == tg.E_RANGE
    bad = dict(t, node_cap=np.where(t["node_type"] == gen.TYPE_GPU, 4, t["node_cap"]).astype(np.int32))
    with pytest.raises(tg.TgError) as e:
        tg.replay_capacity(bad)
    assert e.value.code == tg.E_INVALID_ARG


def _pooled_trace(S, A, seed, n_gpu, rate, horizon_s, n_cpu=2):
    t = gen.make_trace(S=S, A=A, seed=seed, cluster=(n_cpu, 16, n_gpu, 1), type_probs=(0.3, 0.6, 0.1), rate_per_s=rate,
                       horizon_s=horizon_s, max_ticks=200_000, pin_frac=0.3)
    t["act_pin_node"] = np.where(t["act_type"] == gen.TYPE_GPU, -1, t["act_pin_node"]).astype(np.int32)
    t["gpu_pooled"] = 1
    return t


@pytest.mark.parametrize("n_gpu", [1, 2, 3, 4, 5])
def test_pooled_gpu_clusters(orc, n_gpu):
    """The GPU nodes of a scenario as one pool: up to 40 candidates and heap entries on one resource, chunk states of the
    summed counts."""
    from pyref import Buddy
    vecs = {Buddy(m).counts() for m in range(256)}
    sums = {(0, 0, 0, 0)}
    for _ in range(n_gpu):
        sums = {tuple(a + b for a, b in zip(u, v)) for u in sums for v in vecs}
    most = max(int(np.prod([max(c, 1) + 1 for c in v])) for v in sums)   # over everything n nodes' masks can add up to
    for queue_prefix in (0, 1):
        t = dict(_pooled_trace(2, 600, 30 + n_gpu, n_gpu, 40.0 * n_gpu + 40, 4.0), queue_prefix=queue_prefix)
        cap, seen = _check(t, orc, f"{n_gpu} pooled nodes")
        assert cap["chunk_states"] >= most and cap["heap_entries"] >= 8 * n_gpu and cap["cand_gpu_elastic"] >= 8 * n_gpu
    assert int(seen["heap_entries"].max()) >= 8 * n_gpu and int(seen["chunk_states"].max()) > (40 if n_gpu > 1 else 8)


def test_pools_the_replay_refuses():
    t = _pooled_trace(1, 40, 3, 6, 50.0, 1.0)
    with pytest.raises(tg.TgError) as e:
        tg.replay_capacity(t)
    assert e.value.code == tg.E_RANGE                               # six nodes: their chunk counts can pass the table's 512 states
