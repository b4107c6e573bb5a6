"""Pins for the pooled GPU mode (Sec. 5.3, Alg. 4: the GPU manager runs the algorithm for the GPU cluster
as a whole; the state counts the free chunks of every size wherever they are): the counts of the pool
against an address-level allocator over several nodes, the pooled step against the plain step on a problem
folded independently in Python, the chunk every action gets, and the degenerate case of one node."""
import itertools

import numpy as np
import pytest

import gen
import pyref


def _pooled_problem(seed, n_gpu, N=80, **kw):
    p = gen.make_random_problem(seed, B=3, N=N, n_cpu=1, n_gpu=n_gpu, n_api=1, pin_frac=0.0,
                                type_probs=(0.2, 0.7, 0.1), **kw)
    M = p["M"]
    for b in range(p["B"]):                                   # a pool has one backlog
        g = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        p["node_backlog_us"][g] = p["node_backlog_us"][g[0]]
    p["act_pin_node"][p["act_type"] == gen.TYPE_GPU] = -1      # actions are not pinned to a node of a pool
    p["gpu_pooled"] = 1
    return p


@pytest.mark.parametrize("seed", range(30))
def test_pool_counts_follow_the_cluster_allocator(orc, seed):
    """Taking chunks from the summed counts == allocating on addresses over all nodes with the cluster-wide
    best fit: the same requests fit, and the counts agree after every request."""
    rng = np.random.default_rng(seed)
    masks = [int(rng.integers(0, 256)) for _ in range(int(rng.integers(1, 6)))]
    cl = pyref.BuddyCluster(masks)
    counts = cl.counts()
    for _ in range(20):
        k = int(rng.choice([1, 2, 4, 8]))
        ok, after = orc.chunk_take(counts, k)
        got = cl.alloc(k)
        assert ok == (got is not None)
        if ok:
            counts = after
        assert tuple(counts) == cl.counts()


@pytest.mark.parametrize("seed", range(12))
def test_pool_dp_against_exhaustive_search(orc, seed):
    """DPArrange on the pool's counts == the best unit vector the cluster allocator can serve in order."""
    rng = np.random.default_rng(100 + seed)
    masks = [int(rng.integers(0, 256)) for _ in range(int(rng.integers(2, 5)))]
    m = int(rng.integers(1, 6))
    klist = [1, 2, 4, 8]
    dur = np.full((m, 4), pyref.INF, np.int64)
    opts = []
    for i in range(m):
        T = int(rng.integers(1000, 9000))
        qs = sorted(rng.choice(4, int(rng.integers(1, 5)), replace=False))
        for q in qs:
            dur[i, q] = -(-T // klist[q]) + int(rng.integers(0, 50))
        opts.append([(klist[q], int(dur[i, q])) for q in qs])
    best = None
    for combo in itertools.product(*opts):
        cl = pyref.BuddyCluster(masks)
        if all(cl.alloc(k) is not None for k, _ in combo):
            v = sum(d for _, d in combo)
            best = v if best is None or v < best else best
    val, ks = orc.dp_chunks(dur, klist, pyref.BuddyCluster(masks).counts())
    if best is None:
        assert val == pyref.INF
    else:
        assert val == best
        cl = pyref.BuddyCluster(masks)
        assert all(cl.alloc(int(k)) is not None for k in ks)


def _fold(p):
    """The same problem with the GPU nodes of every snapshot merged into the first of them (built here,
    independently of the oracle): one node with all their units, chunks and running actions."""
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    q["gpu_pooled"] = 0
    M = p["M"]
    off, rel = p.get("node_busy_off"), p.get("node_busy_rel_us")
    busy = [[] for _ in range(p["B"] * M)]
    if off is not None:
        busy = [list(rel[off[n]:off[n + 1]]) for n in range(p["B"] * M)]
    ch = q["node_chunks"].reshape(-1, 4)
    for b in range(p["B"]):
        g = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        if len(g) == 0:
            continue
        r = g[0]
        for n in g[1:]:
            q["node_cap"][r] += q["node_cap"][n]
            q["node_free"][r] += q["node_free"][n]; q["node_free"][n] = 0
            ch[r] += ch[n]; ch[n] = 0
            busy[r] += busy[n]; busy[n] = []
    if off is not None:
        q["node_busy_off"] = np.concatenate([[0], np.cumsum([len(x) for x in busy])]).astype(np.int32)
        q["node_busy_rel_us"] = np.array([v for x in busy for v in x], np.int64)
    return q


@pytest.mark.parametrize("seed", range(12))
def test_pooled_step_equals_the_step_on_the_folded_problem(orc, seed):
    p = _pooled_problem(700 + seed, n_gpu=2 + seed % 4, N=60 + 10 * seed, busy=seed % 2 == 0, depth=1 + seed % 3)
    p["order_policy"] = seed % 2
    got, want = orc.assign(p), orc.assign(_fold(p))
    for k in ("units", "act_us", "reason", "task_sum"):
        np.testing.assert_array_equal(got[k], want[k], err_msg=k)
    for k in ("sum_act_us", "n_assigned", "n_prefix", "n_evicted", "n_infeasible", "units_used", "units_free"):
        np.testing.assert_array_equal(got["summary"][k], want["summary"][k], err_msg=k)
    assert (got["units"][p["act_type"] == gen.TYPE_GPU] > 0).any()


@pytest.mark.parametrize("seed", range(12))
def test_every_action_gets_the_chunk_the_cluster_allocator_gives(orc, seed):
    """Selected GPU actions in queue order, replayed on addresses: the oracle's node is the one the
    cluster-wide best fit picks; per node the units add up to node_used and never exceed what was free."""
    p = _pooled_problem(740 + seed, n_gpu=2 + seed % 5, N=90, busy=seed % 2 == 1)
    o = orc.assign(p)
    N, M = p["N"], p["M"]
    for b in range(p["B"]):
        g = [j for j in range(M) if p["node_type"][b * M + j] == gen.TYPE_GPU]
        cl = pyref.BuddyCluster([int(p["gpu_mask_"][b * M + j]) for j in g])
        used = np.zeros(M, np.int64)
        for i in range(N):
            a = b * N + i
            if p["act_type"][a] != gen.TYPE_GPU or o["units"][a] == 0:
                continue
            j, _ = cl.alloc(int(o["units"][a]))
            assert g[j] == o["node"][a], (b, i)
            used[g[j]] += o["units"][a]
        for j in g:
            assert used[j] == o["node_used"][b * M + j] <= p["node_free"][b * M + j]


def test_one_gpu_node_is_its_own_pool(orc):
    p = _pooled_problem(780, n_gpu=1, N=70)
    a = orc.assign(p)
    b = orc.assign(dict(p, gpu_pooled=0))
    for k in a:
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)


def test_pooling_sees_chunks_that_single_nodes_hide(orc):
    """Two nodes, each with one free 4-GPU chunk; two non-elastic actions that need 4 GPUs each and arrive
    when node 0 is the better choice for both.  Node by node, both go to node 0 and the second one has to
    wait; as one pool, both run."""
    p = gen.make_random_problem(5, B=1, N=2, n_cpu=0, n_gpu=2, n_api=0, shuffle_nodes=False, busy=False, bad_frac=0.0)
    p["node_free"][:] = 4
    p["node_chunks"] = np.array([0, 0, 1, 0, 0, 0, 1, 0], np.uint8)
    p["gpu_mask_"] = np.array([0x0F, 0x0F], np.int32)
    p["node_backlog_us"][:] = 0
    p["act_type"][:] = gen.TYPE_GPU
    p["act_model"][:] = 0
    p["act_kmask"][:] = 0b100
    p["act_pin_node"][:] = 0
    o = orc.assign(p)
    assert list(o["reason"]) == [0, 1] and list(o["node"]) == [0, -1]
    p["act_pin_node"][:] = -1
    p["gpu_pooled"] = 1
    o = orc.assign(p)
    assert list(o["reason"]) == [0, 0] and list(o["node"]) == [0, 1] and list(o["units"]) == [4, 4]
