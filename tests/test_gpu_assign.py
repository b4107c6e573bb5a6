"""GPU parity of tg_assign against the CPU oracle.  Integer outputs (node, units, ACT, defer
reason, counts, sums, per-node and per-task sums, per-node objective) must match bit for
bit; the two derived floats (mean ACT, utilisation) within 1e-9 relative."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tg():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_13019_amd import tg as _tg
    _tg.load()
    return _tg


def _assign_gpu(tg, p, use_cost=False):
    import torch
    P = tg.Problem(p)
    cost = P.score() if use_cost else None
    bufs = P.alloc_assign()
    for k in ("node", "units", "act_us", "defer_reason", "node_used", "task_sum_us", "node_obj", "core_set"):
        if k in bufs:
            bufs[k].fill_(-3 if bufs[k].dtype != torch.uint8 else 77)      # every entry must be written
    P.assign(cost, bufs)
    torch.cuda.synchronize()
    out = {k: v.cpu().numpy() for k, v in bufs.items() if k not in ("ws", "summary")}
    out["summary"] = tg.summary_to_numpy(bufs["summary"])
    P.free()
    return out


def _compare(got, want, where=""):
    for k_got, k_want in (("defer_reason", "reason"), ("node", "node"), ("units", "units"), ("act_us", "act_us"),
                          ("node_used", "node_used"), ("task_sum_us", "task_sum"), ("node_obj", "node_obj")):
        np.testing.assert_array_equal(got[k_got], want[k_want], err_msg=f"{where} {k_got}")
    gs, ws = got["summary"], want["summary"]
    for k_got, k_want in (("sum_act_us", "sum_act_us"), ("n_selected", "n_assigned"), ("n_prefix", "n_prefix"),
                          ("n_evicted", "n_evicted"), ("n_infeasible", "n_infeasible"),
                          ("units_used", "units_used"), ("units_free", "units_free")):
        np.testing.assert_array_equal(gs[k_got], ws[k_want], err_msg=f"{where} summary.{k_got}")
    np.testing.assert_allclose(gs["mean_act_us"], ws["mean_act_us"], rtol=1e-9, atol=0)
    np.testing.assert_allclose(gs["util"], ws["util"], rtol=1e-9, atol=0)
    assert ("core_set" in got) == ("core_set" in want)
    if "core_set" in want:
        np.testing.assert_array_equal(got["core_set"].view(np.uint64), want["core_set"], err_msg=f"{where} core_set")


@pytest.mark.parametrize("seed", range(24))
def test_assign_random_problems(tg, orc, seed):
    print("case", seed, flush=True)
    p = gen.make_random_problem(seed, B=4, N=60 + 7 * seed, n_cpu=1 + seed % 4, n_gpu=seed % 3, n_api=seed % 2 + (seed % 5 == 0),
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=24 + 8 * (seed % 3))
    _compare(_assign_gpu(tg, p, use_cost=seed % 4 == 3), orc.assign(p), f"seed {seed}")


@pytest.mark.parametrize("case", ["single_action", "zero_capacity", "all_pinned_one_node", "all_nonelastic", "k1", "ties"])
def test_assign_degenerate(tg, orc, case):
    print("case", case, flush=True)
    if case == "single_action":
        p = gen.make_random_problem(3, B=2, N=1, n_cpu=1, n_gpu=1, n_api=1, bad_frac=0.0)
    elif case == "zero_capacity":
        p = gen.make_random_problem(4, B=2, N=50)
        p["node_free"][:] = 0
        p["node_chunks"][:] = 0
        p["node_busy_off"], p["node_busy_rel_us"] = None, None
    elif case == "all_pinned_one_node":
        p = gen.make_random_problem(5, B=2, N=80, n_cpu=3, n_gpu=0, n_api=0, shuffle_nodes=False)
        p["act_pin_node"][:] = 1
    elif case == "all_nonelastic":
        p = gen.make_random_problem(6, B=2, N=80)
        p["act_model"][:] = 0
    elif case == "k1":
        p = gen.make_random_problem(7, B=2, N=80, n_gpu=0, k_list=(1,))
    else:
        p = gen.make_random_problem(8, B=2, N=120, n_cpu=4, n_gpu=2, n_api=0, bad_frac=0.0)
        p["act_t_ori_us"][:] = 1_000_000                        # identical durations: every choice is a tie
        p["act_param"][p["act_model"] == 1] = 900_000
        p["node_backlog_us"][:] = 0
    _compare(_assign_gpu(tg, p), orc.assign(p), case)


@pytest.mark.parametrize("seed", [40, 41, 42, 43])
def test_assign_wide_times(tg, orc, seed):
    """Durations close to 2^36 us and backlogs close to 2^40: sums leave 32 bits, so the 64-bit
    paths of the dynamic program and of the heap estimate are the ones that run."""
    print("case wide", seed, flush=True)
    p = gen.make_random_problem(seed, B=3, N=90, n_cpu=2 + seed % 2, n_gpu=1, n_api=1, depth=2, busy=seed % 2 == 0)
    rng = np.random.default_rng(seed)
    p["act_t_ori_us"] = np.minimum(p["act_t_ori_us"] * rng.integers(2000, 9000, p["act_t_ori_us"].shape), (1 << 36) - 1)
    p["node_backlog_us"] = p["node_backlog_us"] * 200_000 + (p["node_type"] != gen.TYPE_API) * ((1 << 39) * (seed % 2))
    if p.get("node_busy_rel_us") is not None:
        p["node_busy_rel_us"] = p["node_busy_rel_us"] * 100_000
    _compare(_assign_gpu(tg, p), orc.assign(p), f"wide {seed}")


def _roomy(p, cap, min1_frac, seed):
    """CPU nodes get `cap` units, all free but the busy ones, and most CPU actions may run on one
    unit, so that nodes collect long candidate lists instead of closing their pool early."""
    rng = np.random.default_rng(seed)
    cpu = p["node_type"] == gen.TYPE_CPU
    nb = np.zeros(len(cpu), np.int64)
    if p.get("node_busy_off") is not None:
        nb = np.diff(p["node_busy_off"])
        assert nb[cpu].max(initial=0) <= cap, "generate with cpu_cap_hi <= cap"
    p["node_cap"][cpu] = cap
    p["node_free"][cpu] = (cap - nb)[cpu]
    a = (p["act_type"] == gen.TYPE_CPU) & (rng.random(len(p["act_type"])) < min1_frac)
    p["act_kmask"][a] |= 1
    return p


CODE_PATHS = {
    # pools of 65..256 nodes: node table in four register slots per lane; tight capacities so
    # that pinned actions close nodes and unpinned ones close whole pools
    "pool_150_cpu_70_gpu_nodes": (dict(seed=50, B=2, N=1500, n_cpu=150, n_gpu=70, n_api=3, cpu_cap_hi=6, pin_frac=0.4), (6, 0.97)),
    # 257..1024 nodes of a kind: sixteen register slots per lane
    "pool_300_cpu_nodes": (dict(seed=51, B=1, N=2000, n_cpu=300, n_gpu=0, n_api=0, cpu_cap_hi=5, pin_frac=0.3), (5, 0.97)),
    # more than 1024 nodes of a kind: node table in LDS
    "pool_1100_cpu_nodes": (dict(seed=60, B=1, N=4000, n_cpu=1100, n_gpu=0, n_api=0, cpu_cap_hi=3, pin_frac=0.3), (3, 0.97)),
    # 256 units per node, some busy: four heap slots per lane, 256-wide DP rows, > 128 candidates
    "cap_256_nodes": (dict(seed=52, B=2, N=700, n_cpu=2, n_gpu=0, n_api=0, cpu_cap_hi=40, k_list=(1, 2, 4, 8, 16)), (256, 0.995)),
    "cap_200_no_busy": (dict(seed=53, B=2, N=500, n_cpu=1, n_gpu=1, n_api=1, cpu_cap_hi=40, busy=False, k_list=(1, 2, 4, 8, 16)), (200, 0.995)),
    # the deepest and an odd depth of Alg. 2 (depths run in pairs)
    "depth_4": (dict(seed=54, B=3, N=150, n_cpu=2, n_gpu=2, n_api=1, cpu_cap_hi=40, depth=4, k_list=(1, 2, 4, 8, 16)), (40, 0.95)),
    "depth_3": (dict(seed=55, B=3, N=150, n_cpu=3, n_gpu=1, n_api=0, cpu_cap_hi=24, depth=3, k_list=(1, 2, 4, 8, 16)), (24, 0.95)),
    # eight options (the 32-bit DP is specialised on the option count)
    "eight_options": (dict(seed=56, B=2, N=200, n_cpu=2, n_gpu=0, n_api=1, cpu_cap_hi=64, k_list=(1, 2, 3, 4, 6, 8, 12, 16)), (64, 0.95)),
    "three_options": (dict(seed=57, B=2, N=200, n_cpu=3, n_gpu=1, n_api=1, cpu_cap_hi=20, k_list=(1, 2, 4)), (20, 0.95)),
    # sums of durations between 2^30 and 2^32 us: 64-bit DP totals, 32-bit heap times
    "dp_totals_beyond_30_bits": (dict(seed=58, B=2, N=160, n_cpu=1, n_gpu=1, n_api=0, cpu_cap_hi=64, t_median=40_000_000), (64, 0.99)),
    # many waiting actions pinned to a node (more than the wavefront stages in LDS)
    "long_pinned_queues": (dict(seed=59, B=2, N=900, n_cpu=2, n_gpu=1, n_api=0, cpu_cap_hi=48, pin_frac=0.9), (48, 0.9)),
}


def _code_path_problem(case):
    kw, (cap, min1) = CODE_PATHS[case]
    p = _roomy(gen.make_random_problem(**kw), cap, min1, kw["seed"])
    if kw["n_gpu"] == 0:
        p["type_k"][gen.TYPE_GPU] = 0        # no GPU kind: its options need not be buddy sizes
    return p


@pytest.mark.parametrize("case", sorted(CODE_PATHS))
def test_assign_code_paths(tg, orc, case):
    """Shapes chosen so that every variant of the kernels' inner loops runs at least once."""
    print("case", case, flush=True)
    p = _code_path_problem(case)
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p), want, case)
    assert (want["reason"] == 0).any() and (want["reason"] == 1).any(), "the case should select and defer"


@pytest.mark.parametrize("seed", range(10))
def test_assign_cost_order_random_problems(tg, orc, seed):
    """Second visiting order (least estimated ACT first): keys, sort and everything downstream."""
    print("case cost order", seed, flush=True)
    p = gen.make_random_problem(200 + seed, B=3, N=80 + 40 * seed, n_cpu=1 + seed % 4, n_gpu=seed % 3, n_api=seed % 2,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=24 + 8 * (seed % 3))
    p["order_policy"] = 1
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p, use_cost=seed % 3 == 2), want, f"cost order {seed}")
    fcfs = orc.assign(dict(p, order_policy=0))
    assert (fcfs["reason"] != want["reason"]).any() or (fcfs["node"] != want["node"]).any(), "the order should matter"


def test_assign_cost_order_code_paths(tg, orc):
    for case in ("pool_150_cpu_70_gpu_nodes", "cap_256_nodes", "long_pinned_queues"):
        print("case cost order", case, flush=True)
        p = _code_path_problem(case)
        p["order_policy"] = 1
        _compare(_assign_gpu(tg, p), orc.assign(p), f"cost order {case}")


LARGE_POOLS = {
    # pools beyond the 8192 keys one workgroup sorts: runs merged pairwise in 1, 2, 3 and 4 passes; a last run of one key;
    # runs that stay single through a pass; pools of very different size side by side
    "two_runs_one_key": dict(seed=70, B=1, N=8193, n_cpu=40, n_gpu=0, n_api=0, cpu_cap_hi=6, pin_frac=0.2, type_probs=(1, 0, 0)),
    "three_runs": dict(seed=71, B=1, N=20000, n_cpu=120, n_gpu=0, n_api=0, cpu_cap_hi=6, pin_frac=0.3, type_probs=(1, 0, 0)),
    "five_runs_two_kinds": dict(seed=72, B=2, N=48000, n_cpu=150, n_gpu=30, n_api=2, cpu_cap_hi=6, pin_frac=0.2, type_probs=(0.8, 0.15, 0.05)),
    "nine_runs": dict(seed=73, B=1, N=70000, n_cpu=200, n_gpu=0, n_api=0, cpu_cap_hi=6, pin_frac=0.1, type_probs=(1, 0, 0)),
    "the_largest_queue": dict(seed=74, B=1, N=131072, n_cpu=250, n_gpu=0, n_api=0, cpu_cap_hi=6, pin_frac=0.1, type_probs=(1, 0, 0)),
}


@pytest.mark.parametrize("case", list(LARGE_POOLS))
def test_assign_cost_order_large_pools(tg, orc, case):
    """Second visiting order on pools larger than one workgroup sorts: sorted runs, merged pairwise."""
    print("case cost order", case, flush=True)
    kw = LARGE_POOLS[case]
    p = _roomy(gen.make_random_problem(**kw), 128, 0.9, kw["seed"])
    if kw["n_gpu"] == 0:
        p["type_k"][gen.TYPE_GPU] = 0
    p["order_policy"] = 1
    want = orc.assign(p)
    assert (want["reason"] == 0).sum() > 2000 and (want["reason"] == 1).any(), "the case should select many and defer"
    _compare(_assign_gpu(tg, p), want, case)
    if case == "three_runs":
        p["queue_prefix"] = 1                                      # the place of every action in the order of the whole queue
        _compare(_assign_gpu(tg, p), orc.assign(p), case + " whole-queue prefix")


def test_assign_cost_order_config4_full(tg, orc):
    """Workload 4 (one snapshot, a CPU pool of 52 000 actions) under the second visiting order."""
    p = gen.make_config(4)
    p["order_policy"] = 1
    _compare(_assign_gpu(tg, p), orc.assign(p))


def test_assign_cost_order_config2_full(tg, orc):
    """Workload 2 at full size under the second visiting order."""
    p = gen.make_config(2)
    p["order_policy"] = 1
    _compare(_assign_gpu(tg, p), orc.assign(p))


def _add_second_resource(p, seed, scarce):
    """Memory-like demand per action and what every node has left of it (Sec. 4.1's cost vector)."""
    rng = np.random.default_rng(seed + 77)
    p["act_aux"] = rng.integers(0, 40, p["B"] * p["N"]).astype(np.int32)
    p["node_aux_free"] = rng.integers(0, 150 if scarce else 5000, p["B"] * p["M"]).astype(np.int32)
    return p


def _add_services(p, seed, n_services=6, resident_frac=0.5, big=False):
    """Which service every action calls, which services every node caches, restore times (Sec. 5.3)."""
    rng = np.random.default_rng(seed + 900)
    n, m = p["B"] * p["N"], p["B"] * p["M"]
    p["act_service"] = rng.integers(-1, n_services, n).astype(np.int32)
    bits = rng.random((m, n_services)) < resident_frac
    res = np.zeros(m, np.uint64)
    for sv in range(n_services):
        res |= bits[:, sv].astype(np.uint64) << np.uint64(sv)
    p["node_resident"] = res
    unit = 40_000_000_000 if big else 250_000                  # big: delays beyond 32 bits
    p["restore_us"] = np.minimum(rng.integers(0, 9, n_services) * unit, (1 << 36) - 1).astype(np.int64)
    return p


@pytest.mark.parametrize("seed", range(8))
def test_assign_services_random_problems(tg, orc, seed):
    print("case services", seed, flush=True)
    p = gen.make_random_problem(600 + seed, B=3, N=150 + 60 * seed, n_cpu=2 + seed % 4, n_gpu=1 + seed % 3, n_api=seed % 2,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=32 + 16 * (seed % 3), pin_frac=0.3)
    p["act_kmask"][p["act_type"] == gen.TYPE_CPU] |= 1
    base = orc.assign(p)
    _add_services(p, seed, n_services=(3, 17, 64)[seed % 3], big=seed == 7)
    p["order_policy"] = seed % 2
    if seed % 4 == 3:
        _add_second_resource(p, seed, scarce=True)
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p, use_cost=seed % 3 == 1), want, f"services {seed}")
    if p["order_policy"] == 0 and seed % 4 != 3:
        assert (base["act_us"] != want["act_us"]).any(), "restore delays should show"


def test_assign_services_code_paths(tg, orc):
    for case in ("pool_150_cpu_70_gpu_nodes", "pool_300_cpu_nodes", "pool_1100_cpu_nodes", "cap_256_nodes", "long_pinned_queues",
                 "dp_totals_beyond_30_bits"):
        for order in (0, 1):
            print("case services", case, order, flush=True)
            p = _add_services(_code_path_problem(case), 6, n_services=9)
            p["order_policy"] = order
            _compare(_assign_gpu(tg, p), orc.assign(p), f"services {case} order {order}")


def test_assign_services_config2_full(tg, orc):
    """Workload 2 at full size with 8 services cached on half of the nodes each."""
    p = _add_services(gen.make_config(2), 2, n_services=8)
    _compare(_assign_gpu(tg, p), orc.assign(p))


@pytest.mark.parametrize("seed", range(8))
def test_assign_second_resource_random_problems(tg, orc, seed):
    print("case second resource", seed, flush=True)
    p = gen.make_random_problem(400 + seed, B=3, N=150 + 60 * seed, n_cpu=2 + seed % 4, n_gpu=seed % 3, n_api=seed % 2,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=32 + 16 * (seed % 3), pin_frac=0.3)
    a = (p["act_type"] == gen.TYPE_CPU)
    p["act_kmask"][a] |= 1
    base = orc.assign(p)
    _add_second_resource(p, seed, scarce=True)
    p["order_policy"] = seed % 2
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p, use_cost=seed % 3 == 1), want, f"second resource {seed}")
    if p["order_policy"] == 0:
        assert (base["node"] != want["node"]).any(), "a scarce second resource should change the placement"


def test_assign_second_resource_code_paths(tg, orc):
    for case in ("pool_150_cpu_70_gpu_nodes", "pool_300_cpu_nodes", "pool_1100_cpu_nodes", "cap_256_nodes"):
        print("case second resource", case, flush=True)
        p = _add_second_resource(_code_path_problem(case), 5, scarce=True)
        _compare(_assign_gpu(tg, p), orc.assign(p), f"second resource {case}")


def _sweep_problem(seed):
    rng = np.random.default_rng(seed)
    k_all = [1, 2, 4, 8, 16, 32]
    kw = dict(B=int(rng.integers(1, 4)), N=int(rng.integers(1, 700)) if seed % 7 else int(rng.integers(700, 3000)),
              n_cpu=int(rng.integers(0, 6)), n_gpu=int(rng.integers(0, 4)), n_api=int(rng.integers(0, 3)),
              cpu_cap_hi=int(rng.choice([4, 16, 40, 100, 256])), k_list=tuple(k_all[:int(rng.integers(1, 7))]),
              depth=int(rng.integers(1, 5)), busy=bool(rng.integers(0, 2)), pin_frac=float(rng.choice([0.0, 0.3, 0.8])),
              t_median=int(rng.choice([20_000, 2_000_000, 60_000_000])))
    if kw["n_cpu"] + kw["n_gpu"] + kw["n_api"] == 0:
        kw["n_cpu"] = 1
    p = gen.make_random_problem(seed, **kw)
    if rng.random() < 0.5:                                   # long candidate lists instead of early pool closure
        a = (p["act_type"] == gen.TYPE_CPU) & (rng.random(len(p["act_type"])) < 0.95)
        p["act_kmask"][a] |= 1
    if kw["n_gpu"] == 0:
        p["type_k"][gen.TYPE_GPU] = 0
    p["order_policy"] = int(rng.integers(0, 2))
    if rng.random() < 0.5:
        _add_second_resource(p, seed, scarce=bool(rng.integers(0, 2)))
    if rng.random() < 0.5:
        _add_services(p, seed, n_services=int(rng.choice([1, 5, 64])), big=bool(rng.integers(0, 2)))
    use_cost = bool(rng.integers(0, 2))
    if kw["n_gpu"] and p.get("act_service") is None and rng.random() < 0.5:
        _pooled(p)                                           # the GPU nodes as one pool of chunks
        if _pool_states(p) > 512:
            p["gpu_pooled"] = 0
    if rng.random() < 0.5:
        gen.with_extra_quotas(p, frac=float(rng.random()), seed=seed, max_extra=int(rng.integers(1, 6)))
    if rng.random() < 0.5:
        gen.with_core_maps(p, int(rng.choice([4, 8, 16, 32, 64])), seed)
    p["queue_prefix"] = int(rng.random() < 0.3)              # one prefix of the whole queue instead of one per pool
    return p, use_cost


def test_assign_random_sweep(tg, orc):
    """200 problems with every parameter drawn at random (sizes, kinds, capacities, options, depth, busy
    lists, pins, duration scale, visiting order, second resource, services, pooled GPUs, several quotas, core maps, whole-queue prefix,
    with and without the score tensor)."""
    for seed in range(3000, 3200):
        p, use_cost = _sweep_problem(seed)
        _compare(_assign_gpu(tg, p, use_cost=use_cost), orc.assign(p), f"sweep seed {seed}")
    print("200 problems compared", flush=True)


@pytest.mark.parametrize("case", ["max_actions_per_snapshot", "max_nodes_of_a_kind"])
def test_assign_at_the_limits(tg, orc, case):
    """The largest snapshot (131 072 actions) and the largest pool (4096 nodes of one kind) the interface takes."""
    print("case", case, flush=True)
    if case == "max_actions_per_snapshot":
        p = gen.make_random_problem(77, B=1, N=131072, n_cpu=500, n_gpu=0, n_api=0, cpu_cap_hi=64, busy=False, pin_frac=0.2,
                                    k_list=(1, 2, 4, 8, 16, 32, 48, 64))
        cap = 64
    else:
        p = gen.make_random_problem(78, B=1, N=16000, n_cpu=4096, n_gpu=0, n_api=0, cpu_cap_hi=8, busy=False, pin_frac=0.2)
        cap = 8
    p["type_k"][gen.TYPE_GPU] = 0
    _roomy(p, cap, 0.999, 1)
    want = orc.assign(p)
    assert (want["reason"] == 0).sum() > 5000 and (want["reason"] == 2).any()
    _compare(_assign_gpu(tg, p), want, case)


def test_assign_config1(tg, orc):
    p = gen.make_config(1)
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p), want)
    _compare(_assign_gpu(tg, p, use_cost=True), want)


def test_assign_config2_full(tg, orc):
    """Workload 2 at full size (B=256, N=1024) in the launch configuration bench.py times."""
    p = gen.make_config(2)
    _compare(_assign_gpu(tg, p), orc.assign(p))


def test_assign_config3_sampled(tg, orc):
    """Workload 3 at full size on the GPU; the oracle re-runs 12 of the 1024 snapshots."""
    p = gen.make_config(3)
    got = _assign_gpu(tg, p)
    pick = [0, 1, 2, 3, 255, 256, 511, 700, 900, 1021, 1022, 1023]
    want = orc.assign(gen.slice_problem(p, pick))
    N, M, T = p["N"], p["M"], p["n_tasks"]
    sub = {}
    for k, per in (("defer_reason", N), ("node", N), ("units", N), ("act_us", N), ("node_used", M),
                   ("task_sum_us", T), ("node_obj", M), ("summary", 1)):
        sub[k] = np.concatenate([got[k][b * per:(b + 1) * per] for b in pick])
    _compare(sub, want)
    # properties over all snapshots: capacity never exceeded, counts add up
    used = got["node_used"].reshape(p["B"], M)
    assert (used <= p["node_free"].reshape(p["B"], M)).all()
    s = got["summary"]
    assert ((s["n_selected"] + s["n_prefix"] + s["n_evicted"] + s["n_infeasible"]) == N).all()


def test_assign_config4_full(tg, orc):
    """Workload 4 (one snapshot, N=65536, 1152 nodes): the latency case."""
    p = gen.make_config(4)
    _compare(_assign_gpu(tg, p), orc.assign(p))


@pytest.mark.parametrize("seed", range(10))
def test_assign_core_sets_random_problems(tg, orc, seed):
    """Sec. 5.2: the cores of every selected CPU action, bit for bit, over all domain sizes."""
    print("case core sets", seed, flush=True)
    p = gen.make_random_problem(800 + seed, B=3, N=150 + 50 * seed, n_cpu=2 + seed % 4, n_gpu=seed % 2, n_api=seed % 2,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=(24, 64, 130, 256)[seed % 4], pin_frac=0.3)
    p["order_policy"] = seed % 2
    gen.with_core_maps(p, (4, 8, 16, 32, 64)[seed % 5], seed)
    want = orc.assign(p)
    assert want["core_set"].any()
    _compare(_assign_gpu(tg, p), want, f"core sets {seed}")


def test_assign_core_sets_code_paths(tg, orc):
    for case, numa in (("cap_256_nodes", 4), ("cap_256_nodes", 64), ("pool_300_cpu_nodes", 8), ("long_pinned_queues", 16),
                       ("eight_options", 32)):
        print("case core sets", case, numa, flush=True)
        p = gen.with_core_maps(_code_path_problem(case), numa, 3)
        _compare(_assign_gpu(tg, p), orc.assign(p), f"core sets {case} numa {numa}")


def test_assign_core_sets_fragmented_nodes(tg, orc):
    """Few free cores scattered over many small domains: most actions have to span domains."""
    p = gen.make_random_problem(860, B=4, N=300, n_cpu=4, n_gpu=0, n_api=0, cpu_cap_hi=256, busy=True, pin_frac=0.2)
    gen.with_core_maps(p, 4, 9)
    want = orc.assign(p)
    sets = want["core_set"].reshape(-1, 4)
    spans = 0
    for g in np.flatnonzero(want["units"] > 1):
        doms = {c // 4 for w in range(4) for c in range(64 * w, 64 * w + 64) if int(sets[g][w]) >> (c % 64) & 1}
        spans += len(doms) > 1
    assert spans > 5
    _compare(_assign_gpu(tg, p), want, "fragmented")


def test_assign_core_sets_config2_full(tg, orc):
    """Workload 2 at full size with a core map per CPU node (domains of 16 cores)."""
    p = gen.with_core_maps(gen.make_config(2), 16, 2)
    _compare(_assign_gpu(tg, p), orc.assign(p))


@pytest.mark.parametrize("seed", range(10))
def test_assign_several_quotas_random_problems(tg, orc, seed):
    """Sec. 4.1: API actions that draw a token from several quotas at once; with and without the score tensor
    (register-resident and LDS node table), under both visiting orders."""
    print("case several quotas", seed, flush=True)
    p = gen.make_random_problem(900 + seed, B=3, N=200 + 60 * seed, n_cpu=1 + seed % 3, n_gpu=seed % 2, n_api=2 + (7 * seed) % 30,
                                depth=1 + seed % 3, busy=seed % 2 == 0, pin_frac=0.3, type_probs=(0.4, 0.1, 0.5))
    base = orc.assign(p)
    gen.with_extra_quotas(p, frac=0.6, seed=seed, max_extra=1 + seed % 4)
    p["order_policy"] = seed % 2
    if seed % 3 == 2:
        _add_second_resource(p, seed, scarce=False)
    want = orc.assign(p)
    assert (base["reason"] != want["reason"]).any() or p["order_policy"] == 1
    _compare(_assign_gpu(tg, p, use_cost=seed % 2 == 1), want, f"several quotas {seed}")


def test_assign_several_quotas_many_api_nodes(tg, orc):
    """70 and 300 quotas in a snapshot: node tables of 4 and 16 register slots; the masks name quotas among the first 64."""
    for n_api in (70, 300):
        print("case several quotas", n_api, flush=True)
        p = gen.make_random_problem(930 + n_api, B=2, N=1500, n_cpu=1, n_gpu=0, n_api=n_api, type_probs=(0.1, 0.0, 0.9))
        p["type_k"][gen.TYPE_GPU] = 0
        gen.with_extra_quotas(p, frac=0.7, seed=n_api, max_extra=5)
        _compare(_assign_gpu(tg, p), orc.assign(p), f"several quotas, {n_api} API nodes")


def _pooled(p):
    """All GPU nodes of a snapshot share one backlog (a pool has one queueing term) and form one pool."""
    M = p["M"]
    for b in range(p["B"]):
        g = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        if len(g):
            p["node_backlog_us"][g] = p["node_backlog_us"][g[0]]
    p["act_pin_node"][p["act_type"] == gen.TYPE_GPU] = -1      # actions are not pinned to a node of a pool
    p["gpu_pooled"] = 1
    return p


def _pool_states(p):
    """Largest number of chunk states a pool of the problem needs (the interface takes up to 512)."""
    M, worst = p["M"], 1
    ch = p["node_chunks"].reshape(-1, 4).astype(np.int64)
    for b in range(p["B"]):
        g = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        if len(g):
            c = ch[g].sum(axis=0)
            worst = max(worst, int(np.prod(np.maximum(c, 1) + 1)))
    return worst


@pytest.mark.parametrize("seed", range(12))
def test_assign_pooled_gpus_random_problems(tg, orc, seed):
    """Sec. 5.3 / Alg. 4 with the GPU cluster as one pool of chunks: units, ACT, reasons and the node whose
    chunk every action gets."""
    print("case pooled", seed, flush=True)
    n_gpu = 1 + seed % 5
    p = _pooled(gen.make_random_problem(1000 + seed, B=4, N=100 + 30 * seed, n_cpu=1 + seed % 2, n_gpu=n_gpu, n_api=seed % 2,
                                        depth=1 + seed % 3, busy=seed % 2 == 0, pin_frac=0.0, type_probs=(0.3, 0.6, 0.1)))
    if _pool_states(p) > 512:
        pytest.skip("pooled chunk counts beyond the supported number of states")
    p["order_policy"] = seed % 2
    want = orc.assign(p)
    assert (want["units"][p["act_type"] == gen.TYPE_GPU] > 0).sum() > 3
    _compare(_assign_gpu(tg, p, use_cost=seed % 3 == 1), want, f"pooled {seed}")


def test_assign_pooled_gpus_eight_free_nodes(tg, orc):
    """The largest pool: eight nodes of eight free GPUs, a long queue of elastic GPU actions."""
    p = gen.make_random_problem(1040, B=3, N=400, n_cpu=1, n_gpu=8, n_api=0, pin_frac=0.0, busy=False, type_probs=(0.1, 0.9, 0.0))
    g = p["node_type"] == gen.TYPE_GPU
    p["node_free"][g] = 8
    ch = p["node_chunks"].reshape(-1, 4)
    ch[g] = (0, 0, 0, 1)
    a = p["act_type"] == gen.TYPE_GPU
    p["act_kmask"][a] |= 1
    _pooled(p)
    want = orc.assign(p)
    assert (want["node_used"][g] > 0).all()                       # every node of the pool hands out chunks
    _compare(_assign_gpu(tg, p), want, "pooled, 8 nodes")


def test_assign_pooled_gpus_config2_full(tg, orc):
    """Workload 2 at full size with the eight GPU nodes of every snapshot as one pool (GPU actions unpinned, the
    GPU nodes of a snapshot at their mean backlog)."""
    p = gen.make_config(2)
    M = p["M"]
    for b in range(p["B"]):
        g = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        p["node_backlog_us"][g] = int(p["node_backlog_us"][g].mean())
    _pooled(p)
    want = orc.assign(p)
    gpu = p["node_type"] == gen.TYPE_GPU
    assert (want["node_used"][gpu] > 0).mean() > 0.9
    _compare(_assign_gpu(tg, p), want)


def test_assign_several_quotas_config3_slice(tg, orc):
    """48 snapshots of workload 3 (4096 actions, 16 quotas each) in which half of the API actions draw on up to three
    further quotas."""
    p = gen.slice_problem(gen.make_config(3), range(0, 1024, 22))
    gen.with_extra_quotas(p, frac=0.5, seed=3)
    want = orc.assign(p)
    base = orc.assign(dict(p, act_quota_mask=None))
    assert (want["reason"] != base["reason"]).any()
    _compare(_assign_gpu(tg, p), want)


@pytest.mark.parametrize("seed", range(16))
def test_assign_queue_prefix_random_problems(tg, orc, seed):
    """One admitted prefix of the whole queue (Alg. 1 as printed): both visiting orders, with and without the
    score tensor, next to the second resource, services, several quotas, core maps and pooled GPUs."""
    print("case", seed, flush=True)
    p = gen.make_random_problem(1300 + seed, B=4, N=80 + 25 * seed, n_cpu=1 + seed % 4, n_gpu=1 + seed % 3, n_api=seed % 3,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=24 + 8 * (seed % 3),
                                pin_frac=(0.0, 0.3, 0.8)[seed % 3])
    if seed % 4 == 1:
        _add_second_resource(p, seed, scarce=False)
    if seed % 4 == 2:
        _add_services(p, seed)
    if seed % 4 == 3 and seed % 3:
        gen.with_extra_quotas(p, 0.5, seed)
    if seed % 5 == 0:
        gen.with_core_maps(p, 8, seed)
    if seed % 4 == 0:
        _pooled(p)
    p["queue_prefix"] = 1
    p["order_policy"] = seed // 2 % 2
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p, use_cost=seed % 2 == 1), want, f"seed {seed}")
    per_pool = orc.assign(dict(p, queue_prefix=0))
    assert (per_pool["reason"] != want["reason"]).any(), "the whole-queue prefix should bind here"


def test_assign_queue_prefix_code_paths(tg, orc):
    for case in sorted(CODE_PATHS):
        for order in (0, 1):
            print("case", case, order, flush=True)
            p = dict(_code_path_problem(case), queue_prefix=1, order_policy=order)
            _compare(_assign_gpu(tg, p), orc.assign(p), f"{case} order {order}")


def test_assign_queue_prefix_config2_full(tg, orc):
    """Workload 2 at full size: the GPU pool of a snapshot runs out long before its CPU pool, so the one prefix
    ends early and far fewer actions are selected than with one prefix per pool."""
    p = dict(gen.make_config(2), queue_prefix=1)
    want = orc.assign(p)
    _compare(_assign_gpu(tg, p), want, "config 2")
    per_pool = orc.assign(dict(p, queue_prefix=0))
    assert want["summary"]["n_assigned"].sum() < per_pool["summary"]["n_assigned"].sum()
    p["order_policy"] = 1
    _compare(_assign_gpu(tg, p), orc.assign(p), "config 2, cost order")


def test_assign_queue_prefix_keeps_the_head(tg, orc):
    """The eviction loop never drops a node's first candidate, even where an empty selection would score better."""
    from test_oracle_queue_prefix import head_problem
    p, cpu = head_problem()
    want = orc.assign(p)
    assert want["reason"][0] == 0 and want["units"][0] == 8
    _compare(_assign_gpu(tg, p), want, "head kept")


@pytest.mark.parametrize("seed", range(8))
def test_assign_flat_elasticity_ties_everywhere(tg, orc, seed):
    """Every elastic action follows a table that gains nothing from more units (E(k) k = 1): all options of an action
    take the same time, so every comparison inside DPArrange is a tie - on CPU nodes fewer units win, on GPU nodes the
    smaller source state, the smaller option and the smallest end state."""
    print("case", seed, flush=True)
    p = gen.make_random_problem(1500 + seed, B=3, N=100 + 30 * seed, n_cpu=1 + seed % 3, n_gpu=1 + seed % 2, n_api=0,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=32, pin_frac=(0.0, 0.4)[seed % 2])
    p["speedup_q16"][:] = 65536
    el = p["act_model"] != 0
    p["act_model"][el] = 2
    p["act_param"][el] = np.arange(el.sum()) % p["n_classes"]
    if seed % 4 == 3:                                          # and one duration for everybody: ties between actions too
        p["act_t_ori_us"][:] = 700_000
    want = orc.assign(p)
    assert (want["reason"] == 0).any()
    _compare(_assign_gpu(tg, p), want, f"flat {seed}")


def test_assign_gpu_nodes_without_chunk_counts(tg, orc):
    """`node_chunks` absent: a GPU node with f free GPUs holds one free chunk per set bit of f.  Nine snapshots with
    0..8 free GPUs on their only node, and requests that fit, split or overflow it."""
    for need in ([8, 8, 1, 1, 1, 1], [4, 4, 4, 1, 1, 1], [1, 2, 4, 8, 1, 1], [2, 2, 2, 2, 2, 2]):
        p = gen.make_random_problem(31, B=9, N=6, n_cpu=0, n_gpu=1, n_api=0, bad_frac=0.0, pin_frac=0.0, busy=False)
        p["act_type"][:] = gen.TYPE_GPU
        p["act_model"][:] = 0
        p["node_cap"][:] = 8
        p["node_free"][:] = np.arange(9)
        p["node_busy_off"], p["node_busy_rel_us"] = None, None
        p["node_chunks"] = None
        p["act_kmask"][:] = np.tile([{1: 1, 2: 2, 4: 4, 8: 8}[k] for k in need], 9)
        want = orc.assign(p)
        _compare(_assign_gpu(tg, p), want, f"need {need}")
        assert (want["units"].reshape(9, 6).sum(axis=1) <= np.arange(9)).all()


def test_assign_quota_with_more_candidates_than_any_node_has_units(tg, orc):
    """A quota with hundreds of tokens next to CPU nodes of 4 cores: the quota's candidate list is far longer than the
    per-node tables (sized for the units of CPU and GPU nodes) - it needs none of them, its actions are not elastic."""
    p = gen.make_random_problem(1600, B=3, N=500, n_cpu=2, n_gpu=1, n_api=1, cpu_cap_hi=4, bad_frac=0.0, pin_frac=0.2,
                                type_probs=(0.15, 0.05, 0.8))
    api = p["node_type"] == gen.TYPE_API
    p["node_cap"][api] = 450
    p["node_free"][api] = 420
    want = orc.assign(p)
    N, M = p["N"], p["M"]
    per_quota = np.bincount(want["node"][(want["reason"] == 0)] + 0, minlength=M)
    assert want["node_used"][api].max() > 300
    _compare(_assign_gpu(tg, p), want, "long quota list")


@pytest.mark.parametrize("seed", range(10))
def test_assign_shared_node_table(tg, orc, seed):
    """nodes_shared: one node table for all snapshots.  The library, given the table once, must produce what the
    oracle produces for B copies of it - tensor, assignment and summaries - also with busy lists, a second
    resource, services and core maps in the table."""
    import torch
    p = gen.make_random_problem(300 + seed, B=5, N=50 + 9 * seed, n_cpu=1 + seed % 4, n_gpu=seed % 3, n_api=seed % 2,
                                depth=1 + seed % 3, busy=seed % 2 == 0, cpu_cap_hi=24 + 8 * (seed % 3))
    if seed % 3 == 1:
        _add_second_resource(p, seed, scarce=True)
    if seed % 3 == 2:
        _add_services(p, seed)
    if seed % 4 == 3:
        gen.with_core_maps(p, 8, seed)
    shared, expanded = gen.with_shared_nodes(p)
    assert len(shared["node_type"]) == p["M"] and len(expanded["node_type"]) == p["B"] * p["M"]
    want = orc.assign(expanded)
    _compare(_assign_gpu(tg, shared, use_cost=seed % 2 == 1), want, f"seed {seed}")
    P = tg.Problem(shared)
    cost = P.score()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cost.cpu().numpy(), orc.score(expanded))
    P.free()
    if seed == 0:
        shared["queue_prefix"] = expanded["queue_prefix"] = 1
        _compare(_assign_gpu(tg, shared), orc.assign(expanded), "whole-queue prefix")
