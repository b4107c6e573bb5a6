"""GPU parity of tg_replay_trace against the CPU oracle: start / finish / units / node of every
action and the per-scenario count, tick count and p99 bit for bit; mean ACT within 1e-9."""
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


def _replay_gpu(tg, t):
    import torch
    T = tg.Trace(t)
    bufs = T.alloc()
    for k in ("start_us", "finish_us", "units", "node", "p99_act_us", "n_started", "n_ticks", "core_set"):
        if k in bufs:
            bufs[k].fill_(-5)
    T.replay(bufs)
    torch.cuda.synchronize()
    out = {k: v.cpu().numpy() for k, v in bufs.items() if k != "ws"}
    T.free()
    return out


def _compare(got, want, scenarios, A):
    for s in scenarios:
        sl = slice(s * A, (s + 1) * A)
        for k in ("start_us", "finish_us", "units", "node"):
            np.testing.assert_array_equal(got[k][sl], want[k][sl], err_msg=f"scenario {s} {k}")
        assert got["n_started"][s] == want["n_started"][s]
        assert got["n_ticks"][s] == want["n_ticks"][s]
        assert got["p99_act_us"][s] == want["p99_act"][s]
        np.testing.assert_allclose(got["mean_act_us"][s], want["mean_act"][s], rtol=1e-9, atol=0)
        assert ("core_set" in got) == ("core_set" in want)
        if "core_set" in want:
            np.testing.assert_array_equal(got["core_set"].view(np.uint64)[4 * s * A:4 * (s + 1) * A], want["core_set"][4 * s * A:4 * (s + 1) * A],
                                          err_msg=f"scenario {s} core_set")


CASES = {
    "contended_small": dict(S=6, A=400, seed=21, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000),
    "contended_burst": dict(S=4, A=700, seed=22, contended=True, rate_per_s=400.0, horizon_s=2.0, max_ticks=30000),
    "default_cluster": dict(S=4, A=1500, seed=23, rate_per_s=50.0, horizon_s=30.0),
    "cpu_only_tiny_cluster": dict(S=5, A=300, seed=24, cluster=(2, 6, 0, 0), rate_per_s=30.0, horizon_s=10.0, max_ticks=50000),
    "gpu_only": dict(S=5, A=300, seed=25, cluster=(0, 0, 3, 0), type_probs=(0, 1, 0), rate_per_s=30.0, horizon_s=10.0, max_ticks=50000),
    "api_only": dict(S=3, A=500, seed=26, cluster=(0, 0, 0, 2), type_probs=(0, 0, 1), rate_per_s=300.0, horizon_s=2.0, max_ticks=50000),
    "tick_limit": dict(S=3, A=500, seed=27, contended=True, rate_per_s=500.0, horizon_s=1.0, max_ticks=40),
    "single_action": dict(S=2, A=1, seed=28, contended=True),
}


@pytest.mark.parametrize("name", list(CASES))
def test_replay_small(tg, orc, name):
    print("case", name, flush=True)
    t = gen.make_trace(**CASES[name])
    want = orc.replay(t)
    got = _replay_gpu(tg, t)
    _compare(got, want, range(t["S"]), t["A"])


def test_replay_random_sweep(tg, orc):
    """60 small traces with cluster shape, load, tick limit, pins, depth, further quotas, services and the prefix rule
    drawn at random."""
    for seed in range(500, 560):
        t = gen.random_trace(seed)
        _compare(_replay_gpu(tg, t), orc.replay(t), range(t["S"]), t["A"])
    print("60 traces compared", flush=True)


_with_aux = gen.trace_with_aux
_with_services = gen.trace_with_services


@pytest.mark.parametrize("seed", range(8))
def test_replay_service_cache(tg, orc, seed):
    """Restore delays and the per-node LRU cache of resident services (Sec. 5.3)."""
    print("case service cache", seed, flush=True)
    t = gen.make_trace(S=3, A=500 + 100 * seed, seed=170 + seed, cluster=(1 + seed % 2, 16, 1 + seed % 3, seed % 2),
                       type_probs=(0.2, 0.7, 0.1) if seed % 2 else (0.3, 0.7, 0.0),
                       rate_per_s=(30.0, 60.0, 150.0)[seed % 3], horizon_s=12.0, max_ticks=80000, pin_frac=0.3)
    base = orc.replay(t)
    _with_services(t, seed, n_services=(2, 5, 9, 64)[seed % 4], slots=(1, 2, 3, 64)[(seed // 2) % 4])
    want = orc.replay(t)
    assert (want["finish_us"] != base["finish_us"]).any()
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])


def test_replay_service_cache_many_gpu_nodes(tg, orc):
    """More than 64 GPU nodes: the pool with services takes the LDS node table."""
    t = gen.make_trace(S=2, A=1500, seed=181, cluster=(0, 0, 70, 0), type_probs=(0, 1, 0), rate_per_s=400.0, horizon_s=4.0,
                       max_ticks=80000, pin_frac=0.2)
    _with_services(t, 9, n_services=12, slots=2)
    _compare(_replay_gpu(tg, t), orc.replay(t), range(t["S"]), t["A"])


def test_replay_depth_and_ties(tg, orc):
    t = gen.make_trace(S=4, A=500, seed=31, contended=True, rate_per_s=120.0, horizon_s=4.0, max_ticks=30000)
    t["depth"] = 3
    t["act_t_ori_us"][:] = (t["act_t_ori_us"] // 500_000 + 1) * 500_000      # few distinct durations: ties
    _compare(_replay_gpu(tg, t), orc.replay(t), range(4), 500)


def test_replay_config5_sampled(tg, orc):
    """Workload 5 shape (10 000 arrivals over 200 s per scenario, default cluster) on 64 scenarios in one
    launch; the oracle replays 3 of them."""
    t = gen.make_trace(S=64, A=10_000, seed=4)
    got = _replay_gpu(tg, t)
    pick = [0, 31, 63]
    want = orc.replay(t, 0, 1)
    for s in pick[1:]:
        w = orc.replay(t, s, s + 1)
        for k in want:
            if want[k].shape[0] == t["S"]:
                want[k][s] = w[k][s]
            else:
                want[k][s * t["A"]:(s + 1) * t["A"]] = w[k][s * t["A"]:(s + 1) * t["A"]]
    _compare(got, want, pick, t["A"])
    assert (got["n_started"] == t["A"]).all()
    assert (got["start_us"] >= t["arrival_us"]).all() and (got["start_us"] % t["tick_us"] == 0).all()


def test_replay_config5_contended_sampled(tg, orc):
    t = gen.make_trace(S=32, A=10_000, seed=5, contended=True, max_ticks=200_000)
    got = _replay_gpu(tg, t)
    pick = [0, 31]
    want = orc.replay(t, 0, 1)
    w = orc.replay(t, 31, 32)
    for k in want:
        if want[k].shape[0] == t["S"]:
            want[k][31] = w[k][31]
        else:
            want[k][31 * t["A"]:32 * t["A"]] = w[k][31 * t["A"]:32 * t["A"]]
    _compare(got, want, pick, t["A"])


def test_replay_elastic_vs_fixed_dop(tg, orc):
    """Scheduler ablation of the paper (its Fig. 7) on synthetic contended traces: the elastic policy against
    fixed DoP 4 and 16 (every elastic action restricted to that unit count).  Parity of the fixed-DoP replays
    with the oracle, and the qualitative shape: elastic gives the lower mean ACT."""
    t = gen.make_trace(S=8, A=2000, seed=7, cluster=(4, 32, 0, 0), type_probs=(1, 0, 0), rate_per_s=30.0,
                       horizon_s=2000 / 30.0, max_ticks=400000, pin_frac=0.0)
    mean = {}
    for name, tt in (("elastic", t), ("dop4", gen.with_fixed_dop(t, 4)), ("dop16", gen.with_fixed_dop(t, 16))):
        got = _replay_gpu(tg, tt)
        _compare(got, orc.replay(tt, 0, 3), range(3), t["A"])
        assert (got["n_started"] == t["A"]).all()
        mean[name] = float(got["mean_act_us"].mean())
    print({k: round(v / 1e6, 3) for k, v in mean.items()}, flush=True)
    assert mean["elastic"] < mean["dop4"] < mean["dop16"]


@pytest.mark.parametrize("seed", range(8))
def test_replay_several_quotas(tg, orc, seed):
    """Sec. 4.1 in the replay: API actions that take a token from several buckets when they start."""
    print("case replay quotas", seed, flush=True)
    n_api = (2, 3, 5, 16, 70)[seed % 5]                        # 70 quotas: the LDS node table of the admission
    t = gen.make_trace(S=3, A=300 + 80 * seed, seed=700 + seed, cluster=(1 + seed % 2, 16, seed % 2, n_api),
                       type_probs=(0.2, 0.1, 0.7), rate_per_s=float((100, 400, 1500)[seed % 3]), horizon_s=3.0, max_ticks=30000)
    t["depth"] = 1 + seed % 3
    gen.with_extra_quotas(t, frac=0.6, seed=seed, max_extra=1 + seed % 4)
    if seed % 2:
        _with_services(t, seed, n_services=5, slots=2)
    want = orc.replay(t)
    if seed % 3 == 2:                                          # the heavily loaded cases: the masks delay somebody
        assert (want["start_us"] != orc.replay(dict(t, act_quota_mask=None))["start_us"]).any()
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])


@pytest.mark.parametrize("name", [n for n in CASES if n not in ("single_action", "api_only")])
def test_replay_queue_prefix_small(tg, orc, name):
    """Every step admits one prefix of the whole waiting queue (Alg. 1 as printed)."""
    print("case", name, flush=True)
    t = dict(gen.make_trace(**CASES[name]), queue_prefix=1)
    want = orc.replay(t)
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])
    if name.startswith("contended"):
        assert (orc.replay(dict(t, queue_prefix=0))["start_us"] != want["start_us"]).any(), "the rule should bind here"


@pytest.mark.parametrize("seed", range(6))
def test_replay_queue_prefix_with_quotas_and_services(tg, orc, seed):
    t = gen.make_trace(S=3, A=500, seed=700 + seed, cluster=(2, 16, 2, 3), rate_per_s=120.0, horizon_s=4.0, max_ticks=30000,
                       pin_frac=(0.0, 0.3, 0.8)[seed % 3])
    t["depth"] = 1 + seed % 3
    if seed % 2:
        gen.with_extra_quotas(t, frac=0.5, seed=seed)
    if seed % 3:
        _with_services(t, seed, n_services=4, slots=2)
    t["queue_prefix"] = 1
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 500)


def test_replay_queue_prefix_config5_contended_sampled(tg, orc):
    """Workload 5's contended shape, 64 scenarios on the GPU, 3 of them against the oracle."""
    t = dict(gen.make_trace(S=64, A=10_000, seed=5, contended=True, max_ticks=200_000), queue_prefix=1)
    got = _replay_gpu(tg, t)
    sample = (0, 31, 63)
    want = orc.replay(t, 0, 1)
    _compare(got, want, (0,), 10_000)
    for s in sample[1:]:
        _compare(got, orc.replay(t, s, s + 1), (s,), 10_000)


def test_replay_quota_with_more_candidates_than_any_node_has_units(tg, orc):
    """A quota can admit far more actions in one step than a CPU or GPU node has units (its actions are never elastic, so
    the per-node tables of the scheduler, sized for the nodes' units, are not used for it): 300 API actions arrive
    together on a cluster whose only other node has 4 cores."""
    t = gen.make_trace(S=3, A=320, seed=71, cluster=(1, 4, 0, 1), type_probs=(0.06, 0, 0.94), rate_per_s=50.0, horizon_s=6.4,
                       max_ticks=20000, pin_frac=0.5)
    t["arrival_us"][:] = np.tile(np.sort(np.concatenate([np.zeros(300, np.int64), np.arange(20) * 150_000 + 7])), 3)
    api = t["node_type"] == gen.TYPE_API
    t["node_cap"][api] = 400
    t["quota_tok0_micro"][api] = 350_000_000
    want = orc.replay(t)
    first = want["start_us"].reshape(3, 320)
    assert ((first == 0).sum(axis=1) > 200).all(), "hundreds of candidates on the quota in the first step"
    _compare(_replay_gpu(tg, t), want, range(3), 320)


def test_replay_gpu_nodes_behind_64_other_nodes(tg, orc):
    """GPU nodes whose index in the scenario is above 64: their start loop and the clearing of the per-node list
    lengths run in different wavefronts of the workgroup."""
    t = gen.make_trace(S=3, A=900, seed=72, cluster=(70, 4, 6, 0), type_probs=(0.4, 0.6, 0), rate_per_s=150.0, horizon_s=6.0,
                       max_ticks=20000, pin_frac=0.3)
    M = t["M"]
    assert (np.flatnonzero(t["node_type"][:M] == gen.TYPE_GPU) >= 64).all()
    want = orc.replay(t)
    assert (want["start_us"] >= 0).all()
    _compare(_replay_gpu(tg, t), want, range(3), 900)


@pytest.mark.parametrize("seed", range(8))
def test_replay_second_resource(tg, orc, seed):
    """A second resource per node (memory next to cores) held from start to finish by every action that was free to
    choose its node: CPU and GPU nodes, with and without pins, services, further quotas and the whole-queue prefix."""
    print("case", seed, flush=True)
    t = gen.make_trace(S=3, A=450, seed=800 + seed, cluster=(2 + seed % 3, 16, 1 + seed % 2, 2), rate_per_s=110.0, horizon_s=4.0,
                       max_ticks=40000, pin_frac=(0.0, 0.3, 0.7)[seed % 3])
    t["depth"] = 1 + seed % 3
    plain = orc.replay(t)
    _with_aux(t, seed, scarce=True)
    if seed % 4 == 1:
        _with_services(t, seed, n_services=4, slots=2)
    if seed % 4 == 2:
        gen.with_extra_quotas(t, frac=0.5, seed=seed)
    t["queue_prefix"] = int(seed % 4 == 3)
    want = orc.replay(t)
    _compare(_replay_gpu(tg, t), want, range(3), 450)
    if seed % 4 == 0:
        assert (plain["start_us"] != want["start_us"]).any(), "the second resource should delay somebody"


def test_replay_second_resource_wide_pools(tg, orc):
    """More than 64 nodes of a kind: the admission with a second resource runs on the node table in LDS."""
    t = gen.make_trace(S=2, A=1200, seed=820, cluster=(90, 8, 3, 0), type_probs=(0.8, 0.2, 0), rate_per_s=400.0, horizon_s=3.0,
                       max_ticks=20000, pin_frac=0.2)
    rng = np.random.default_rng(3)
    t["act_aux"] = rng.integers(0, 40, t["S"] * t["A"]).astype(np.int32)
    t["node_aux"] = rng.integers(20, 60, t["S"] * t["M"]).astype(np.int32)
    _compare(_replay_gpu(tg, t), orc.replay(t), range(2), 1200)


def test_replay_longest_trace(tg, orc):
    """The most arrivals a scenario may have (131 072), 400 per second on the default cluster: 40 new actions per tick."""
    t = gen.make_trace(S=1, A=131072, seed=31, rate_per_s=400.0, horizon_s=131072 / 400.0, max_ticks=100000)
    want = orc.replay(t)
    assert want["n_started"][0] == 131072
    _compare(_replay_gpu(tg, t), want, (0,), 131072)


@pytest.mark.parametrize("seed", range(8))
def test_replay_core_sets(tg, orc, seed):
    """Named cores (NUMA domains of 4-64 cores, nodes of 16-256 cores): every CPU action keeps the cores its step gave
    it until it finishes; with pins, the second resource and the whole-queue prefix in the mix."""
    print("case", seed, flush=True)
    cap, numa = ((16, 4), (48, 8), (128, 16), (256, 64), (256, 4), (40, 16), (128, 32), (24, 8))[seed]
    t = gen.make_trace(S=3, A=500, seed=840 + seed, cluster=(2 + seed % 3, cap, 1, 1), rate_per_s=130.0, horizon_s=4.0,
                       max_ticks=40000, pin_frac=(0.0, 0.3)[seed % 2], type_probs=(0.8, 0.1, 0.1))
    t["numa_cores"] = numa
    if seed % 4 == 2:
        _with_aux(t, seed, scarce=True)
    t["queue_prefix"] = int(seed % 4 == 3)
    want = orc.replay(t)
    sets = want["core_set"].reshape(-1, 4)
    bits = np.array([sum(bin(int(w)).count("1") for w in row) for row in sets])
    cpu = (t["act_type"] == gen.TYPE_CPU) & (want["start_us"] >= 0)
    assert (bits[cpu] == want["units"][cpu]).all() and (bits[~cpu] == 0).all()
    _compare(_replay_gpu(tg, t), want, range(3), 500)


def test_replay_core_sets_many_cpu_nodes(tg, orc):
    """More CPU nodes than a wavefront has lanes: the nodes with starts are found 64 at a time."""
    t = gen.make_trace(S=2, A=1500, seed=860, cluster=(150, 16, 2, 0), type_probs=(0.9, 0.1, 0), rate_per_s=500.0, horizon_s=3.0,
                       max_ticks=20000, pin_frac=0.2)
    t["numa_cores"] = 8
    _compare(_replay_gpu(tg, t), orc.replay(t), range(2), 1500)


def test_replay_with_named_cores_needs_the_output_map(tg):
    t = gen.make_trace(S=1, A=20, seed=1, contended=True)
    t["numa_cores"] = 8
    T = tg.Trace(t)
    bufs = T.alloc()
    bufs["core_set"] = None
    with pytest.raises(tg.TgError):
        T.replay(bufs)
    T.free()


@pytest.mark.parametrize("name", ["contended_small", "contended_burst", "default_cluster", "cpu_only_tiny_cluster", "gpu_only", "api_only",
                                  "tick_limit", "single_action"])
@pytest.mark.parametrize("queue_prefix", [0, 1])
def test_replay_cost_order_small(tg, orc, name, queue_prefix):
    """Second visiting order in the replay (least estimated ACT first): sorted waiting lists, the arrivals of a tick merged in."""
    print("case cost order", name, queue_prefix, flush=True)
    t = dict(gen.make_trace(**CASES[name]), order_policy=1, queue_prefix=queue_prefix)
    want = orc.replay(t)
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])
    if name.startswith("contended") and not queue_prefix:
        assert (want["start_us"] != orc.replay(dict(t, order_policy=0))["start_us"]).any(), "the order should matter"


def test_replay_cost_order_bursts_and_ties(tg, orc):
    """Hundreds of arrivals in one tick (merged 64 at a time), everybody at time 0, and few distinct durations (equal keys:
    arrival order decides)."""
    t = gen.make_trace(S=3, A=900, seed=41, contended=True, rate_per_s=3000.0, horizon_s=0.3, max_ticks=60000)
    t["order_policy"] = 1
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 900)
    t["arrival_us"][:] = 0
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 900)
    t["act_t_ori_us"] = (1 + t["act_t_ori_us"] % 3) * 400_000
    t["arrival_us"] = np.tile(np.sort(np.random.default_rng(2).integers(0, 40, 900)) * 50_000, 3).astype(np.int64)
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 900)


@pytest.mark.parametrize("seed", range(6))
def test_replay_cost_order_with_every_other_option(tg, orc, seed):
    """Cost order next to further quotas, the second resource, named cores, the whole-queue prefix, depths 1-4, pins."""
    t = gen.make_trace(S=3, A=450, seed=900 + seed, cluster=(2 + seed % 3, 16, 1 + seed % 2, 3), rate_per_s=130.0, horizon_s=3.5,
                       max_ticks=40000, pin_frac=(0.0, 0.3, 0.8)[seed % 3])
    t["depth"] = 1 + seed % 4
    gen.with_extra_quotas(t, frac=0.5, seed=seed)
    if seed % 2:
        _with_aux(t, seed, scarce=bool(seed & 2))
    if seed % 3 == 0:
        t["numa_cores"] = 8
    t["queue_prefix"] = int(seed >= 3)
    t["order_policy"] = 1
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 450)


def test_replay_cost_order_config5_contended_sampled(tg, orc):
    S, A = 64, 10_000
    t = dict(gen.make_trace(S=S, A=A, seed=5, contended=True, max_ticks=200_000), order_policy=1)
    got = _replay_gpu(tg, t)
    pick = [0, 31, 63]
    want = orc.replay(t, 0, 1)
    for s in pick[1:]:
        w = orc.replay(t, s, s + 1)
        for k in want:
            per = want[k].shape[0] // S
            want[k][s * per:(s + 1) * per] = w[k][s * per:(s + 1) * per]
    _compare(got, want, pick, A)
    assert (got["n_started"] == A).all()


_pooled = gen.trace_with_pooled_gpus


@pytest.mark.parametrize("n_gpu", [1, 2, 3, 4, 5])
def test_replay_pooled_gpus(tg, orc, n_gpu):
    """The GPU nodes of a scenario scheduled as one pool of chunks in every tick (Sec. 5.3, Alg. 4): pooled placement, Alg. 4 on the
    summed chunk counts, real chunks handed out cluster-wide."""
    print("case pooled", n_gpu, flush=True)
    for seed, probs, rate in ((0, (0, 1, 0), 50.0 * n_gpu), (1, (0.4, 0.5, 0.1), 80.0 * n_gpu)):
        t = _pooled(gen.make_trace(S=3, A=500, seed=950 + 10 * n_gpu + seed, cluster=(2 * seed, 16, n_gpu, seed), type_probs=probs,
                                   rate_per_s=rate, horizon_s=4.0, max_ticks=100_000, pin_frac=0.3))
        t["depth"] = 1 + (n_gpu + seed) % 4
        want = orc.replay(t)
        _compare(_replay_gpu(tg, t), want, range(3), 500)
        if n_gpu > 1 and seed == 0:
            plain = orc.replay(dict(t, gpu_pooled=0))
            assert (plain["start_us"] != want["start_us"]).any() or (plain["node"] != want["node"]).any(), "pooling should matter"


@pytest.mark.parametrize("seed", range(4))
def test_replay_pooled_gpus_with_other_options(tg, orc, seed):
    """Pooled GPUs next to the whole-queue prefix, the cost order, named cores and further quotas."""
    t = _pooled(gen.make_trace(S=3, A=450, seed=980 + seed, cluster=(2, 16, 2 + seed, 3), rate_per_s=140.0, horizon_s=3.0,
                               max_ticks=60_000, pin_frac=0.4))
    gen.with_extra_quotas(t, frac=0.5, seed=seed)
    t["queue_prefix"] = seed % 2
    t["order_policy"] = int(seed >= 2)
    if seed % 2 == 0:
        t["numa_cores"] = 8
    _compare(_replay_gpu(tg, t), orc.replay(t), range(3), 450)


def test_replay_pooled_gpus_burst_on_five_nodes(tg, orc):
    """Thousands of GPU actions within half a second on a pool of 40 GPUs: up to 39 candidates on the one resource, Alg. 4 on
    hundreds of chunk states, queues of thousands."""
    t = _pooled(gen.make_trace(S=2, A=3000, seed=77, cluster=(0, 0, 5, 0), type_probs=(0, 1, 0), rate_per_s=5000.0, horizon_s=0.5,
                               max_ticks=400000))
    want = orc.replay(t)
    assert (want["n_started"] == 3000).all()
    _compare(_replay_gpu(tg, t), want, range(2), 3000)


def test_replay_cost_order_longest_trace(tg, orc):
    """The longest trace the builder takes (131 072 arrivals) in the second visiting order."""
    A = 131072
    t = gen.make_trace(S=1, A=A, seed=31, rate_per_s=400.0, horizon_s=A / 400.0, max_ticks=100000)
    t["order_policy"] = 1
    _compare(_replay_gpu(tg, t), orc.replay(t), [0], A)


@pytest.mark.parametrize("seed", range(10))
def test_replay_cache_per_gpu(tg, orc, seed):
    """Sec. 5.3 with a cache on every GPU: the block that caches the service comes first, the delay follows the GPUs
    an action gets.  Clusters of 1-3 GPU nodes, 2-64 services, 1-64 slots, with pins, the prefix rule, a second
    resource and further quotas."""
    print("case cache per gpu", seed, flush=True)
    t = gen.make_trace(S=3, A=500 + 100 * seed, seed=370 + seed, cluster=(1 + seed % 2, 16, 1 + seed % 3, seed % 2 * 3),
                       type_probs=(0.2, 0.7, 0.1) if seed % 2 else (0.3, 0.7, 0.0),
                       rate_per_s=(30.0, 60.0, 150.0)[seed % 3], horizon_s=12.0, max_ticks=80000, pin_frac=0.3)
    _with_services(t, seed, n_services=(2, 5, 9, 64)[seed % 4], slots=(1, 2, 3, 64)[(seed // 2) % 4])
    if seed % 4 == 1:
        t["queue_prefix"] = 1
    if seed % 4 == 2:
        _with_aux(t, seed, scarce=True)
    if seed % 4 == 3:
        gen.with_extra_quotas(t, frac=0.6, seed=seed)
    per_node = orc.replay(t)
    t["cache_per_gpu"] = 1
    want = orc.replay(t)
    assert (want["finish_us"] != per_node["finish_us"]).any()
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])


def test_replay_cache_per_gpu_many_gpu_nodes(tg, orc):
    t = gen.make_trace(S=2, A=1500, seed=381, cluster=(0, 0, 70, 0), type_probs=(0, 1, 0), rate_per_s=400.0, horizon_s=4.0,
                       max_ticks=80000, pin_frac=0.2)
    _with_services(t, 9, n_services=12, slots=2)
    t["cache_per_gpu"] = 1
    _compare(_replay_gpu(tg, t), orc.replay(t), range(t["S"]), t["A"])


def test_replay_cache_per_gpu_block_choice(tg, orc):
    """One node, hand-made arrivals: the chunk that caches the service before the lowest one, the level before the
    cache, the block inside a larger chunk, blocks of 2, 4 and 8 GPUs."""
    from test_oracle_replay_gpu_cache import _node_trace
    cases = [
        [(0, 1, 1000, -1), (1, 1, 5, 0), (2, 1, 1000, -1), (3, 1, 5, 1), (100, 1, 50, 1), (110, 1, 50, 0)],
        [(0, 4, 20, -1), (1, 1, 5, 0), (100, 1, 1000, -1), (101, 1, 5, 0)],
        [(0, 4, 20, -1), (1, 1, 5, 0), (100, 1, 50, 0), (101, 1, 50, 0), (200, 1, 50, 0), (201, 1, 50, 0), (202, 1, 50, 0)],
        [(0, 1, 5, 0), (100, 2, 5, 0), (200, 2, 5, 0), (300, 4, 5, 0), (400, 4, 5, 0), (500, 8, 5, 0), (600, 8, 5, 0), (700, 1, 5, 0)],
        [(0, 2, 50, 1), (1, 2, 50, 0), (2, 4, 50, 1), (100, 4, 5, 1), (101, 2, 5, 0), (102, 2, 5, 1), (103, 1, 5, 0)],
    ]
    for rows in cases:
        for slots in (1, 2):
            t = _node_trace(rows, [300_000, 700_000], slots)
            _compare(_replay_gpu(tg, t), orc.replay(t), range(1), len(rows))


@pytest.mark.parametrize("seed", range(12))
def test_replay_cost_order_with_services(tg, orc, seed):
    """The second visiting order next to the service cache: this tick's keys count the restore time unless a node the
    action may run on caches its service.  GPU-heavy clusters under load (queues of tens to hundreds), caches per node
    and per GPU, pins, the prefix rule, a second resource."""
    print("case cost order with services", seed, flush=True)
    t = gen.make_trace(S=3, A=500 + 100 * seed, seed=470 + seed, cluster=(1 + seed % 2, 16, 1 + seed % 3, seed % 2 * 2),
                       type_probs=(0.2, 0.7, 0.1) if seed % 2 else (0.3, 0.7, 0.0),
                       rate_per_s=(60.0, 150.0, 400.0)[seed % 3], horizon_s=(12.0, 6.0, 3.0)[seed % 3], max_ticks=80000,
                       pin_frac=(0.3, 0.0, 0.8)[(seed // 3) % 3])
    _with_services(t, seed, n_services=(2, 5, 9, 64)[seed % 4], slots=(1, 2, 3, 64)[(seed // 2) % 4])
    t["order_policy"] = 1
    t["cache_per_gpu"] = seed % 2
    if seed % 4 == 1:
        t["queue_prefix"] = 1
    if seed % 4 == 2:
        _with_aux(t, seed, scarce=True)
    want = orc.replay(t)
    fcfs = orc.replay(dict(t, order_policy=0))
    assert (want["start_us"] != fcfs["start_us"]).any()
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])


def test_replay_cost_order_with_services_one_machine(tg, orc):
    """Whole-node actions on one node: the machine whose set-up time follows its cache (the oracle's pin)."""
    from test_oracle_replay_order import _whole_node_trace
    for seed in range(6):
        rng = np.random.default_rng(900 + seed)
        A = 40
        T = rng.integers(1, 6, A).tolist()
        n_sv = int(rng.integers(2, 5))
        sv = rng.integers(-1, n_sv, A).tolist()
        restore = rng.integers(1, 9, n_sv).tolist()
        slots = int(rng.integers(1, 3))
        arr = sorted(rng.integers(0, 60 if seed % 2 else 1, A).tolist())
        for per_gpu in (0, 1):
            t = _whole_node_trace(T, sv, restore, slots, arr, per_gpu=per_gpu)
            _compare(_replay_gpu(tg, t), orc.replay(t), range(1), A)


def test_replay_cost_order_with_services_long_queue(tg, orc):
    """A burst that leaves more than a thousand GPU actions waiting: the ordering pass runs over many blocks of 64."""
    t = gen.make_trace(S=2, A=3000, seed=483, cluster=(0, 0, 2, 0), type_probs=(0, 1, 0), rate_per_s=3000.0, horizon_s=1.0,
                       max_ticks=400000, pin_frac=0.2)
    _with_services(t, 11, n_services=7, slots=2)
    t["order_policy"] = 1
    want = orc.replay(t)
    _compare(_replay_gpu(tg, t), want, range(t["S"]), t["A"])
