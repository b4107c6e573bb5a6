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
    for k in ("node", "units", "act_us", "defer_reason", "node_used", "task_sum_us", "node_obj"):
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
