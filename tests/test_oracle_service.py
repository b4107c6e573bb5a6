"""Pins for the oracle's service residency (Sec. 5.3, evict on execution): an action whose
service is not cached on a node is delayed there by the service's restore time.  Closed forms,
equivalences with the service-free problem, the score tensor against its definition, and the
admission loop / the cost order re-run independently with the delay."""
import numpy as np
import pytest

import gen
import pyref
from test_oracle_order import _keys, _relabel
from test_oracle_vector import _place

INF = pyref.INF


def _with_services(p, seed, n_services=6, resident_frac=0.5):
    rng = np.random.default_rng(seed + 900)
    n, m = p["B"] * p["N"], p["B"] * p["M"]
    p["act_service"] = rng.integers(-1, n_services, n).astype(np.int32)
    bits = rng.random((m, n_services)) < resident_frac
    p["node_resident"] = (bits * (1 << np.arange(n_services, dtype=np.uint64))).sum(axis=1).astype(np.uint64)
    p["restore_us"] = (rng.integers(1, 9, n_services) * 250_000).astype(np.int64)
    return p


def test_one_action_goes_where_it_finishes_first(orc):
    """Two nodes: the service is cached on the busier one.  The action goes there exactly when
    its backlog is smaller than the restore time elsewhere (ties: smaller index)."""
    p = gen.subset_problem(gen.make_config(1), 0, 1, n_cpu_nodes=2, cap=8)
    p["act_model"][:] = 0
    p["act_pin_node"][:] = -1
    T = int(p["act_t_ori_us"][0])
    p["act_service"] = np.array([2], np.int32)
    p["node_resident"] = np.array([0, 1 << 2], np.uint64)
    p["restore_us"] = np.array([5, 5, 300_000, 5], np.int64)
    for backlog1, node in ((0, 1), (299_999, 1), (300_000, 0), (900_000, 0)):
        p["node_backlog_us"][:] = [0, backlog1]
        o = orc.assign(p)
        assert o["node"][0] == node
        assert o["act_us"][0] == int(p["act_age_us"][0]) + T + (backlog1 if node == 1 else 300_000)


@pytest.mark.parametrize("seed", range(6))
def test_everything_resident_changes_nothing(orc, seed):
    p = gen.make_random_problem(500 + seed, B=2, N=120, n_cpu=3, n_gpu=2, n_api=1, cpu_cap_hi=40)
    base = orc.assign(p)
    base_cost = orc.score(p)
    _with_services(p, seed)
    p["node_resident"][:] = np.uint64((1 << 6) - 1)
    o = orc.assign(p)
    for k in ("node", "units", "act_us", "reason", "node_obj"):
        np.testing.assert_array_equal(o[k], base[k], err_msg=k)
    np.testing.assert_array_equal(orc.score(p), base_cost)
    p["act_service"][:] = -1                                   # nobody calls a service: nothing resident matters
    p["node_resident"][:] = 0
    np.testing.assert_array_equal(orc.assign(p)["act_us"], base["act_us"])


def test_nothing_resident_delays_every_nonelastic_action_by_its_restore_time(orc):
    N = 10
    p = gen.subset_problem(gen.make_config(1), 0, N, n_cpu_nodes=1, cap=32)
    p["act_model"][:] = 0
    base = orc.assign(p)
    assert (base["reason"] == 0).all()
    p["act_service"] = (np.arange(N) % 3).astype(np.int32)
    p["node_resident"] = np.zeros(1, np.uint64)
    p["restore_us"] = np.array([111, 2222, 33333], np.int64)
    o = orc.assign(p)
    np.testing.assert_array_equal(o["act_us"], base["act_us"] + p["restore_us"][p["act_service"]])
    np.testing.assert_array_equal(o["units"], base["units"])


@pytest.mark.parametrize("seed", range(4))
def test_score_tensor_adds_the_delay_where_the_service_is_not_resident(orc, seed):
    p = gen.make_random_problem(520 + seed, B=2, N=40, n_cpu=2, n_gpu=2, n_api=1)
    base = orc.score(p)
    _with_services(p, seed)
    got = orc.score(p)
    # walk the tensor in its layout: snapshot, kind, actions of the kind (FCFS), nodes of the kind, options
    w = 0
    N, M = p["N"], p["M"]
    for b in range(p["B"]):
        for t in range(3):
            acts = [i for i in range(N) if p["act_type"][b * N + i] == t]
            nodes = [j for j in range(M) if p["node_type"][b * M + j] == t]
            for i in acts:
                s = int(p["act_service"][b * N + i])
                for j in nodes:
                    extra = 0 if s < 0 or int(p["node_resident"][b * M + j]) >> s & 1 else int(p["restore_us"][s])
                    for q in range(int(p["type_k"][t])):
                        assert got[w] == (INF if base[w] == INF else base[w] + extra)
                        w += 1
    assert w == len(got)


@pytest.mark.parametrize("seed", range(10))
def test_admission_loop_rerun_in_python_with_services(orc, seed):
    p = gen.make_random_problem(540 + seed, B=3, N=80 + 10 * seed, n_cpu=2 + seed % 4, n_gpu=0, n_api=seed % 3,
                                busy=False, cpu_cap_hi=16 + 8 * (seed % 3), pin_frac=0.3)
    p["type_k"][gen.TYPE_GPU] = 0
    p["act_kmask"][p["act_type"] == gen.TYPE_CPU] |= 1
    p["node_free"][:] = p["node_cap"]                          # roomy nodes: many admissions, many node choices
    base = orc.assign(p)
    _with_services(p, seed, resident_frac=0.4)
    o = orc.assign(p)
    N = p["N"]
    for b in range(p["B"]):
        home, reason = _place(p, b)
        np.testing.assert_array_equal(o["home"][b * N:(b + 1) * N], home, err_msg=f"snapshot {b} home")
        np.testing.assert_array_equal(o["reason"][b * N:(b + 1) * N] == 1, reason == 1)
    if (base["home"] >= 0).sum() > 20 and p["M"] > 2:
        assert (o["home"] != base["home"]).any(), "the delays should move somebody"


@pytest.mark.parametrize("seed", range(6))
def test_cost_order_with_services_is_fcfs_on_the_relabelled_problem(orc, seed):
    p = _with_services(gen.make_random_problem(560 + seed, B=2, N=90, n_cpu=3, n_gpu=2, n_api=1, cpu_cap_hi=30), seed)
    key = _keys(p)
    N = p["N"]
    perm = [sorted(range(N), key=lambda i, b=b: (key[b * N + i], i)) for b in range(p["B"])]
    q, idx = _relabel(p, perm)
    want = orc.assign(q)
    got = orc.assign(dict(p, order_policy=1))
    for k in ("node", "units", "act_us", "reason"):
        np.testing.assert_array_equal(got[k][idx], want[k], err_msg=k)
