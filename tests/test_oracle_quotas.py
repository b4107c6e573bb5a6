"""Pins for actions that draw on several quotas at once (Sec. 4.1: a DeepSearch action may query several
websites, each with its own quota, and each is one component of its cost vector): a hand-worked case,
the admission loop re-run by the independent Python simulator, and token conservation."""
import numpy as np
import pytest

import gen
from test_oracle_vector import _place


def _api_problem(n_api, tokens, pins, extras, t_us=1000):
    """One snapshot of API quotas only; action i is pinned to quota pins[i] and also names the quotas in extras[i]."""
    n = len(pins)
    p = gen.make_random_problem(1, B=1, N=n, n_cpu=0, n_gpu=0, n_api=n_api, shuffle_nodes=False, busy=False, bad_frac=0.0)
    assert (p["node_type"] == gen.TYPE_API).all() and p["M"] == n_api
    p["node_cap"][:] = 1000
    p["node_free"][:] = tokens
    p["node_backlog_us"][:] = 0
    p["act_type"][:] = gen.TYPE_API
    p["act_model"][:] = 0
    p["act_kmask"][:] = 1
    p["act_t_ori_us"][:] = t_us
    p["act_pin_node"][:] = pins
    p["act_quota_mask"] = np.array([sum(1 << r for r in e) for e in extras], np.uint64)
    return p


def test_hand_worked_case(orc):
    # tokens: quota 0 has 3, quota 1 has 1, quota 2 has 2
    pins = [0, 0, 0, 2, 1, 2]
    extras = [[1], [1], [], [], [], [0]]
    p = _api_problem(3, [3, 1, 2], pins, extras)
    o = orc.assign(p)
    # a0 takes (0,1): left 2,0,2.  a1 needs quota 1: none left -> does not fit, closes the queue of quota 0.
    # a2 waits behind a1.  a3 takes quota 2: left 2,0,1.  a4 is pinned to quota 1: empty -> closes quota 1.
    # a5 takes (2,0): left 1,0,0.
    assert list(o["reason"]) == [0, 1, 1, 0, 1, 0]
    assert list(o["node"]) == [0, -1, -1, 2, -1, 2]
    assert list(o["node_used"]) == [2, 1, 2]                  # tokens taken, further quotas included
    assert int(o["summary"]["units_used"][0][gen.TYPE_API]) == 5
    assert int(o["summary"]["n_assigned"][0]) == 3


def test_only_the_first_64_quotas_can_be_named(orc):
    """70 quotas: a mask has 64 bits, so quotas of rank 64 and above can be pinned to but not named.  Quota 64 is
    empty; an action pinned to quota 1 that names quota 0 does not care, one pinned to quota 64 waits."""
    tokens = [2] * 70
    tokens[0], tokens[64] = 3, 0
    p = _api_problem(70, tokens, pins=[1, 64, 69, 1], extras=[[0], [], [0, 63], [0]])
    o = orc.assign(p)
    assert list(o["reason"]) == [0, 1, 0, 0]
    assert o["node_used"][0] == 3 and o["node_used"][1] == 2 and o["node_used"][63] == 1 and o["node_used"][69] == 1
    assert o["node_used"][64] == 0


def test_no_extras_is_the_plain_problem(orc):
    p = gen.make_random_problem(40, B=2, N=120, n_cpu=1, n_gpu=1, n_api=4)
    a = orc.assign(p)
    p["act_quota_mask"] = np.zeros(p["B"] * p["N"], np.uint64)
    b = orc.assign(p)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


@pytest.mark.parametrize("seed", range(12))
def test_admission_loop_rerun_in_python(orc, seed):
    p = gen.make_random_problem(500 + seed, B=3, N=150 + 20 * seed, n_cpu=1 + seed % 2, n_gpu=0, n_api=2 + seed % 5,
                                busy=False, pin_frac=0.3, type_probs=(0.3, 0.0, 0.7))
    p["type_k"][gen.TYPE_GPU] = 0
    gen.with_extra_quotas(p, frac=0.6, seed=seed)
    assert p["act_quota_mask"].any()
    o = orc.assign(p)
    N = p["N"]
    for b in range(p["B"]):
        home, reason = _place(p, b)
        np.testing.assert_array_equal(o["home"][b * N:(b + 1) * N], home, err_msg=f"snapshot {b} home")
        got = o["reason"][b * N:(b + 1) * N]
        np.testing.assert_array_equal(got == 3, reason == 3)
        np.testing.assert_array_equal(got == 1, reason == 1)
    q = dict(p); q["act_quota_mask"] = None
    assert (orc.assign(q)["reason"] != o["reason"]).any(), "further quotas should defer some actions"


@pytest.mark.parametrize("seed", range(8))
def test_tokens_are_conserved(orc, seed):
    p = gen.make_random_problem(540 + seed, B=3, N=300, n_cpu=2, n_gpu=1, n_api=3 + seed % 4, type_probs=(0.3, 0.2, 0.5))
    gen.with_extra_quotas(p, frac=0.7, seed=seed)
    o = orc.assign(p)
    N, M = p["N"], p["M"]
    for b in range(p["B"]):
        api = [j for j in range(M) if p["node_type"][b * M + j] == gen.TYPE_API]
        taken = np.zeros(M, np.int64)
        for i in range(N):
            g = b * N + i
            if o["units"][g] > 0:
                taken[o["node"][g]] += o["units"][g]
                for r, j in enumerate(api):
                    if int(p["act_quota_mask"][g]) >> r & 1:
                        taken[j] += 1
        np.testing.assert_array_equal(o["node_used"][b * M:(b + 1) * M], taken)
        assert (taken <= p["node_free"][b * M:(b + 1) * M]).all()
        used = o["summary"]["units_used"][b]
        assert int(used[gen.TYPE_API]) == int(taken[api].sum())
