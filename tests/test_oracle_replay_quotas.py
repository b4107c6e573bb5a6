"""Pins for API actions that draw on several quotas in the trace replay (Sec. 4.1, Sec. 5.1): two buckets
drained together against an independent integer simulation, masks that cannot bind, and the token levels
re-derived from the oracle's own start times."""
import numpy as np
import pytest

import gen


def _api_trace(S, A, n_api, seed):
    t = gen.make_trace(S=S, A=A, seed=seed, cluster=(0, 0, 0, n_api), type_probs=(0, 0, 1), max_ticks=20000)
    assert (t["node_type"] == gen.TYPE_API).all()
    return t


@pytest.mark.parametrize("seed", range(4))
def test_two_buckets_drained_together(orc, seed):
    """Everything queued at time zero, every action pinned to quota 0 and also naming quota 1: per tick as many
    start as both buckets hold whole tokens."""
    A = 300
    t = _api_trace(2, A, 2, 40 + seed)
    t["arrival_us"][:] = 0
    t["act_pin_node"][:] = 0
    t["act_quota_mask"] = np.full(2 * A, 2, np.uint64)
    o = orc.replay(t)
    tick = int(t["tick_us"])
    for s in range(2):
        cap = [int(t["node_cap"][s * 2 + j]) * 10**6 for j in range(2)]
        rate = [int(t["quota_rate"][s * 2 + j]) for j in range(2)]
        tok = [int(t["quota_tok0_micro"][s * 2 + j]) for j in range(2)]
        starts = o["start_us"][s * A:(s + 1) * A]
        done, n = 0, 0
        while done < A and n < 20000:
            if n > 0:
                tok = [min(cap[j], tok[j] + rate[j] * tick) for j in range(2)]
            go = min(tok[0] // 10**6, tok[1] // 10**6, A - done)
            assert (starts[done:done + go] == n * tick).all(), (s, n)
            tok = [x - go * 10**6 for x in tok]
            done += go
            n += 1
        assert done == A or (starts[done:] == -1).all()


def test_masks_that_cannot_bind(orc):
    t = gen.make_trace(S=3, A=400, seed=50, cluster=(2, 16, 1, 4), rate_per_s=300.0, horizon_s=3.0, max_ticks=4000)
    base = orc.replay(t)
    zero = orc.replay(dict(t, act_quota_mask=np.zeros(3 * 400, np.uint64)))
    for k in base:
        np.testing.assert_array_equal(base[k], zero[k], err_msg=k)
    # quota of rank 3 never runs dry and nobody is pinned to it: naming it changes nothing
    M = t["M"]
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in t.items()}
    for s in range(3):
        api = np.flatnonzero(q["node_type"][s * M:(s + 1) * M] == gen.TYPE_API) + s * M
        rich = api[3]
        pinned = (q["act_pin_node"][s * 400:(s + 1) * 400] == rich - s * M)
        q["act_pin_node"][s * 400:(s + 1) * 400][pinned] = api[0] - s * M
        q["node_cap"][rich] = 10**6
        q["quota_tok0_micro"][rich] = 10**12
    base = orc.replay(q)
    mask = np.where((q["act_type"] == gen.TYPE_API), np.uint64(8), np.uint64(0)).astype(np.uint64)
    named = orc.replay(dict(q, act_quota_mask=mask))
    for k in base:
        np.testing.assert_array_equal(base[k], named[k], err_msg=k)


@pytest.mark.parametrize("seed", range(6))
def test_token_levels_from_the_oracles_own_starts(orc, seed):
    """Buckets re-run in Python from the start times the oracle reports: every start finds a whole token in the
    action's own quota and in every quota it names, and binding masks delay somebody."""
    S, A = 3, 500
    t = gen.make_trace(S=S, A=A, seed=60 + seed, cluster=(1, 16, 0, 2 + seed % 4), type_probs=(0.2, 0.0, 0.8),
                       rate_per_s=400.0, horizon_s=2.0, max_ticks=20000)
    gen.with_extra_quotas(t, frac=0.7, seed=seed)
    assert t["act_quota_mask"].any()
    o = orc.replay(t)
    plain = orc.replay(dict(t, act_quota_mask=None))
    assert (o["start_us"] != plain["start_us"]).any()
    M, tick = t["M"], int(t["tick_us"])
    for s in range(S):
        api = [j for j in range(M) if t["node_type"][s * M + j] == gen.TYPE_API]
        cap = {j: int(t["node_cap"][s * M + j]) * 10**6 for j in api}
        rate = {j: int(t["quota_rate"][s * M + j]) for j in api}
        tok = {j: int(t["quota_tok0_micro"][s * M + j]) for j in api}
        starts = o["start_us"][s * A:(s + 1) * A]
        by_tick = {}
        for i in np.flatnonzero(starts >= 0):
            if t["act_type"][s * A + i] == gen.TYPE_API:
                by_tick.setdefault(int(starts[i]) // tick, []).append(int(i))
        last = max(by_tick) if by_tick else 0
        for n in range(last + 1):
            if n > 0:
                tok = {j: min(cap[j], tok[j] + rate[j] * tick) for j in api}
            for i in by_tick.get(n, []):
                g = s * A + i
                need = [int(t["act_pin_node"][g])] + [api[r] for r in range(len(api)) if int(t["act_quota_mask"][g]) >> r & 1]
                for j in need:
                    tok[j] -= 10**6
            assert all(v >= 0 for v in tok.values()), (s, n)


def test_a_quota_beyond_rank_63_is_never_named(orc):
    """66 quotas: a mask names ranks 0-63 only, so the bucket of rank 64 is drawn on by its own actions alone - their
    start times do not depend on what the actions of other quotas name (bit 0 of a mask must not reach rank 64)."""
    A, n_api = 400, 66
    t = _api_trace(1, A, n_api, 77)
    t["arrival_us"][:] = 0
    rng = np.random.default_rng(5)
    pin = rng.integers(0, n_api, A).astype(np.int32)
    pin[::3] = 64                                                   # a third of the actions belong to the quota of rank 64
    t["act_pin_node"] = pin
    t["node_cap"][:] = 3; t["quota_tok0_micro"][:] = 2_000_000; t["quota_rate"][:] = 4   # scarce tokens everywhere
    plain = orc.replay(t)
    mask = np.where(pin == 64, 0, 1).astype(np.uint64)             # everybody else also names rank 0 ...
    mask[pin == 0] = 2                                              # ... (its own actions name rank 1 instead)
    t["act_quota_mask"] = mask
    named = orc.replay(t)
    own = pin == 64
    np.testing.assert_array_equal(named["start_us"][own], plain["start_us"][own])
    assert (named["start_us"][~own] != plain["start_us"][~own]).any()     # the masks do bind for the others
    # and the bucket of rank 64 follows its closed form: 2 tokens at first, 4 micro-tokens x tick per tick after
    tick = int(t["tick_us"])
    tok, done, n, starts = 2_000_000, 0, 0, named["start_us"][own]
    while done < own.sum() and n < 20000:
        if n > 0:
            tok = min(3_000_000, tok + 4 * tick)
        go = min(tok // 10**6, int(own.sum()) - done)
        assert (starts[done:done + go] == n * tick).all(), n
        tok -= go * 10**6
        done += go
        n += 1
