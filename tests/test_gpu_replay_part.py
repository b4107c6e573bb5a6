"""tg_replay_trace_part: a replay cut into pieces gives, after every piece, the oracle's replay with the tick limit set
to the tick reached, and at the end the result of tg_replay_trace in one go - bit for bit (mean ACT within 1e-9)."""
import numpy as np
import pytest

import gen
from test_gpu_replay import _compare, _replay_gpu, tg  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _pieces(tg, orc, t, cuts, check_every=1):
    """Replays ``t`` in pieces of ``cuts`` ticks (the last one repeated to the trace's limit); compares with the
    oracle after every ``check_every``-th piece and at the end."""
    import torch
    T = tg.Trace(t)
    bufs = T.alloc()
    for k in ("start_us", "finish_us", "units", "node", "p99_act_us", "n_started", "n_ticks", "core_set"):
        if k in bufs:
            bufs[k].fill_(-5)
    limit, reached, i = int(t["max_ticks"]), 0, 0
    while reached < limit:
        n = cuts[min(i, len(cuts) - 1)]
        T.replay_part(bufs, restart=(i == 0), n_ticks=n)
        reached = min(limit, reached + n)
        i += 1
        if i % check_every == 0 or reached == limit:
            torch.cuda.synchronize()
            got = {k: v.cpu().numpy() for k, v in bufs.items() if k != "ws"}
            part = dict(t, max_ticks=reached)
            _compare(got, orc.replay(part), range(t["S"]), t["A"])
    T.free()
    return got, i


@pytest.mark.parametrize("seed", range(700, 724))
def test_replay_in_pieces_random_traces(tg, orc, seed):
    """Random clusters, loads and options (pins, depth, quotas, services, prefix rule, cost order, pooled GPUs)."""
    print("case pieces", seed, flush=True)
    t = gen.random_trace(seed)
    rng = np.random.default_rng(seed)
    span = max(int(t["max_ticks"]), 8)
    cuts = [int(c) for c in rng.integers(1, max(span // 6, 2), size=5)] + [max(span // 3, 1)]
    got, n = _pieces(tg, orc, t, cuts)
    assert n >= 3
    whole = _replay_gpu(tg, t)
    for k in got:
        np.testing.assert_array_equal(got[k], whole[k], err_msg=k)


@pytest.mark.parametrize("opts", [dict(), dict(queue_prefix=1), dict(order_policy=1), dict(order_policy=1, queue_prefix=1)])
def test_replay_in_pieces_contended(tg, orc, opts):
    """A contended cluster under bursts, cut at single ticks first: every waiting list, the running set and (in the
    cost order) the side of the sorted lists' two buffers carry over."""
    print("case pieces contended", opts, flush=True)
    t = gen.make_trace(S=4, A=900, seed=41, contended=True, rate_per_s=300.0, horizon_s=3.0, max_ticks=30000)
    t.update(opts)
    got, _ = _pieces(tg, orc, t, [1, 1, 2, 3, 17, 100, 1000, 4000], check_every=2)
    whole = _replay_gpu(tg, t)
    for k in got:
        np.testing.assert_array_equal(got[k], whole[k], err_msg=k)


def test_replay_in_pieces_restart_starts_over(tg, orc):
    """restart on buffers that hold an earlier, unfinished run: the same result as on fresh ones."""
    import torch
    t = gen.make_trace(S=3, A=600, seed=42, contended=True, rate_per_s=200.0, horizon_s=3.0, max_ticks=30000)
    T = tg.Trace(t)
    bufs = T.alloc()
    T.replay_part(bufs, restart=True, n_ticks=37)
    T.replay_part(bufs, restart=False, n_ticks=5)
    T.replay_part(bufs, restart=True, n_ticks=int(t["max_ticks"]))
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in bufs.items() if k != "ws"}
    T.free()
    _compare(got, orc.replay(t), range(3), 600)


def test_replay_in_pieces_rejects_no_ticks(tg):
    t = gen.make_trace(S=1, A=10, seed=43, contended=True)
    T = tg.Trace(t)
    bufs = T.alloc()
    for n in (0, -3):
        with pytest.raises(tg.TgError) as e:
            T.replay_part(bufs, restart=True, n_ticks=n)
        assert e.value.code == tg.E_INVALID_ARG
    T.free()


def test_replay_in_pieces_refuses_a_workspace_without_a_run(tg):
    """Going on from a workspace that no call has written: every scenario reports -1 ticks, nothing else is written."""
    import torch
    t = gen.make_trace(S=3, A=50, seed=44, contended=True)
    T = tg.Trace(t)
    bufs = T.alloc()
    bufs["ws"].zero_()
    for k in ("start_us", "n_started", "n_ticks"):
        bufs[k].fill_(-5)
    T.replay_part(bufs, restart=False, n_ticks=10)
    torch.cuda.synchronize()
    assert (bufs["n_ticks"].cpu().numpy() == -1).all()
    assert (bufs["start_us"].cpu().numpy() == -5).all() and (bufs["n_started"].cpu().numpy() == -5).all()
    T.free()
