"""GPU parity at the full size of the two largest workloads, in the launch configuration bench.py times.

Workload 3 (B=1024 snapshots x N=4096 actions, 3.34 G candidates, a 26.7 GB tensor whose byte offsets
pass 2^32 and whose entry offsets pass 2^31): the whole score tensor, snapshot by snapshot, and the
assignment of every fourth snapshot, against the oracle run on the same snapshots.  Workload 5
(S=4096 scenarios x 10 000 arrivals): one launch per cluster, scenarios spread over the whole grid
re-run by the oracle, conservation properties on all of them.

The oracle is called on independent slices from a few host threads (ctypes releases the GIL, the
oracle keeps no state between calls); what it computes per slice is unchanged.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

THREADS = 12


@pytest.fixture(scope="module")
def tg():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_13019_amd import tg as _tg
    _tg.load()
    return _tg


@pytest.fixture(scope="module")
def config3():
    return gen.make_config(3)


def _snapshot_offsets(p):
    """First entry of every snapshot in the score tensor, from the counts of actions and nodes per kind
    (a block per kind: its actions x its nodes x its options)."""
    B, N, M = p["B"], p["N"], p["M"]
    at, nt = p["act_type"].reshape(B, N), p["node_type"].reshape(B, M)
    per = np.zeros(B, np.int64)
    for t in range(3):
        per += (at == t).sum(1).astype(np.int64) * (nt == t).sum(1) * int(p["type_k"][t])
    return np.concatenate([[0], np.cumsum(per)])


def test_score_config3_every_snapshot(tg, orc, config3):
    import torch
    p = config3
    P = tg.Problem(p)
    n = P.num_candidates
    assert n == 3_340_606_896 and n > 2**31 and 8 * n > 2**34
    out = torch.empty(n + 2, dtype=torch.int64, device="cuda")
    out[n:] = -7
    P.score(out)
    torch.cuda.synchronize()
    P.free()
    assert (out[n:].cpu().numpy() == -7).all()                    # nothing written past the tensor
    off = _snapshot_offsets(p)
    assert off[-1] == n
    # snapshots whose block straddles the 2^29-th entry (byte offset 2^32) and the 2^31-st entry are among them
    assert any(off[b] < 2**29 < off[b + 1] for b in range(p["B"])) and any(off[b] < 2**31 < off[b + 1] for b in range(p["B"]))
    group = 32
    with ThreadPoolExecutor(THREADS) as pool:
        for b0 in range(0, p["B"], group):
            bs = range(b0, min(b0 + group, p["B"]))
            want = pool.map(lambda b: orc.score(gen.slice_problem(p, [b])), bs)
            got = out[off[b0]:off[bs[-1] + 1]].cpu().numpy()
            for b, w in zip(bs, want):
                np.testing.assert_array_equal(got[off[b] - off[b0]:off[b + 1] - off[b0]], w, err_msg=f"snapshot {b}")
            if b0 % 256 == 0:
                print("score parity through snapshot", bs[-1], flush=True)


def test_assign_config3_every_fourth_snapshot(tg, orc, config3):
    from test_gpu_assign import _assign_gpu, _compare
    p = config3
    got = _assign_gpu(tg, p)
    pick = sorted(set(range(0, 1024, 4)) | {1, 2, 3, 1021, 1022, 1023})
    with ThreadPoolExecutor(THREADS) as pool:
        wants = list(pool.map(lambda b: orc.assign(gen.slice_problem(p, [b])), pick))
    N, M, T = p["N"], p["M"], p["n_tasks"]
    for b, want in zip(pick, wants):
        sub = {k: got[k][b * per:(b + 1) * per] for k, per in (("defer_reason", N), ("node", N), ("units", N), ("act_us", N),
                                                               ("node_used", M), ("task_sum_us", T), ("node_obj", M), ("summary", 1))}
        _compare(sub, want, f"snapshot {b}")
    # properties over all snapshots: capacity never exceeded, counts add up, selected actions carry their units
    used = got["node_used"].reshape(p["B"], M)
    assert (used <= p["node_free"].reshape(p["B"], M)).all()
    s = got["summary"]
    assert ((s["n_selected"] + s["n_prefix"] + s["n_evicted"] + s["n_infeasible"]) == N).all()
    sel = got["defer_reason"] == 0
    assert ((got["units"] > 0) == sel).all() and ((got["node"] >= 0) == sel).all() and ((got["act_us"] >= 0) == sel).all()
    assert (np.bincount(np.flatnonzero(sel) // N, minlength=p["B"]) == s["n_selected"]).all()


@pytest.mark.parametrize("contended", [False, True])
def test_replay_config5_full(tg, orc, contended):
    """One launch over all 4096 scenarios (the workgroups of the launch take them in rounds); the oracle
    replays scenarios from the first, the middle and the last rounds."""
    from test_gpu_replay import _compare, _replay_gpu
    S, A = 4096, 10_000
    t = gen.make_trace(S=S, A=A, seed=4 + int(contended), contended=contended, max_ticks=200_000 if contended else 8000)
    print("trace made", flush=True)
    got = _replay_gpu(tg, t)
    print("replayed", flush=True)
    pick = [0, 1, 511, 512, 1023, 2047, 2048, 3000, 3583, 3584, 4094, 4095]
    with ThreadPoolExecutor(THREADS) as pool:
        parts = list(pool.map(lambda s: orc.replay(t, s, s + 1), pick))
    want = parts[0]
    for s, w in zip(pick[1:], parts[1:]):
        for k in want:
            per = want[k].shape[0] // S
            want[k][s * per:(s + 1) * per] = w[k][s * per:(s + 1) * per]
    _compare(got, want, pick, A)
    # every scenario: each action starts at most once, on a tick at or after its arrival, and runs for a positive time
    started = got["start_us"] >= 0
    assert (got["n_started"] == started.reshape(S, A).sum(1)).all()
    assert (got["n_started"] == A).all()                                      # both clusters drain within the tick limit
    assert (got["start_us"] >= t["arrival_us"]).all() and (got["start_us"] % t["tick_us"] == 0).all()
    assert (got["finish_us"] > got["start_us"]).all() and (got["units"] >= 1).all()
    nt = t["node_type"].reshape(S, t["M"])
    node = got["node"].reshape(S, A)
    assert (np.take_along_axis(nt, node, 1) == t["act_type"].reshape(S, A)).all()   # every action on a node of its kind
    # cores in use never exceed a CPU node's capacity: checked at every start instant of 64 scenarios spread over the launch
    for s in range(0, S, 64):
        sl = slice(s * A, (s + 1) * A)
        st, fi, un, no = got["start_us"][sl], got["finish_us"][sl], got["units"][sl], got["node"][sl]
        cpu = t["act_type"][sl] == gen.TYPE_CPU
        for j in np.unique(no[cpu]):
            m = cpu & (no == j)
            rel = -(-fi[m] // t["tick_us"]) * t["tick_us"]                    # units come back at the first tick at or after the finish
            ev = np.concatenate([st[m], rel])
            dl = np.concatenate([un[m], -un[m]]).astype(np.int64)
            order = np.lexsort((dl, ev))                                      # releases before starts at the same instant
            assert np.cumsum(dl[order]).max() <= t["node_cap"][s * t["M"] + j]
