"""Pins for the oracle's trace replay: closed forms for an uncontended cluster, a single
non-elastic unit (Lindley recursion on tick-quantised starts) and a token bucket, plus
conservation checks on contended traces."""
import numpy as np
import pytest

import gen
import pyref


def _dur(t, g, k):
    K = t["K"]
    q = [int(x) for x in t["k_list"]].index(k)
    sp = int(t["speedup_q16"][int(t["act_param"][g]) * K + q]) if t["act_model"][g] == 2 else 0
    return pyref.duration(int(t["act_model"][g]), int(t["act_t_ori_us"][g]), int(t["act_param"][g]), k, sp)


def _kmax(t, g, cap):
    ty = int(t["act_type"][g])
    ks = [int(t["k_list"][q]) for q in range(int(t["type_k"][ty])) if t["act_kmask"][g] >> q & 1]
    if t["act_model"][g] == 0:
        ks = ks[:1]
    return max(k for k in ks if k <= cap)


def _stats(t, o, s):
    A = t["A"]
    sl = slice(s * A, (s + 1) * A)
    st = o["start_us"][sl] >= 0
    acts = np.sort((o["finish_us"][sl] - t["arrival_us"][sl])[st])
    n = int(st.sum())
    assert o["n_started"][s] == n
    if n:
        assert abs(o["mean_act"][s] - acts.mean()) <= 1e-9 * acts.mean()
        assert o["p99_act"][s] == acts[int(np.ceil(0.99 * n)) - 1]     # nearest rank


def test_uncontended_closed_form(orc):
    t = gen.make_trace(S=2, A=300, seed=11, cluster=(2, 100_000, 0, 4), pin_frac=0.0, rate_per_s=20.0, horizon_s=30.0)
    t["node_cap"][t["node_type"] == gen.TYPE_API] = 10**6            # quotas never bind
    t["quota_tok0_micro"][t["node_type"] == gen.TYPE_API] = 10**12
    o = orc.replay(t)
    tick = t["tick_us"]
    for s in range(2):
        for i in range(t["A"]):
            gidx = s * t["A"] + i
            arr = int(t["arrival_us"][gidx])
            start = -(-arr // tick) * tick                           # next tick at or after arrival
            k = _kmax(t, gidx, 100_000)
            assert o["start_us"][gidx] == start
            assert o["units"][gidx] == k                              # room for everyone: largest allowed option
            assert o["finish_us"][gidx] == start + _dur(t, gidx, k)
        _stats(t, o, s)
        last = int(o["start_us"][s * t["A"]:(s + 1) * t["A"]].max())
        assert o["n_ticks"][s] == last // tick + 1                   # the replay ends with the tick of the last start


def test_uncontended_gpu_one_at_a_time(orc):
    t = gen.make_trace(S=1, A=40, seed=14, cluster=(0, 0, 2, 0), type_probs=(0, 1, 0), pin_frac=0.0)
    t["arrival_us"][:] = np.arange(40) * 5_000_000 + 17               # far apart: the node is empty again
    t["act_t_ori_us"][:] = np.minimum(t["act_t_ori_us"], 4_000_000)
    o = orc.replay(t)
    for i in range(40):
        k = _kmax(t, i, 8)
        assert o["start_us"][i] == -(-int(t["arrival_us"][i]) // t["tick_us"]) * t["tick_us"]
        assert o["units"][i] == k and o["node"][i] == 0
        assert o["finish_us"][i] == o["start_us"][i] + _dur(t, i, k)


def test_single_unit_lindley(orc):
    t = gen.make_trace(S=3, A=60, seed=12, cluster=(1, 1, 0, 0), rate_per_s=2.0, horizon_s=40.0,
                       cpu_median=400_000, max_ticks=100000)
    t["act_model"][:] = 0
    t["act_kmask"][:] = 1
    o = orc.replay(t)
    tick = t["tick_us"]
    for s in range(3):
        prev_fin = 0
        for i in range(t["A"]):
            g = s * t["A"] + i
            ready = max(int(t["arrival_us"][g]), prev_fin)
            start = -(-ready // tick) * tick
            assert o["start_us"][g] == start and o["units"][g] == 1
            prev_fin = start + int(t["act_t_ori_us"][g])
            assert o["finish_us"][g] == prev_fin
        _stats(t, o, s)


def test_token_bucket(orc):
    A = 400
    t = gen.make_trace(S=2, A=A, seed=13, cluster=(0, 0, 0, 1), type_probs=(0, 0, 1), max_ticks=5000)
    t["arrival_us"][:] = 0                                           # everything queued at time zero
    o = orc.replay(t)
    tick = t["tick_us"]
    for s in range(2):
        rate, burst, tok0 = int(t["quota_rate"][s]), int(t["node_cap"][s]), int(t["quota_tok0_micro"][s])
        assert rate * tick < burst * 10**6                            # bucket never saturates while drained each tick
        starts = o["start_us"][s * A:(s + 1) * A]
        assert (np.diff(starts) >= 0).all()                           # FCFS
        for n in range(0, 200, 7):
            total = min(A, (tok0 + n * rate * tick) // 10**6)
            assert int((starts <= n * tick).sum()) == total
        _stats(t, o, s)


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_contended_conservation(orc, seed):
    t = gen.make_trace(S=2, A=400, seed=seed, contended=True, rate_per_s=80.0, horizon_s=5.0, max_ticks=20000)
    o = orc.replay(t)
    S, A, M = t["S"], t["A"], t["M"]
    for s in range(S):
        sl = slice(s * A, (s + 1) * A)
        st, fin, un, nd = o["start_us"][sl], o["finish_us"][sl], o["units"][sl], o["node"][sl]
        assert (st >= 0).all()                                        # everything eventually runs
        assert (st % t["tick_us"] == 0).all() and (st >= t["arrival_us"][sl]).all()
        for i in range(A):
            assert fin[i] == st[i] + _dur(t, s * A + i, int(un[i]))
        for j in range(M):
            n = s * M + j
            ty = int(t["node_type"][n])
            mine = np.flatnonzero(nd == j)
            assert (t["act_type"][sl][mine] == ty).all()
            if ty == gen.TYPE_API:
                continue
            ev = sorted([(int(st[i]), 1, int(un[i])) for i in mine] + [(int(fin[i]), 0, -int(un[i])) for i in mine])
            use = 0
            for _, _, d in ev:                                        # releases sort before starts at equal times
                use += d
                assert 0 <= use <= t["node_cap"][n]
            if ty == gen.TYPE_GPU:                                    # chunk-feasible on real addresses
                b = pyref.Buddy(0xFF)
                where = {}
                for tm, is_start, d in ev:
                    pass
                order = sorted([(int(st[i]), 1, i) for i in mine] + [(int(fin[i]), 0, i) for i in mine])
                for tm, is_start, i in order:
                    if is_start:
                        where[i] = b.alloc(int(un[i]))
                        assert where[i] is not None
                    else:
                        b.free(where[i], int(un[i]))
        _stats(t, o, s)


def test_tick_limit_ends_the_replay(orc):
    """A single core and ten-second actions arriving together: one start per 100 ticks; with `max_ticks` = 250 the replay
    stops after exactly that many ticks with three actions started (ticks 0, 100, 200), the others never start."""
    t = gen.make_trace(S=1, A=6, seed=15, cluster=(1, 1, 0, 0), type_probs=(1, 0, 0), pin_frac=0.0, max_ticks=250)
    t["arrival_us"][:] = 0
    t["act_model"][:] = 0
    t["act_kmask"][:] = 1
    t["act_t_ori_us"][:] = 10_000_000
    o = orc.replay(t)
    assert list(o["start_us"]) == [0, 10_000_000, 20_000_000, -1, -1, -1]
    assert o["n_started"][0] == 3 and o["n_ticks"][0] == 250
    o = orc.replay(dict(t, max_ticks=10_000))
    assert list(o["start_us"]) == [i * 10_000_000 for i in range(6)]
    assert o["n_ticks"][0] == 501                                    # ticks 0..500


@pytest.mark.parametrize("seed", range(6))
def test_every_tick_is_one_step_on_the_snapshot_rebuilt_from_the_replays_own_times(orc, seed):
    """The tick loop around the step: at every tick the cluster state (free cores, release time of every core in use,
    whole tokens, who waits) is rebuilt here from the start / finish times, units and nodes the replay reported, and one
    scheduling step on that snapshot (pinned on its own elsewhere) must select exactly the actions the replay started at
    that tick, on the same nodes with the same units.  CPU nodes and quotas (GPU nodes would need their addresses)."""
    A = 260
    t = gen.make_trace(S=1, A=A, seed=120 + seed, cluster=(2 + seed % 2, 8 + 4 * (seed % 3), 0, 2), type_probs=(0.8, 0, 0.2),
                       rate_per_s=70.0, horizon_s=A / 70.0, max_ticks=50_000, pin_frac=(0.0, 0.3)[seed % 2], cpu_median=700_000)
    t["depth"] = 1 + seed % 3
    api = np.flatnonzero(t["node_type"] == gen.TYPE_API)
    t["quota_rate"][api] = 3 + seed
    with_aux = seed >= 3                                         # a second resource held from start to finish by unpinned actions
    if with_aux:
        rng = np.random.default_rng(seed)
        t["act_aux"] = rng.integers(0, 30, A).astype(np.int32)
        t["node_aux"] = rng.integers(40, 100, t["M"]).astype(np.int32)
    _, evicted_somewhere = check_every_tick_is_one_step(orc, t, with_aux)
    if seed % 3:
        assert evicted_somewhere


def check_every_tick_is_one_step(orc, t, with_aux=False):
    """Body of the pin above, for CPU nodes and quotas; the trace's visiting order (``order_policy``) is the step's."""
    A = t["A"]
    api = np.flatnonzero(t["node_type"] == gen.TYPE_API)
    o = orc.replay(t)
    M, tick = t["M"], int(t["tick_us"])
    start, fin, units, node = o["start_us"], o["finish_us"], o["units"], o["node"]
    arr = t["arrival_us"]
    assert (start >= 0).all()
    tok = t["quota_tok0_micro"].astype(np.int64).copy()
    evicted_somewhere = waited_somewhere = False
    for n in range(int(o["n_ticks"][0])):
        now = n * tick
        if n > 0:
            tok[api] = np.minimum(t["node_cap"][api].astype(np.int64) * 10**6, tok[api] + t["quota_rate"][api].astype(np.int64) * tick)
        waiting = np.flatnonzero((arr <= now) & (start >= now))
        if len(waiting):
            running = np.flatnonzero((start < now) & (fin > now) & (t["act_type"] == gen.TYPE_CPU))
            free = t["node_cap"].astype(np.int32).copy()
            busy = [[] for _ in range(M)]
            for i in running:
                free[node[i]] -= units[i]
                busy[node[i]] += [int(fin[i]) - now] * int(units[i])
            free[api] = (tok[api] // 10**6).astype(np.int32)
            extra = {}
            if with_aux:
                left = t["node_aux"].astype(np.int64).copy()
                for i in running:
                    if t["act_pin_node"][i] < 0:
                        left[node[i]] -= t["act_aux"][i]
                extra = dict(node_aux_free=left.astype(np.int32), act_aux=t["act_aux"][waiting])
            p = dict(B=1, N=len(waiting), M=M, K=t["K"], n_classes=t["n_classes"], n_tasks=1, depth=t["depth"],
                     order_policy=int(t.get("order_policy", 0)),
                     k_list=t["k_list"], type_k=t["type_k"], speedup_q16=t["speedup_q16"],
                     node_type=t["node_type"], node_cap=t["node_cap"], node_free=free, node_backlog_us=np.zeros(M, np.int64),
                     node_chunks=None, node_busy_off=np.concatenate([[0], np.cumsum([len(b) for b in busy])]).astype(np.int32),
                     node_busy_rel_us=np.array([x for b in busy for x in b] or [0], np.int64),
                     act_age_us=(now - arr[waiting]).astype(np.int64), act_task=None, **extra,
                     **{k: t[k][waiting] for k in ("act_type", "act_model", "act_t_ori_us", "act_kmask", "act_param", "act_pin_node")})
            s = orc.assign(p)
            go = start[waiting] == now
            np.testing.assert_array_equal(s["reason"] == 0, go, err_msg=f"tick {n}")
            np.testing.assert_array_equal(s["node"][go], node[waiting][go], err_msg=f"tick {n}")
            np.testing.assert_array_equal(s["units"][go], units[waiting][go], err_msg=f"tick {n}")
            np.testing.assert_array_equal(s["act_us"][go], (fin - arr)[waiting][go], err_msg=f"tick {n}")
            evicted_somewhere |= bool((s["reason"] == 2).any())
            waited_somewhere |= bool((s["reason"] == 1).any())
        for i in np.flatnonzero((start == now) & (t["act_type"] == gen.TYPE_API)):
            tok[node[i]] -= 10**6
    assert waited_somewhere
    return o, evicted_somewhere
