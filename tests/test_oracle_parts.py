"""Pins for the oracle's building blocks: durations (Eq. 1), the score tensor (Eq. 2),
DPArrange with both operators (Alg. 3, Alg. 4), the heap estimate (Alg. 2) and the chunk model
(Sec. 5.3).  Each pin is a closed form, an exhaustive enumeration or an independent second
algorithm from tests/pyref.py, never the oracle's own formula retyped."""
import itertools

import numpy as np
import pytest

import gen
import pyref

INF = pyref.INF


# ---------------------------------------------------------------- Eq. 1 durations
def test_duration_closed_forms(orc):
    rng = np.random.default_rng(0)
    for _ in range(300):
        T = int(rng.integers(1, 1 << 36))
        k = int(rng.choice([1, 2, 3, 4, 8, 16, 32, 64]))
        p = int(rng.integers(0, 10**6 + 1))
        assert orc.duration(1, T, p, 1) == T                       # one unit: T_ori itself
        assert orc.duration(1, T, 0, k) == T                       # nothing parallel
        assert orc.duration(1, T, 10**6, k) == -(-T // k)          # perfectly parallel: ceil(T/k)
        assert orc.duration(2, T, 0, k, 65536 * k) == -(-T // k)   # table with E = 1
        assert orc.duration(2, T, 0, k, 65536) == T                # table with E k = 1
        assert orc.duration(0, T, p, k) == T                       # elasticity unknown
        assert orc.duration(1, T, p, k) == pyref.duration(1, T, p, k)
        sp = int(rng.integers(65536, 65536 * k + 1))
        assert orc.duration(2, T, 0, k, sp) == pyref.duration(2, T, 0, k, sp)


def test_duration_extremes_and_monotone(orc):
    T = (1 << 36) - 1
    for p in (0, 1, 499_999, 999_999, 10**6):
        prev = None
        for k in (1, 2, 4, 8, 16, 32, 64):
            d = orc.duration(1, T, p, k)
            assert d == pyref.duration(1, T, p, k)
            assert prev is None or d <= prev                        # more units never slower
            assert d >= -(-T // k)                                  # E(k) <= 1
            prev = d
    assert orc.duration(1, 1, 10**6, 64) == 1                       # never below one microsecond
    assert orc.duration(2, 1, 0, 64, 65536 * 64) == 1


# ---------------------------------------------------------------- Eq. 2 score tensor
def _py_score(p):
    """Direct loops over the layout [b][type][action][node][q] with exact rational durations."""
    B, N, M, K = p["B"], p["N"], p["M"], p["K"]
    out = []
    for b in range(B):
        for t in range(3):
            for i in range(N):
                g = b * N + i
                if p["act_type"][g] != t:
                    continue
                allowed = [q for q in range(int(p["type_k"][t])) if p["act_kmask"][g] >> q & 1]
                if p["act_model"][g] == 0:
                    allowed = allowed[:1]
                for j in range(M):
                    n = b * M + j
                    if p["node_type"][n] != t:
                        continue
                    for q in range(int(p["type_k"][t])):
                        k = int(p["k_list"][q])
                        ok = q in allowed and k <= p["node_cap"][n] and p["act_pin_node"][g] in (-1, j)
                        if p["act_pin_node"][g] < -1:
                            ok = q in allowed and k <= p["node_cap"][n]
                        if not ok:
                            out.append(INF)
                            continue
                        sp = int(p["speedup_q16"][int(p["act_param"][g]) * K + q]) if p["act_model"][g] == 2 else 0
                        d = pyref.duration(int(p["act_model"][g]), int(p["act_t_ori_us"][g]), int(p["act_param"][g]), k, sp)
                        out.append(int(p["node_backlog_us"][n]) + d)
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_score_matches_direct_loops(orc, seed):
    p = gen.make_random_problem(seed, B=2, N=30)
    got = orc.score(p)
    assert got.shape[0] == orc.num_candidates(p)
    np.testing.assert_array_equal(got, _py_score(p))


def test_score_config1_and_monotone_in_backlog(orc):
    p = gen.make_config(1)
    c0 = orc.score(p)
    assert c0.shape == (64 * 4 * 4,)
    np.testing.assert_array_equal(c0, _py_score(p))
    q = dict(p)
    q["node_backlog_us"] = p["node_backlog_us"] + np.array([0, 7, 0, 123456], np.int64)
    c1 = orc.score(q).reshape(64, 4, 4)
    d = c1 - c0.reshape(64, 4, 4)
    assert (d[:, 0] == 0).all() and (d[:, 1] == 7).all() and (d[:, 3] == 123456).all()  # ACT monotone in load


# ---------------------------------------------------------------- Alg. 3 basic operator
def _rand_durs(rng, m, k_list, convex=False, full=False):
    K = len(k_list)
    dur = np.full((m, K), INF, np.int64)
    opts = []
    for i in range(m):
        T = int(rng.integers(1, 50)) * 1000
        p = int(rng.integers(0, 11)) * 100_000
        mask = (1 << K) - 1 if full else int(rng.integers(1, 1 << K))
        o = []
        for q, k in enumerate(k_list):
            if mask >> q & 1:
                dur[i, q] = pyref.duration(1, T, p, k)
                o.append((k, int(dur[i, q])))
        opts.append(o)
    return dur, opts


@pytest.mark.parametrize("seed", range(12))
def test_dp_units_is_optimal(orc, seed):
    rng = np.random.default_rng(seed)
    k_list = [1, 2, 4, 8] if seed % 2 else [1, 2, 3, 5, 7]
    m = int(rng.integers(1, 7))
    dur, opts = _rand_durs(rng, m, k_list)
    lo = sum(o[0][0] for o in opts)
    U = int(rng.integers(lo, lo + 12))
    v, ks = orc.dp_units(dur, k_list, U)
    assert v == pyref.best_units_exhaustive(opts, U)
    assert ks.sum() <= U
    assert sum(dict(opts[i])[int(ks[i])] for i in range(m)) == v      # returned units realise the value


def test_dp_units_singletons_and_infeasible(orc):
    k_list = [1, 2, 4, 8]
    dur = np.full((3, 4), INF, np.int64)
    dur[0, 1], dur[1, 0], dur[2, 2] = 700, 50, 9
    v, ks = orc.dp_units(dur, k_list, 7)
    assert v == 759 and list(ks) == [2, 1, 4]                         # all sets singleton: plain sum
    v, _ = orc.dp_units(dur, k_list, 6)
    assert v == INF                                                   # minimum demands exceed U
    # sparse sets, U not exactly fillable (S={1,2,4,8}, m=2, U=7): best over used <= U
    dur = np.array([[80, 40, 20, 10], [80, 40, 20, 10]], np.int64)
    v, ks = orc.dp_units(dur, k_list, 7)
    assert v == 60 and sorted(ks) == [2, 4]


def test_dp_units_ties_prefer_fewer_units(orc):
    k_list = [1, 2, 4]
    dur = np.array([[10, 10, 10], [10, 10, 5]], np.int64)
    v, ks = orc.dp_units(dur, k_list, 8)
    assert v == 15 and list(ks) == [1, 4]
    # three units for two tasks that take 10 on one unit and 7 on two: [2,1] and [1,2] both total 17 on all three
    # units; the strict comparison with the options in ascending order keeps the smaller option of the later task
    dur = np.array([[10, 7, pyref.INF], [10, 7, pyref.INF]], np.int64)
    v, ks = orc.dp_units(dur, k_list, 3)
    assert v == 17 and list(ks) == [2, 1]


@pytest.mark.parametrize("seed", range(6))
def test_dp_units_equals_marginal_gain_greedy_when_convex(orc, seed):
    """With S = {1..kmax} and convex non-increasing durations, separable convex allocation is
    solved by handing units one at a time to the largest marginal gain (a textbook result)."""
    rng = np.random.default_rng(100 + seed)
    kmax, m = 6, int(rng.integers(2, 7))
    k_list = list(range(1, kmax + 1))
    T = rng.integers(1000, 100_000, m)
    dur = np.array([[-(-int(T[i]) // k) for k in k_list] for i in range(m)], np.int64)
    # enforce convexity of the integer sequences (ceil can break it by one unit)
    for i in range(m):
        for _ in range(kmax):
            for q in range(1, kmax - 1):
                if dur[i, q - 1] - dur[i, q] < dur[i, q] - dur[i, q + 1]:
                    dur[i, q] = (dur[i, q - 1] + dur[i, q + 1]) // 2
    U = int(rng.integers(m, m * kmax))
    units = [1] * m
    for _ in range(U - m):
        gains = [(dur[i, units[i] - 1] - dur[i, units[i]]) if units[i] < kmax else -1 for i in range(m)]
        i = int(np.argmax(gains))
        if gains[i] <= 0:
            break
        units[i] += 1
    greedy = sum(int(dur[i, units[i] - 1]) for i in range(m))
    v, _ = orc.dp_units(dur, k_list, U)
    assert v == greedy


# ---------------------------------------------------------------- Alg. 4 chunk operator, Sec. 5.3
def test_chunk_encode_decode_roundtrip(orc):
    for bound in [(1, 1, 1, 1), (4, 2, 1, 1), (8, 4, 2, 1), (3, 1, 2, 5)]:
        size = np.prod([b + 1 for b in bound])
        seen = set()
        for j in range(int(size)):
            e, c = orc.chunk_roundtrip(bound, j)
            assert e == j and all(0 <= c[x] <= bound[x] for x in range(4))
            seen.add(c)
        assert len(seen) == size                                       # collision free


def test_chunk_counts_follow_address_level_buddy(orc):
    rng = np.random.default_rng(5)
    for _ in range(300):
        mask = int(rng.integers(0, 256))
        b = pyref.Buddy(mask)
        assert orc.mask_chunks(mask) == b.counts()
        counts = list(b.counts())
        m2 = mask
        for _ in range(int(rng.integers(1, 6))):
            k = int(rng.choice([1, 2, 4, 8]))
            s_ref = b.alloc(k)
            ok, c_new = orc.chunk_take(counts, k)
            s, m2 = orc.mask_alloc(m2, k)
            assert ok == (s_ref is not None)
            if ok:
                counts = list(c_new)
                assert s == s_ref and m2 == b.mask
            else:
                assert s == -1
            assert tuple(counts) == b.counts()                          # counts model == real addresses


def test_fresh_node_power_of_two_requests_fit_iff_sum_le_8(orc):
    for reqs in itertools.product([1, 2, 4, 8], repeat=4):
        c = (0, 0, 0, 1)
        ok_all = True
        for k in reqs:
            ok, c = orc.chunk_take(c, k)
            if not ok:
                ok_all = False
                break
        prefix_ok = all(sum(reqs[: n + 1]) <= 8 for n in range(4))
        assert ok_all == prefix_ok                                      # buddy lemma


@pytest.mark.parametrize("seed", range(10))
def test_dp_chunks_is_optimal(orc, seed):
    rng = np.random.default_rng(200 + seed)
    k_list = [1, 2, 4, 8]
    mask = 0xFF if seed < 3 else int(rng.integers(1, 256))
    chunks = pyref.Buddy(mask).counts()
    free = bin(mask).count("1")
    m = int(rng.integers(1, min(free, 5) + 1))
    while True:
        dur, opts = _rand_durs(rng, m, k_list)
        want = pyref.best_chunks_exhaustive(opts, mask)
        if want is not None:
            break
    v, ks = orc.dp_chunks(dur, k_list, chunks)
    assert v == want
    b = pyref.Buddy(mask)
    assert all(b.alloc(int(k)) is not None for k in ks)                  # served in order on real addresses
    assert sum(dict(opts[i])[int(ks[i])] for i in range(m)) == v


def test_dp_chunks_tie_rules(orc):
    """Equal totals: the end state with the smallest code (fewest large chunks left) wins, and on the way to a
    state the smaller source state, then the smaller option.  Hand-worked on tiny cases."""
    INF = pyref.INF
    k_list = [1, 2, 4, 8]
    # one action, every option costs 5, one free chunk of 8: the end states are (1,1,1,0), (0,1,1,0), (0,0,1,0)
    # and (0,0,0,0); the last has the smallest code, so the action gets all 8 GPUs
    v, ks = orc.dp_chunks(np.array([[5, 5, 5, 5]], np.int64), k_list, (0, 0, 0, 1))
    assert (v, list(ks)) == (5, [8])
    # a free chunk of 2 and one of 4, two actions that may take 2 or 4 GPUs at 10 each: [2,4] and [4,2] both end
    # in the empty state (code 0, the smallest; [2,2] leaves a chunk of 2).  Bounds (1,1,1,1): after [2] the state is
    # (0,0,1,0) = code 4, after [4] it is (0,1,0,0) = code 2 - the smaller source state wins: [4,2]
    dur = np.array([[INF, 10, 10, INF], [INF, 10, 10, INF]], np.int64)
    v, ks = orc.dp_chunks(dur, k_list, (0, 1, 1, 0))
    assert (v, list(ks)) == (20, [4, 2])
    # same source state, two options with the same total and the same end state cannot happen (an option fixes the
    # end state), so the option only decides between end states: cheaper total first, then the smaller code
    v, ks = orc.dp_chunks(np.array([[7, 5, 5, 9]], np.int64), k_list, (0, 0, 0, 1))
    assert (v, list(ks)) == (5, [4])


# ---------------------------------------------------------------- Alg. 2 estimate
def test_estimate_single_machine_sum_of_completion_times(orc):
    T = [5, 3, 9, 1, 7]
    dur = np.array([[t] for t in T], np.int64)
    want = int(np.cumsum(T).sum()) + 10 * len(T)                         # textbook sum C_j, machine free at 10
    assert orc.estimate([10], dur, [1], 2) == want


def test_estimate_uncontended_and_empty(orc):
    k_list = [1, 2]
    dur = np.array([[7, INF], [4, INF], [9, INF]], np.int64)
    assert orc.estimate([100] * 3, dur, k_list, 1) == 3 * 100 + 20       # everyone starts at once
    assert orc.estimate([100] * 3, np.zeros((0, 2), np.int64), k_list, 2) == 0
    assert orc.estimate([1, 2], np.array([[INF, INF]], np.int64), k_list, 2) == 0   # can never run: left out
    # second option of the first action is explored: 2 units, starts when the second frees
    dur = np.array([[100, 10]], np.int64)
    assert orc.estimate([0, 50], dur, k_list, 1) == 100
    assert orc.estimate([0, 50], dur, k_list, 2) == 60


@pytest.mark.parametrize("seed", range(20))
def test_estimate_matches_heapq_and_depth_monotone(orc, seed):
    rng = np.random.default_rng(300 + seed)
    k_list = [1, 2, 4, 8]
    H = int(rng.integers(1, 12))
    heap = rng.integers(0, 1000, H)
    n = int(rng.integers(0, 9))
    dur, opts = _rand_durs(rng, n, k_list) if n else (np.zeros((0, 4), np.int64), [])
    prev = None
    for depth in (1, 2, 3):
        got = orc.estimate(heap, dur, k_list, depth)
        assert got == pyref.estimate([int(x) for x in heap], opts, depth)
        assert prev is None or got <= prev                                # more choices never hurt
        prev = got
