"""Pins of the oracle's core-set choice (Sec. 5.2: the manager names the cores of an action and
prefers cores of one NUMA domain) against exhaustive search, hand-worked cases and invariants."""
import itertools

import numpy as np
import pytest

import gen
from oracle import orc


def _domains(free, numa):
    return [free[d * numa:(d + 1) * numa] for d in range((len(free) + numa - 1) // numa)]


def _fewest_domains(free, numa, k):
    """Smallest number of domains whose free cores add up to k, by exhaustive search over subsets."""
    cnt = [int(np.sum(d)) for d in _domains(free, numa)]
    for r in range(1, len(cnt) + 1):
        for sub in itertools.combinations(range(len(cnt)), r):
            if sum(cnt[d] for d in sub) >= k:
                return r
    return None


def test_hand_worked_sequence():
    # two domains of 8, all free: requests 4, 4, 8 -> the second 4 completes domain 0 (fewest free cores that fit)
    free = np.ones(16, np.uint8)
    got, free = orc.take_cores(free, 8, 4)
    assert got == [0, 1, 2, 3]
    got, free = orc.take_cores(free, 8, 4)
    assert got == [4, 5, 6, 7]
    got, free = orc.take_cores(free, 8, 8)
    assert got == list(range(8, 16)) and free.sum() == 0


def test_best_fit_prefers_the_fuller_domain_and_lowest_on_ties():
    free = np.array([1, 1, 1, 0, 0, 0, 0, 0,  1, 1, 1, 1, 1, 1, 0, 0,  0, 1, 0, 1, 0, 1, 0, 0,  1] * 1, np.uint8)
    got, after = orc.take_cores(free, 8, 3)           # domains hold 3, 6, 3, 1: both 3s fit exactly, the lower one wins
    assert got == [0, 1, 2]
    got, after = orc.take_cores(after, 8, 2)          # 0, 6, 3, 1 -> domain 2 (3 free) over domain 1 (6 free)
    assert got == [17, 19]
    got, after = orc.take_cores(after, 8, 1)          # 0, 6, 1, 1 -> domain 2 before domain 3
    assert got == [21]


def test_spill_takes_the_largest_domains_first():
    free = np.array([1, 1, 0, 0, 1, 1, 1, 1,  1, 1, 1, 0, 0, 0, 0, 0], np.uint8)   # 6 and 3 free
    got, after = orc.take_cores(free, 8, 7)
    assert got == [0, 1, 4, 5, 6, 7, 8] and list(np.flatnonzero(after)) == [9, 10]


def test_spill_takes_the_lower_of_two_equally_free_domains_first():
    free = np.ones(8, np.uint8)                       # two domains of 4, all free; 6 cores do not fit in one
    got, after = orc.take_cores(free, 4, 6)
    assert got == [0, 1, 2, 3, 4, 5] and list(np.flatnonzero(after)) == [6, 7]
    free = np.array([0, 1, 1, 1,  1, 1, 1, 0,  1, 1, 1, 1], np.uint8)   # 3, 3 and 4 free: the 4 first, then the lower 3
    got, after = orc.take_cores(free, 4, 6)
    assert got == [1, 2, 8, 9, 10, 11] and list(np.flatnonzero(after)) == [3, 4, 5, 6]


@pytest.mark.parametrize("seed", range(40))
def test_single_allocation_against_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    numa = int(rng.choice([4, 8, 16]))
    cap = int(rng.integers(numa, 6 * numa + 1))
    free = (rng.random(cap) < rng.choice([0.3, 0.6, 0.9])).astype(np.uint8)
    if free.sum() == 0:
        free[rng.integers(cap)] = 1
    k = int(rng.integers(1, free.sum() + 1))
    got, after = orc.take_cores(free, numa, k)
    assert len(got) == k and len(set(got)) == k
    assert all(free[c] for c in got)
    assert (after == free - np.isin(np.arange(cap), got)).all()
    spanned = sorted({c // numa for c in got})
    assert len(spanned) == _fewest_domains(free, numa, k)
    cnt = [int(np.sum(d)) for d in _domains(free, numa)]
    if len(spanned) == 1:
        d = spanned[0]
        fitting = [x for x in range(len(cnt)) if cnt[x] >= k]
        assert cnt[d] == min(cnt[x] for x in fitting) and d == min(x for x in fitting if cnt[x] == cnt[d])
        assert got == [c for c in range(d * numa, min(cap, (d + 1) * numa)) if free[c]][:k]   # lowest ids first
    else:
        # every spanned domain but the last one taken is emptied
        left = [int(np.sum(x)) for x in _domains(after, numa)]
        assert sum(1 for d in spanned if left[d] > 0) <= 1


@pytest.mark.parametrize("seed", range(6))
def test_core_sets_of_a_step(seed):
    """In a whole step: a selected CPU action gets exactly `units` cores that were free on its node, no core
    is given twice, nothing else gets cores, and node choice, units and ACT do not depend on the core maps."""
    p = gen.make_random_problem(3100 + seed, B=2, N=120 + 40 * seed, n_cpu=3, n_gpu=1, n_api=1, cpu_cap_hi=(24, 64, 200)[seed % 3],
                                busy=seed % 2 == 0, pin_frac=0.3)
    base = orc.assign(p)
    numa = (4, 8, 16, 32, 64)[seed % 5]
    gen.with_core_maps(p, numa, seed)
    out = orc.assign(p)
    for k in ("node", "units", "act_us", "reason"):
        assert (base[k] == out[k]).all()
    sets = out["core_set"].reshape(-1, 4)
    maps = p["node_core_free"].reshape(-1, 4)
    N, M = p["N"], p["M"]
    used = np.zeros_like(maps)
    n_sets = 0
    for g in range(p["B"] * N):
        b = g // N
        bits = sum(bin(int(w)).count("1") for w in sets[g])
        if out["units"][g] > 0 and p["act_type"][g] == gen.TYPE_CPU:
            j = b * M + out["node"][g]
            assert bits == out["units"][g]
            assert all(int(sets[g][w]) & ~int(maps[j][w]) == 0 for w in range(4))
            assert all(int(sets[g][w]) & int(used[j][w]) == 0 for w in range(4))
            used[j] |= sets[g]
            n_sets += 1
        else:
            assert bits == 0
    assert n_sets > 0


def test_one_domain_whenever_the_node_allows_it():
    """Roomy nodes with wide domains: every action's cores lie in one domain."""
    p = gen.make_random_problem(3200, B=1, N=60, n_cpu=4, n_gpu=0, n_api=0, cpu_cap_hi=256, busy=False, pin_frac=0.0)
    c = p["node_type"] == gen.TYPE_CPU
    p["node_cap"][c] = 256
    p["node_free"][c] = 256
    gen.with_core_maps(p, 64, 1)
    out = orc.assign(p)
    sets = out["core_set"].reshape(-1, 4)
    sel = np.flatnonzero(out["units"] > 0)
    assert len(sel) > 10
    for g in sel:
        assert sum(1 for w in range(4) if sets[g][w]) == 1
