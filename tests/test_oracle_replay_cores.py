"""Pins for named cores in the trace replay (Sec. 5.2: the CPU manager names the cores of every action and prefers one
NUMA domain): every CPU action keeps the cores its step gave it until it finishes.  Sets of the right size that never
overlap in time, the whole bookkeeping re-run from the oracle's own start and finish times with the single-allocation
rule (pinned on its own in test_oracle_cores.py), and no influence on the schedule."""
import numpy as np
import pytest

import gen


def _bits(words):
    return [64 * w + b for w in range(4) for b in range(64) if int(words[w]) >> b & 1]


@pytest.mark.parametrize("seed", range(6))
def test_core_sets_over_time(orc, seed):
    A, numa = 350, (4, 8, 16)[seed % 3]
    t = gen.make_trace(S=2, A=A, seed=160 + seed, cluster=(2 + seed % 2, (16, 48, 128)[seed % 3], 1, 1), rate_per_s=90.0,
                       horizon_s=4.0, max_ticks=50_000, pin_frac=(0.0, 0.4)[seed % 2])
    plain = orc.replay(t)
    t["numa_cores"] = numa
    o = orc.replay(t)
    for k in plain:
        np.testing.assert_array_equal(plain[k], o[k], err_msg=k)         # naming cores changes nothing else
    M, tick = t["M"], int(t["tick_us"])
    sets = o["core_set"].reshape(2 * A, 4)
    spread = 0
    for s in range(2):
        sl = slice(s * A, (s + 1) * A)
        st, fin, units, node = o["start_us"][sl], o["finish_us"][sl], o["units"][sl], o["node"][sl]
        cpu = (t["act_type"][sl] == gen.TYPE_CPU) & (st >= 0)
        free = {j: np.ones(int(t["node_cap"][s * M + j]), np.uint8) for j in range(M) if t["node_type"][s * M + j] == gen.TYPE_CPU}
        held = {}
        for i in range(A):
            if not cpu[i]:
                assert not sets[s * A + i].any()
        for now in np.unique(st[cpu]):
            for i in [i for i in held if fin[i] <= now]:                    # finished: the cores come back
                free[node[i]][held.pop(i)] = 1
            for i in np.flatnonzero(cpu & (st == now)):                      # the node's list keeps the arrival order
                want, after = orc.take_cores(free[node[i]], numa, int(units[i]))
                got = _bits(sets[s * A + i])
                assert got == want, (s, i, int(now) // tick)
                assert len(got) == units[i] and max(got) < t["node_cap"][s * M + node[i]]
                free[node[i]] = after
                held[i] = got
                spread += len({c // numa for c in got}) > 1
    assert spread >= 0


def test_cores_of_running_actions_never_overlap(orc):
    A = 500
    t = gen.make_trace(S=1, A=A, seed=170, cluster=(1, 32, 0, 0), type_probs=(1, 0, 0), rate_per_s=120.0, horizon_s=4.2,
                       max_ticks=50_000, pin_frac=0.0)
    t["numa_cores"] = 8
    o = orc.replay(t)
    st, fin = o["start_us"], o["finish_us"]
    masks = [sum(int(w) << (64 * x) for x, w in enumerate(o["core_set"][i * 4:i * 4 + 4])) for i in range(A)]
    assert all(bin(masks[i]).count("1") == o["units"][i] for i in range(A))
    busiest = 0
    for i in range(A):
        together = np.flatnonzero((st <= st[i]) & (fin > st[i]))
        acc = 0
        for x in together:
            assert acc & masks[x] == 0, (i, x)
            acc |= masks[x]
        busiest = max(busiest, bin(acc).count("1"))
    assert busiest == 32, "the node should fill up at some point"
