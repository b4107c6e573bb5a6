"""GPU checks that are not parity with the oracle: run-to-run determinism, back-to-back launches
without host synchronisation (tg_assign forks onto side streams and joins), reuse of one problem,
and the time the formulation stage (tg_build_problem: host validation + packing + H2D) takes."""
import time

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


def test_assign_is_deterministic_and_reentrant(tg):
    import torch
    p = gen.make_config(2, B=32)
    P = tg.Problem(p)
    cost = P.score()
    first = None
    bufs_a, bufs_b = P.alloc_assign(), P.alloc_assign()
    for rep in range(3):
        # two launches in flight on the same stream, different outputs and workspaces, no sync between
        P.assign(None, bufs_a)
        P.assign(cost, bufs_b)
        torch.cuda.synchronize()
        snap = {k: bufs_a[k].cpu().numpy().copy() for k in ("node", "units", "act_us", "defer_reason", "summary", "node_used", "node_obj")}
        for k in snap:
            np.testing.assert_array_equal(snap[k], bufs_b[k].cpu().numpy(), err_msg=k)   # tensor path == recompute path
        if first is None:
            first = snap
        for k in snap:
            np.testing.assert_array_equal(snap[k], first[k], err_msg=f"run {rep} {k}")
    P.free()


def test_score_and_assign_side_by_side(tg):
    """tg_score_candidates on a second stream while tg_assign runs on the first (the launch pattern of
    bench.py): both results equal those of the calls made one after the other."""
    import torch
    p = gen.make_config(2, B=48)
    P = tg.Problem(p)
    cost_ref = P.score()
    bufs_ref = P.alloc_assign()
    P.assign(None, bufs_ref)
    torch.cuda.synchronize()
    keys = ("node", "units", "act_us", "defer_reason", "summary", "node_used", "node_obj", "task_sum_us")
    want = {k: bufs_ref[k].cpu().numpy().copy() for k in keys}
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    cost, bufs = P.alloc_cost(), P.alloc_assign()
    for rep in range(5):
        cost.fill_(-7)
        fork = torch.cuda.Event()
        fork.record(main)
        side.wait_event(fork)
        with torch.cuda.stream(side):
            P.score(cost)
            done = torch.cuda.Event()
            done.record(side)
        P.assign(None, bufs)
        main.wait_event(done)
        torch.cuda.synchronize()
        assert torch.equal(cost, cost_ref), f"run {rep}: score tensor"
        for k in keys:
            np.testing.assert_array_equal(bufs[k].cpu().numpy(), want[k], err_msg=f"run {rep} {k}")
    P.free()


def test_step_in_one_call(tg):
    """tg_step == tg_score_candidates + tg_assign, also back to back without host synchronisation."""
    import torch
    p = gen.make_config(2, B=40)
    P = tg.Problem(p)
    cost_ref = P.score()
    bufs_ref = P.alloc_assign()
    P.assign(None, bufs_ref)
    torch.cuda.synchronize()
    keys = ("node", "units", "act_us", "defer_reason", "summary", "node_used", "node_obj", "task_sum_us")
    cost, bufs = P.alloc_cost(), P.alloc_assign()
    for rep in range(3):
        cost.fill_(-7)
        for k in keys:
            bufs[k].fill_(0)
        P.step(cost, bufs)
        P.step(cost, bufs)
        torch.cuda.synchronize()
        assert torch.equal(cost, cost_ref), f"run {rep}: score tensor"
        for k in keys:
            np.testing.assert_array_equal(bufs[k].cpu().numpy(), bufs_ref[k].cpu().numpy(), err_msg=f"run {rep} {k}")
    P.free()


def test_replay_is_deterministic(tg):
    import torch
    t = gen.make_trace(S=16, A=1500, seed=33, contended=True, rate_per_s=150.0, horizon_s=10.0, max_ticks=50000)
    T = tg.Trace(t)
    outs = []
    for _ in range(2):
        bufs = T.replay()
        torch.cuda.synchronize()
        outs.append({k: v.cpu().numpy().copy() for k, v in bufs.items() if k != "ws"})
    for k in outs[0]:
        np.testing.assert_array_equal(outs[0][k], outs[1][k], err_msg=k)
    T.free()


def test_build_problem_time_is_reported(tg):
    """Boundary-inclusive cost: the formulation stage takes host buffers; its time is printed."""
    import torch
    p = gen.make_config(2)
    t0 = time.perf_counter()
    P = tg.Problem(p)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    print(f"tg_build_problem on workload 2 (262144 actions, 18432 nodes): {dt * 1e3:.1f} ms", flush=True)
    assert P.num_candidates == 68787392
    P.free()


@pytest.mark.parametrize("one_call", [False, True])
def test_step_can_be_captured_into_a_graph(tg, one_call):
    """tg_score_candidates + tg_assign, or tg_step (streams forked and joined with events, no memsets) recorded
    into a HIP graph: every replay, with eager launches and synchronisations in between, reproduces the
    eager result."""
    import torch
    p = gen.make_config(2, B=24)
    P = tg.Problem(p)
    cost, bufs = P.alloc_cost(), P.alloc_assign()

    def step():
        if one_call:
            P.step(cost, bufs)
        else:
            P.score(cost)
            P.assign(cost, bufs)

    step()
    torch.cuda.synchronize()
    keys = ("node", "units", "act_us", "defer_reason", "node_used", "node_obj", "summary")
    ref = {k: bufs[k].clone() for k in keys}
    ref_cost = cost.clone()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        step()                                                   # the stream has run the step once before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        cost.fill_(0)
        for k in keys:
            bufs[k].fill_(0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(cost, ref_cost), f"replay {rep}: score tensor"
        for k in keys:
            assert torch.equal(bufs[k], ref[k]), f"replay {rep}: {k}"
        step()                                                   # eager work between the replays
        torch.cuda.synchronize()
    del g
    P.free()


def test_steps_of_several_problems_in_flight(tg):
    """Independent problems stepped at the same time on streams of their own (each problem has its own internal streams
    and events) give what each gives alone; also two launches of the same problem into different outputs."""
    import torch
    probs = [gen.make_config(2, B=24, seed=70 + i) for i in range(3)]
    P = [tg.Problem(p) for p in probs]
    keys = ("node", "units", "act_us", "defer_reason", "summary", "node_used", "node_obj", "task_sum_us")
    ref = []
    for x in P:                                                # one at a time
        c, b = x.alloc_cost(), x.alloc_assign()
        x.step(c, b)
        torch.cuda.synchronize()
        ref.append((c.clone(), {k: b[k].clone() for k in keys}))
    streams = [torch.cuda.Stream() for _ in range(4)]
    work = [(P[0], P[0].alloc_cost(), P[0].alloc_assign()), (P[1], P[1].alloc_cost(), P[1].alloc_assign()),
            (P[2], P[2].alloc_cost(), P[2].alloc_assign()), (P[0], P[0].alloc_cost(), P[0].alloc_assign())]
    which = [0, 1, 2, 0]
    torch.cuda.synchronize()
    for rep in range(4):
        for x, (prob, c, b) in enumerate(work):
            c.fill_(-7)
            for k in keys:
                b[k].fill_(0)
        torch.cuda.synchronize()
        for x, (prob, c, b) in enumerate(work):
            with torch.cuda.stream(streams[x]):
                prob.step(c, b)
        torch.cuda.synchronize()
        for x, (prob, c, b) in enumerate(work):
            assert torch.equal(c, ref[which[x]][0]), f"run {rep} launch {x}: score tensor"
            for k in keys:
                assert torch.equal(b[k], ref[which[x]][1][k]), f"run {rep} launch {x}: {k}"
    for x in P:
        x.free()
