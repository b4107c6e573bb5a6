"""Benchmark of the scheduling hot path on one MI355X.

A step is one pass of the whole path over one batch of snapshots already resident in HBM:
tg_score_candidates (the (action, node, option) cost tensor) and tg_assign (admission, node
choice, DPArrange + eviction, summaries).  Workload: benchmark configuration 3, the largest
that fits one GPU (B=1024 snapshots, N=4096 actions, 256 CPU nodes x 128 cores + 32 GPU nodes
x 8 GPUs + 16 quotas, 3.34 G candidates, a 26.7 GB tensor).

Prints ONE JSON line.  `value` is candidates per second over whole steps; `roofline` is the
score kernel (8 bytes written per candidate) against the 8 TB/s HBM peak, its duration
measured with HIP events on the launch stream inside the timed region; `cpu_baseline` is the
single-threaded C++ oracle on a stated sample of the same snapshots, timed in this process -
and the GPU's results for those snapshots are compared with the oracle's before anything is
printed.  Further keys: the same step on workloads 2 and 4, options of tg_assign on workload 2,
the batched trace replay of workload 5.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per tg_score_candidates call on workload 3 (8 slabs of tg_score_dur_kernel + tg_score_kernel) from the
# FETCH_SIZE / WRITE_SIZE counter runs (profiles/score_config3_hbm_counters.md), each scaled by what the same counter reads
# for a plain device copy of the tensor: (26 108 256 + 196 608) KiB written x 1.000 + (535 280 + 50 968) KiB fetched x 2.000.
# Valid for the kernels as profiled; set to None when they change.
SCORE_TRAFFIC_CONFIG3_BYTES = (26108256 + 196608 + 2 * (535280 + 50968)) * 1024


def order_section(a, tg, torch, p, s_fcfs):
    """The same workload scheduled in the second visiting order (least estimated ACT first instead of first come
    first served): time of tg_assign, and what the order does to the selected set."""
    P = tg.Problem(dict(p, order_policy=1))
    bufs = P.alloc_assign()
    for _ in range(3):
        P.assign(None, bufs)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(5, a.steps // 5)
    e0.record()
    for _ in range(n):
        P.assign(None, bufs)
    e1.record()
    torch.cuda.synchronize()
    s = tg.summary_to_numpy(bufs["summary"])
    P.free()
    sel_f, sel_c = int(s_fcfs["n_selected"].sum()), int(s["n_selected"].sum())
    return {"assign_ms": e0.elapsed_time(e1) / n,
            "selected": {"fcfs": sel_f, "cost": sel_c},
            "mean_act_us_of_selected": {"fcfs": float(s_fcfs["sum_act_us"].sum()) / max(sel_f, 1),
                                        "cost": float(s["sum_act_us"].sum()) / max(sel_c, 1)}}


def core_sets_section(a, tg, gen, torch, p):
    """The same workload with a core map per CPU node (NUMA domains of 16 cores): tg_assign then also names the
    cores of every selected CPU action.  Time of tg_assign with that output, and how many of the selected
    multi-core actions got all their cores inside one domain."""
    import numpy as np
    q = gen.with_core_maps(dict(p), 16, 2)
    P = tg.Problem(q)
    bufs = P.alloc_assign()
    for _ in range(3):
        P.assign(None, bufs)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(5, a.steps // 5)
    e0.record()
    for _ in range(n):
        P.assign(None, bufs)
    e1.record()
    torch.cuda.synchronize()
    sets = bufs["core_set"].cpu().numpy().view(np.uint64).reshape(-1, 4)
    units = bufs["units"].cpu().numpy()
    P.free()
    multi = np.flatnonzero((units > 1) & sets.any(axis=1))
    one = 0
    for g in multi:
        dom = set()
        for w in range(4):
            v = int(sets[g][w])
            dom |= {(64 * w + c) // 16 for c in range(0, 64, 16) if v >> c & 0xffff}
        one += len(dom) == 1
    return {"assign_ms": e0.elapsed_time(e1) / n, "numa_cores": 16, "multi_core_actions": int(len(multi)),
            "in_one_domain": int(one)}


def pooled_section(a, tg, gen, torch, p):
    """The same workload with the GPU nodes of every snapshot scheduled as one pool of chunks (the GPU actions unpinned,
    the GPU nodes of a snapshot given their mean backlog, which a pool needs) against the same modified workload
    scheduled node by node: time of tg_assign, GPU actions selected and their mean ACT."""
    import numpy as np
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    M = q["M"]
    gpu_a = q["act_type"] == gen.TYPE_GPU
    q["act_pin_node"][gpu_a] = -1
    for b in range(q["B"]):
        g = np.flatnonzero(q["node_type"][b * M:(b + 1) * M] == gen.TYPE_GPU) + b * M
        if len(g):
            q["node_backlog_us"][g] = int(q["node_backlog_us"][g].mean())
    res = {}
    for name, pooled in (("per_node", 0), ("pooled", 1)):
        try:
            P = tg.Problem(dict(q, gpu_pooled=pooled))
        except tg.TgError as e:
            return {"skipped": f"this workload's GPU nodes cannot form a pool ({e})"}
        bufs = P.alloc_assign()
        for _ in range(3):
            P.assign(None, bufs)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = max(5, a.steps // 5)
        e0.record()
        for _ in range(n):
            P.assign(None, bufs)
        e1.record()
        torch.cuda.synchronize()
        units = bufs["units"].cpu().numpy()
        act = bufs["act_us"].cpu().numpy()
        P.free()
        sel = gpu_a & (units > 0)
        res[name] = {"assign_ms": e0.elapsed_time(e1) / n, "gpu_actions_selected": int(sel.sum()),
                     "mean_act_us": float(act[sel].mean()) if sel.any() else None,
                     "gpus_handed_out": int(units[sel].sum())}
    return res


def queue_prefix_section(a, tg, torch, p):
    """The same workload with one admitted prefix of the whole queue (Alg. 1 as printed) instead of one per pool:
    time of tg_assign (the placement runs twice) and how many actions are still selected."""
    P = tg.Problem(dict(p, queue_prefix=1))
    bufs = P.alloc_assign()
    for _ in range(3):
        P.assign(None, bufs)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(5, a.steps // 5)
    e0.record()
    for _ in range(n):
        P.assign(None, bufs)
    e1.record()
    torch.cuda.synchronize()
    s = tg.summary_to_numpy(bufs["summary"])
    P.free()
    return {"assign_ms": e0.elapsed_time(e1) / n, "selected_fraction": float(s["n_selected"].sum()) / (P.B * P.N)}


def replay_section(a, tg, gen, torch):
    """Workload 5 (batched trace replay): S scenarios x 10 000 Poisson arrivals over 200 s, rescheduling every
    100 ms, on the default cluster (256x128 cores, 32x8 GPUs, 16 quotas) and on the contended one (4x32 cores,
    2x8 GPUs).  One launch each after one warm-up launch; actions per second over the whole launch."""
    res = {}
    for name, contended in (("default_cluster", False), ("contended_cluster", True)):
        t = gen.make_trace(S=a.replay_scenarios, A=10_000, seed=4 + int(contended), contended=contended,
                           max_ticks=8000 if not contended else 200_000)
        T = tg.Trace(t)
        bufs = T.alloc()
        T.replay(bufs)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        T.replay(bufs)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        started = int(bufs["n_started"].sum().item())
        res[name] = {"scenarios": a.replay_scenarios, "actions": a.replay_scenarios * 10_000, "started": started,
                     "ms": ms, "actions_scheduled_per_sec": started / (ms * 1e-3),
                     "mean_act_us": float(bufs["mean_act_us"].mean().item()),
                     "mean_p99_act_us": float(bufs["p99_act_us"].double().mean().item()),
                     "mean_ticks": float(bufs["n_ticks"].double().mean().item())}
        if not a.no_cpu_baseline:
            from oracle import orc
            n = 4
            t0 = time.perf_counter()
            orc.replay(t, 0, n)
            dt = time.perf_counter() - t0
            res[name]["cpu_oracle_actions_per_sec"] = n * 10_000 / dt
            res[name]["cpu_oracle_sample"] = f"{n} scenarios, 1 core"
        # the same replay cut into pieces of 250 ticks (tg_replay_trace_part): what stopping and going on costs
        whole = {k: bufs[k].clone() for k in ("start_us", "finish_us", "units", "node")}
        limit, done, first = int(t["max_ticks"]), 0, True
        torch.cuda.synchronize()
        e0.record()
        pieces = 0
        while done < limit and a.replay_pieces:
            n = 250 if done < 2500 else limit - done                # the arrivals end after 2000 ticks: one last piece for the rest
            T.replay_part(bufs, restart=first, n_ticks=n)
            first = False
            done += n
            pieces += 1
        e1.record()
        torch.cuda.synchronize()
        if pieces:
            res[name]["in_pieces"] = {"pieces": pieces, "ms": e0.elapsed_time(e1),
                                      "equal": all(bool(torch.equal(whole[k], bufs[k])) for k in whole)}
        T.free()
        if contended:
            # the same trace with one admitted prefix of the whole queue per step (Alg. 1 as printed): two admission passes per tick
            T = tg.Trace(dict(t, queue_prefix=1))
            bufs = T.alloc()
            T.replay(bufs)
            torch.cuda.synchronize()
            e0.record()
            T.replay(bufs)
            e1.record()
            torch.cuda.synchronize()
            res[name]["queue_prefix"] = {"ms": e0.elapsed_time(e1), "mean_act_us": float(bufs["mean_act_us"].mean().item()),
                                         "started": int(bufs["n_started"].sum().item())}
            T.free()
            # the same trace in the second visiting order, with pooled GPU nodes, with named cores (NUMA domains of 16) and with a second resource per node that binds now and then
            import numpy as np
            rng = np.random.default_rng(11)
            variants = {"cost_order": dict(t, order_policy=1),       # the queue visited by least estimated ACT every tick
                        "gpu_pooled": gen.trace_with_pooled_gpus(dict(t)),   # the GPU nodes as one pool of chunks (GPU actions unpinned)
                        "named_cores": dict(t, numa_cores=16),
                        "second_resource": dict(t, act_aux=rng.integers(0, 40, t["S"] * t["A"]).astype(np.int32),
                                                node_aux=rng.integers(300, 600, t["S"] * t["M"]).astype(np.int32))}
            for vname, tv in variants.items():
                T = tg.Trace(tv)
                bufs = T.alloc()
                T.replay(bufs)
                torch.cuda.synchronize()
                e0.record()
                T.replay(bufs)
                e1.record()
                torch.cuda.synchronize()
                res[name][vname] = {"ms": e0.elapsed_time(e1), "mean_act_us": float(bufs["mean_act_us"].mean().item()),
                                    "started": int(bufs["n_started"].sum().item())}
                if vname == "named_cores":                       # sample: multi-core CPU actions of 8 scenarios whose cores share a domain
                    n8 = 8 * t["A"]
                    sets = bufs["core_set"][:4 * n8].cpu().numpy().view(np.uint64).reshape(-1, 4)
                    units = bufs["units"][:n8].cpu().numpy()
                    multi = np.flatnonzero((units > 1) & sets.any(axis=1))
                    one = sum(len({(64 * w + c) // 16 for w in range(4) for c in range(0, 64, 16) if int(sets[g][w]) >> c & 0xffff}) == 1
                              for g in multi)
                    res[name][vname].update(multi_core_actions_sampled=int(len(multi)), in_one_domain=int(one))
                T.free()
    # scheduler ablation (the paper's Fig. 7 on synthetic traces): elastic units against fixed DoP 4 and 16
    t = gen.make_trace(S=64, A=2000, seed=7, cluster=(4, 32, 0, 0), type_probs=(1, 0, 0), rate_per_s=30.0,
                       horizon_s=2000 / 30.0, max_ticks=400000, pin_frac=0.0)
    abl = {}
    for name, tt in (("elastic", t), ("dop4", gen.with_fixed_dop(t, 4)), ("dop16", gen.with_fixed_dop(t, 16))):
        T = tg.Trace(tt)
        bufs = T.replay()
        torch.cuda.synchronize()
        abl[name] = float(bufs["mean_act_us"].mean().item())
        T.free()
    res["ablation_mean_act_us"] = dict(abl, workload="64 scenarios x 2000 CPU actions at 30/s on 4 nodes x 32 cores",
                                       elastic_vs_dop4=abl["dop4"] / abl["elastic"], elastic_vs_dop16=abl["dop16"] / abl["elastic"])
    # service cache (evict on execution, LRU): the same GPU trace with room for 1, 2 and all 6 services per node
    import numpy as np
    t = gen.make_trace(S=64, A=2000, seed=8, cluster=(0, 0, 4, 0), type_probs=(0, 1, 0), rate_per_s=20.0,
                       horizon_s=100.0, max_ticks=400000, pin_frac=0.0)
    rng = np.random.default_rng(8)
    t["act_service"] = rng.integers(0, 6, t["S"] * t["A"]).astype(np.int32)
    t["restore_us"] = np.full(6, 2_000_000, np.int64)
    cache = {}
    for slots in (1, 2, 6):
        t["cache_slots"] = slots
        T = tg.Trace(t)
        bufs = T.replay()
        torch.cuda.synchronize()
        cache[f"slots_{slots}"] = float(bufs["mean_act_us"].mean().item())
        T.free()
        # the same with the cache on every GPU (Sec. 5.3: the chunk that caches the service comes first)
        T = tg.Trace(dict(t, cache_per_gpu=1))
        bufs = T.replay()
        torch.cuda.synchronize()
        cache[f"slots_{slots}_per_gpu"] = float(bufs["mean_act_us"].mean().item())
        T.free()
    res["service_cache_mean_act_us"] = dict(cache, workload="64 scenarios x 2000 GPU actions at 20/s on 4 nodes x 8 GPUs, "
                                                           "6 services, 2 s to restore one")
    return res


def host_cpu_model():
    """Model name of the host processor the oracle is timed on (first entry of /proc/cpuinfo), or None."""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def time_steps(a, tg, torch, P, cost, bufs, mode, steps, warmup):
    """`steps` timed steps after `warmup` untimed ones.  Returns (ms per step, mean ms of the score kernels, mean ms of
    tg_assign or None), stage times from HIP events on the stream the kernels are launched on.
    mode "two_streams": tg_score_candidates on a second stream next to tg_assign on the first; "serial": the two calls
    one after the other on one stream; "score" / "assign": that call alone.  (The events are recorded right after the
    call they bracket is enqueued, before the next one: two streams may share a hardware queue.)"""
    import numpy as np
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream() if mode == "two_streams" else None

    def step(ev=None):
        e0, e1, e2, e3 = ev if ev else (None,) * 4
        if mode == "two_streams":
            fork = torch.cuda.Event()
            fork.record(main_stream)
            side_stream.wait_event(fork)
            with torch.cuda.stream(side_stream):
                if ev:
                    e0.record(side_stream)
                P.score(cost)
                done = e1 if ev else torch.cuda.Event()
                done.record(side_stream)
            if ev:
                e2.record(main_stream)
            P.assign(None, bufs)
            if ev:
                e3.record(main_stream)
            main_stream.wait_event(done)
            return
        if ev:
            e0.record()
        if mode in ("serial", "score"):
            P.score(cost)
        if ev:
            e1.record(); e2.record()
        if mode in ("serial", "assign"):
            P.assign(cost if a.use_cost else None, bufs)
        if ev:
            e3.record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(4)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(ev[k])       # events bracket each call on the stream it is launched on
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    score = float(np.mean([e0.elapsed_time(e1) for e0, e1, _, _ in ev])) if mode != "assign" else None
    assign = float(np.mean([e2.elapsed_time(e3) for _, _, e2, e3 in ev])) if mode != "score" else None
    return (t1 - t0) * 1e3 / steps, score, assign


def check_against_oracle(p, gen, orc, tg, P, cost, bufs, snapshots):
    """The GPU's score tensor and assignment of the listed snapshots against the oracle run on the same snapshots;
    raises on any difference.  Returns the oracle's times (score seconds, assign seconds) and the candidates of the sample."""
    import numpy as np
    B, N, M = p["B"], p["N"], p["M"]
    at, nt = p["act_type"].reshape(B, N), p["node_type"].reshape(B, M)
    per = np.zeros(B, np.int64)
    for t in range(3):
        per += (at == t).sum(1).astype(np.int64) * (nt == t).sum(1) * int(p["type_k"][t])
    off = np.concatenate([[0], np.cumsum(per)])
    q = gen.slice_problem(p, snapshots)
    t0 = time.perf_counter()
    want_cost = orc.score(q)
    t_score = time.perf_counter() - t0
    t0 = time.perf_counter()
    want = orc.assign(q)
    t_assign = time.perf_counter() - t0
    pos = 0
    for b in snapshots:
        got = cost[int(off[b]):int(off[b + 1])].cpu().numpy()
        if not np.array_equal(got, want_cost[pos:pos + len(got)]):
            raise RuntimeError(f"score tensor of snapshot {b} differs from the oracle's")
        pos += len(got)
    summ = tg.summary_to_numpy(bufs["summary"])
    for x, b in enumerate(snapshots):
        for k_got, k_want, n in (("node", "node", N), ("units", "units", N), ("act_us", "act_us", N),
                                 ("defer_reason", "reason", N), ("node_used", "node_used", M), ("node_obj", "node_obj", M)):
            got = bufs[k_got][b * n:(b + 1) * n].cpu().numpy()
            if not np.array_equal(got, want[k_want][x * n:(x + 1) * n]):
                raise RuntimeError(f"{k_got} of snapshot {b} differs from the oracle's")
        if int(summ[b]["sum_act_us"]) != int(want["summary"][x]["sum_act_us"]) or \
                int(summ[b]["n_selected"]) != int(want["summary"][x]["n_assigned"]):
            raise RuntimeError(f"summary of snapshot {b} differs from the oracle's")
    return t_score, t_assign, int(len(want_cost))


def other_workload(a, tg, gen, torch, cfg):
    """One of the smaller workloads stepped the same way (not the headline): step time, stage times, score rate."""
    p = gen.make_config(cfg)
    P = tg.Problem(p)
    cost, bufs = P.alloc_cost(), P.alloc_assign()
    steps = max(10, a.steps)
    ms_step, score_ms, assign_ms = time_steps(a, tg, torch, P, cost, bufs, "two_streams", steps, 3)
    _, score_alone, _ = time_steps(a, tg, torch, P, cost, bufs, "score", steps, 2)
    _, _, assign_alone = time_steps(a, tg, torch, P, cost, bufs, "assign", steps, 2)
    for _ in range(3):
        P.step(cost, bufs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        P.step(cost, bufs)
    torch.cuda.synchronize()
    ms_lib = (time.perf_counter() - t0) * 1e3 / steps
    res = {"workload": f"config{cfg}: B={P.B} x N={P.N}, M={P.M}, {P.num_candidates} candidates; tg_score_candidates on a second "
                       "stream next to tg_assign",
           "ms_per_step": ms_step, "candidates_per_sec": P.num_candidates / (ms_step * 1e-3),
           "actions_scheduled_per_sec": P.B * P.N / (ms_step * 1e-3), "tg_step_ms_per_step": ms_lib,
           "stage_ms": {"score": score_ms, "assign": assign_ms, "score_alone": score_alone, "assign_alone": assign_alone},
           "score_hbm_frac_in_step": 8.0 * P.num_candidates / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "score_hbm_frac_alone": 8.0 * P.num_candidates / (score_alone * 1e-3) / 1e9 / HBM_PEAK_GBS}
    P.free()
    return res, p


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4])
    ap.add_argument("--snapshots", type=int, default=None, help="override B (sampling of big configs)")
    ap.add_argument("--use-cost", type=int, default=0, help="1: tg_assign reads its estimates from the score tensor")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (no baseline, no check of the results)")
    ap.add_argument("--replay-scenarios", type=int, default=4096,
                    help="scenarios of workload 5 (10 000 arrivals each) replayed after the timed steps; 0 = skip")
    ap.add_argument("--replay-pieces", type=int, default=1, help="0: leave out the replays cut into pieces")
    ap.add_argument("--extras", type=int, default=1, help="0: only the timed steps of the chosen workload (and the baseline)")
    ap.add_argument("--only", choices=["step", "score", "assign"], default="step")
    ap.add_argument("--overlap", type=int, default=-1,
                    help="0: tg_score_candidates, then tg_assign, on one stream; 1: tg_score_candidates on a second stream next "
                         "to tg_assign; default: as tg_step does, 0 for a tensor of 4 GB and more, else 1")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain device copies of the score tensor's size (reference for the HBM byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: the path runs on a single MI355X and uses no "
              "collectives; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import gen
    from paper_2603_13019_amd import tg

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    tg.load()
    p = gen.make_config(a.config, B=a.snapshots)
    P = tg.Problem(p)
    cost = P.alloc_cost()
    bufs = P.alloc_assign()
    n_cand, n_act = P.num_candidates, P.B * P.N

    # A step is the two calls in the order tg_step runs them: a tensor of 4 GB and more is written first and the assignment
    # follows on the same stream (side by side the two only slow each other down, see two_calls_on_two_streams); a smaller
    # tensor is written on a second stream next to the assignment.  --overlap 0 / 1 forces one or the other.
    big = n_cand >= 1 << 29
    mode = a.only if a.only != "step" else ("serial" if a.use_cost or a.overlap == 0 or (a.overlap < 0 and big) else "two_streams")
    ms_step, score_ms, assign_ms = time_steps(a, tg, torch, P, cost, bufs, mode, a.steps, a.warmup)
    if a.calibrate_copy:      # a copy kernel reads and writes exactly 8 * n_cand bytes
        dst = torch.empty_like(cost)
        for _ in range(3):
            dst.copy_(cost)
        torch.cuda.synchronize()
        del dst

    s = tg.summary_to_numpy(bufs["summary"]) if a.only != "score" else None
    achieved = 8.0 * n_cand / (score_ms * 1e-3) / 1e9 if a.only != "assign" and score_ms > 0 else None
    out = {
        "metric": "candidates_per_sec", "value": n_cand / (ms_step * 1e-3), "unit": "candidates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"config{a.config}: B={P.B} snapshots x N={P.N} actions, M={P.M} nodes, "
                               f"{n_cand} candidates; step = "
                               + {"two_streams": "tg_score_candidates on a second stream next to tg_assign",
                                  "serial": "tg_score_candidates, then tg_assign, on one stream (the order tg_step uses for a tensor of this size)",
                                  "score": "tg_score_candidates only", "assign": "tg_assign only"}[mode],
                   "B": P.B, "N": P.N, "M": P.M, "candidates": n_cand, "assign_reads_score_tensor": bool(a.use_cost),
                   "only": a.only, "mode": mode},
        "actions_scheduled_per_sec": n_act / (ms_step * 1e-3) if a.only != "score" else None,
        "stage_ms": {"score": score_ms, "assign": assign_ms},
        "selected_fraction": float(s["n_selected"].sum()) / n_act if s is not None else None,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS if achieved else None,
                     "traffic": SCORE_TRAFFIC_CONFIG3_BYTES if (a.config == 3 and a.snapshots is None) else None,
                     "kernel": "tg_score_kernel (the events bracket all score kernels of a step on their stream: slabs of "
                               "tg_score_dur_kernel, 2 % of the time, and tg_score_kernel)",
                     "bytes_per_launch": 8 * n_cand, "avg_kernel_ms": score_ms},
    }

    if a.only == "step" and a.extras:
        # each call alone, back to back with itself, and the two calls on two streams side by side (not the headline)
        n_x = max(5, a.steps // 4)
        _, score_alone, _ = time_steps(a, tg, torch, P, cost, bufs, "score", n_x, 1)
        _, _, assign_alone = time_steps(a, tg, torch, P, cost, bufs, "assign", n_x, 1)
        out["stage_ms_alone"] = {"score": score_alone, "assign": assign_alone}
        out["roofline"]["frac_alone"] = 8.0 * n_cand / (score_alone * 1e-3) / 1e9 / HBM_PEAK_GBS
        other = "two_streams" if mode == "serial" else "serial"
        ms_o, score_o, assign_o = time_steps(a, tg, torch, P, cost, bufs, other, n_x, 1)
        out["other_order"] = {"order": "two streams side by side" if other == "two_streams" else "one after the other",
                              "ms_per_step": ms_o, "score": score_o, "assign": assign_o,
                              "score_hbm_frac": 8.0 * n_cand / (score_o * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # the same step through the library's one-call entry point
        for _ in range(3):
            P.step(cost, bufs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            P.step(cost, bufs)
        torch.cuda.synchronize()
        out["tg_step_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / a.steps

    if not a.no_cpu_baseline and a.only == "step":
        # the oracle on a bounded sample of the same snapshots (one host core), and the GPU's results for exactly those
        # snapshots compared with it: a line is only printed for results that agree
        from oracle import orc
        orc.lib()
        P.score(cost)
        P.assign(None, bufs)
        torch.cuda.synchronize()
        n_s = min(P.B, {1: 1, 2: 256, 3: 56, 4: 1}[a.config])
        sample = sorted({int(x) for x in np.linspace(0, P.B - 1, n_s)})
        t_score, t_assign, cand_s = check_against_oracle(p, gen, orc, tg, P, cost, bufs, sample)
        out["cpu_baseline"] = {
            "value": cand_s / (t_score + t_assign), "unit": "candidates/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(sample)} of the {P.B} snapshots of the same workload, evenly spaced ({cand_s} candidates), one pass "
                      f"(score {t_score:.2f} s + assign {t_assign:.2f} s); the GPU's tensor and assignment of these "
                      f"snapshots were compared with the oracle's: equal",
            "actions_scheduled_per_sec": len(sample) * P.N / t_assign, "score_candidates_per_sec": cand_s / t_score,
            "host_cores_total": os.cpu_count(), "host_cpu": host_cpu_model(),
        }

    if a.only == "step" and a.extras:
        # Several batches in flight: a step is bound by the latency of single wavefronts, so a caller with several
        # independent batches of snapshots can overlap their steps.  n problems (the same workload n times, each with its
        # own outputs, tensor and workspace) stepped in turn on n streams; not the headline.
        extra = []
        out["batches_in_flight"] = {}
        for n_fly in (2,):
            while len(extra) < n_fly - 1:
                Pn = tg.Problem(p)
                extra.append((Pn, Pn.alloc_cost(), Pn.alloc_assign()))
            group = [(P, cost, bufs)] + extra[:n_fly - 1]
            streams = [torch.cuda.Stream() for _ in range(n_fly)]
            torch.cuda.synchronize()
            for rounds, timed in ((2, False), (max(5, a.steps // 2), True)):
                t0 = time.perf_counter()
                for _ in range(rounds):
                    for x in range(n_fly):
                        with torch.cuda.stream(streams[x]):
                            group[x][0].step(group[x][1], group[x][2])
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
            same = all(bool(torch.equal(bufs[k], g[2][k])) for g in group[1:] for k in ("node", "units", "act_us", "defer_reason"))
            out["batches_in_flight"][str(n_fly)] = {"ms_per_step": dt * 1e3 / (n_fly * rounds), "steps": n_fly * rounds,
                                                    "candidates_per_sec": n_cand * n_fly * rounds / dt, "results_equal": same}
        for g in extra:
            g[0].free()
            del g
        del extra
        # Alg. 1 as printed (one admitted prefix of the whole queue) on the headline workload, next to the default
        out["queue_prefix_headline_workload"] = queue_prefix_section(a, tg, torch, p)
    P.free()
    del cost, bufs

    if a.only == "step" and a.extras:
        out["other_workloads"] = {}
        for cfg in (2, 4):
            if cfg == a.config:
                continue
            res, p_small = other_workload(a, tg, gen, torch, cfg)
            out["other_workloads"][f"config{cfg}"] = res
            if cfg == 2:
                P2 = tg.Problem(p_small)
                b2 = P2.alloc_assign()
                P2.assign(None, b2)
                torch.cuda.synchronize()
                s2 = tg.summary_to_numpy(b2["summary"])
                P2.free()
                opt = {"workload": res["workload"]}
                opt["order_policy_cost"] = order_section(a, tg, torch, p_small, s2)
                opt["core_sets"] = core_sets_section(a, tg, gen, torch, p_small)
                opt["gpu_pooled"] = pooled_section(a, tg, gen, torch, p_small)
                opt["queue_prefix"] = queue_prefix_section(a, tg, torch, p_small)
                out["assign_options"] = opt
    if a.replay_scenarios > 0 and a.only == "step" and a.extras:
        out["replay"] = replay_section(a, tg, gen, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
