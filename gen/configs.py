"""Seeded generators for the five benchmark workloads and for random test problems.

A *problem* is a dict of numpy arrays describing B independent cluster
snapshots (N queued actions in first-come order, M resource nodes) and a
*trace* is a dict describing S independent arrival traces.  Array names follow
the C interface of the scheduler library.  Everything is drawn from
``numpy.random.default_rng(seed)``; nothing here evaluates durations, costs or
assignments.
"""
from __future__ import annotations

import numpy as np

TYPE_CPU, TYPE_GPU, TYPE_API = 0, 1, 2
MODEL_NONE, MODEL_AMDAHL, MODEL_TABLE = 0, 1, 2

T_MAX = (1 << 36) - 1

PROBLEM_ARRAYS = (
    "k_list", "type_k", "speedup_q16",
    "node_type", "node_cap", "node_free", "node_backlog_us", "node_chunks",
    "node_busy_off", "node_busy_rel_us",
    "act_type", "act_model", "act_t_ori_us", "act_age_us", "act_kmask",
    "act_param", "act_pin_node", "act_task",
)
TRACE_ARRAYS = (
    "k_list", "type_k", "speedup_q16",
    "node_type", "node_cap", "quota_rate", "quota_tok0_micro",
    "arrival_us", "act_type", "act_model", "act_t_ori_us", "act_kmask",
    "act_param", "act_pin_node",
)

# elasticity classes of the table model: speedup(k) = k**alpha
CLASS_ALPHA = (0.8, 0.9, 1.0, 0.5)


def _lognormal_us(rng, median_us, sigma, size):
    z = rng.standard_normal(size)
    t = np.rint(np.exp(np.log(median_us) + sigma * z))
    return np.clip(t, 1, T_MAX).astype(np.int64)


def _speedup_table(k_list):
    k = np.asarray(k_list, dtype=np.float64)
    rows = [np.rint(65536.0 * k ** a) for a in CLASS_ALPHA]
    return np.stack(rows).astype(np.uint32).reshape(-1)


def _chunks_from_free(free):
    """Binary decomposition of a free-GPU count into chunks of size 1,2,4,8."""
    free = np.asarray(free, dtype=np.int64)
    out = np.zeros(free.shape + (4,), dtype=np.uint8)
    out[..., 3] = free // 8
    r = free % 8
    out[..., 2] = (r >> 2) & 1
    out[..., 1] = (r >> 1) & 1
    out[..., 0] = r & 1
    return out


def _chunks_from_mask(mask8):
    """Free buddy chunks (sizes 1,2,4,8) of an 8-GPU node whose free GPUs are the set bits."""
    c = [0, 0, 0, 0]
    m = int(mask8) & 0xFF
    if m == 0xFF:
        return (0, 0, 0, 1)
    for half in (0, 4):
        h = (m >> half) & 0xF
        if h == 0xF:
            c[2] += 1
            continue
        for pair in (0, 2):
            p = (h >> pair) & 0x3
            if p == 0x3:
                c[1] += 1
            else:
                c[0] += bin(p).count("1")
    return tuple(c)


def _base(B, N, M, k_list, type_k, depth=2, n_tasks=1):
    K = len(k_list)
    p = dict(
        B=B, N=N, M=M, K=K, n_classes=len(CLASS_ALPHA), n_tasks=n_tasks, depth=depth,
        k_list=np.asarray(k_list, dtype=np.int32),
        type_k=np.asarray(type_k, dtype=np.int32),
        speedup_q16=_speedup_table(k_list),
        node_busy_off=None, node_busy_rel_us=None,
    )
    return p


def _cluster(rng, B, n_cpu, cpu_cap, n_gpu, n_api, backlog_hi=5_000_000):
    """Node tables [B*M]: CPU nodes, then 8-GPU nodes, then API quotas."""
    M = n_cpu + n_gpu + n_api
    node_type = np.concatenate([
        np.full(n_cpu, TYPE_CPU, np.uint8), np.full(n_gpu, TYPE_GPU, np.uint8),
        np.full(n_api, TYPE_API, np.uint8)])
    node_type = np.tile(node_type, B)
    cap = np.concatenate([
        np.full(n_cpu, cpu_cap, np.int32), np.full(n_gpu, 8, np.int32), np.zeros(n_api, np.int32)])
    cap = np.tile(cap, B)
    free = cap.copy()
    rate = np.zeros(B * M, np.int32)
    if n_api:
        api = node_type == TYPE_API
        n = int(api.sum())
        rate[api] = rng.integers(10, 201, n)
        burst = rng.integers(20, 501, n).astype(np.int32)
        cap[api] = burst
        free[api] = np.floor(rng.random(n) * (burst + 1)).astype(np.int32).clip(0, burst)
    backlog = rng.integers(0, backlog_hi + 1, B * M).astype(np.int64)
    backlog[node_type == TYPE_API] = 0
    chunks = np.zeros((B * M, 4), np.uint8)
    g = node_type == TYPE_GPU
    chunks[g] = _chunks_from_free(free[g])
    return M, node_type, cap, free, backlog, chunks.reshape(-1), rate


def _cpu_masks(rng, n, K):
    full = (1 << K) - 1
    u = rng.random(n)
    m = np.full(n, full, np.uint32)
    m[u < 0.10] = full & ~1            # needs at least k_list[1] units
    lim = (1 << min(K, 3)) - 1
    m[u > 0.90] = lim                  # capped at k_list[2]
    return m


def _actions(rng, p, type_probs, cpu_median=2_000_000, cpu_sigma=1.0,
             pin_frac=0.25, nonelastic_frac=0.10, age_hi=1_000_000):
    B, N, M = p["B"], p["N"], p["M"]
    n = B * N
    node_type = p["node_type"].reshape(B, M)
    t = rng.choice(3, size=n, p=type_probs).astype(np.uint8)
    model = np.zeros(n, np.uint8)
    T = np.zeros(n, np.int64)
    kmask = np.zeros(n, np.uint32)
    param = np.zeros(n, np.uint32)
    pin = np.full(n, -1, np.int32)
    snap = np.repeat(np.arange(B), N)

    c = t == TYPE_CPU
    nc = int(c.sum())
    T[c] = _lognormal_us(rng, cpu_median, cpu_sigma, nc)
    model[c] = np.where(rng.random(nc) < nonelastic_frac, MODEL_NONE, MODEL_AMDAHL)
    param[c] = np.rint(rng.uniform(0.5, 0.95, nc) * 1e6).astype(np.uint32)
    kmask[c] = _cpu_masks(rng, nc, int(p["type_k"][TYPE_CPU]))

    g = t == TYPE_GPU
    ng = int(g.sum())
    if ng:
        T[g] = _lognormal_us(rng, 300_000, 0.7, ng)
        model[g] = MODEL_TABLE
        param[g] = rng.integers(0, 2, ng)          # class 0 (k^0.8) or 1 (k^0.9)
        kg = int(p["type_k"][TYPE_GPU])
        mg = np.full(ng, (1 << kg) - 1, np.uint32)
        mg[rng.random(ng) < 0.10] = ((1 << kg) - 1) & ~1
        kmask[g] = mg

    a = t == TYPE_API
    na = int(a.sum())
    if na:
        T[a] = _lognormal_us(rng, 300_000, 0.7, na)
        model[a] = MODEL_NONE
        kmask[a] = 1

    # pins: API actions always name their quota; a fraction of CPU/GPU actions
    # belong to a trajectory already bound to a node
    for ty, frac in ((TYPE_CPU, pin_frac), (TYPE_GPU, pin_frac), (TYPE_API, 1.0)):
        sel = np.flatnonzero(t == ty)
        if sel.size == 0:
            continue
        ids = np.flatnonzero(node_type[0] == ty)   # same layout in every snapshot
        if ids.size == 0:
            continue
        chosen = sel[rng.random(sel.size) < frac] if frac < 1.0 else sel
        pin[chosen] = ids[rng.integers(0, ids.size, chosen.size)]

    p.update(act_type=t, act_model=model, act_t_ori_us=T,
             act_age_us=rng.integers(0, age_hi + 1, n).astype(np.int64),
             act_kmask=kmask, act_param=param, act_pin_node=pin,
             act_task=np.zeros(n, np.int32))
    del snap
    return p


def make_config(cfg: int, B: int | None = None, seed: int | None = None):
    """Benchmark snapshot workloads 1-4 (``B`` overrides the snapshot count for sampling)."""
    if seed is None:
        seed = cfg - 1
    rng = np.random.default_rng(seed)
    if cfg == 1:
        B = B or 1
        p = _base(B, 64, 4, [1, 2, 4, 8], [4, 0, 0])
        M, nt, cap, free, bl, ch, _ = _cluster(rng, B, 4, 32, 0, 0)
        p.update(node_type=nt, node_cap=cap, node_free=free, node_backlog_us=bl, node_chunks=ch)
        _actions(rng, p, [1.0, 0.0, 0.0], pin_frac=0.0, nonelastic_frac=0.0, age_hi=0)
        p["act_kmask"][:] = 0xF
        return p
    if cfg == 2:
        B = B or 256
        p = _base(B, 1024, 72, [1, 2, 4, 8, 16], [5, 4, 0])
        M, nt, cap, free, bl, ch, _ = _cluster(rng, B, 64, 128, 8, 0)
        p.update(node_type=nt, node_cap=cap, node_free=free, node_backlog_us=bl, node_chunks=ch)
        return _actions(rng, p, [0.8, 0.2, 0.0])
    if cfg == 3:
        B = B or 1024
        p = _base(B, 4096, 304, [1, 2, 4, 8, 16], [5, 4, 1])
        M, nt, cap, free, bl, ch, _ = _cluster(rng, B, 256, 128, 32, 16)
        p.update(node_type=nt, node_cap=cap, node_free=free, node_backlog_us=bl, node_chunks=ch)
        return _actions(rng, p, [0.6, 0.2, 0.2])
    if cfg == 4:
        B = B or 1
        n_tasks = 64
        p = _base(B, 65536, 1152, [1, 2, 4, 8, 16, 32], [6, 4, 0], n_tasks=n_tasks)
        M, nt, cap, free, bl, ch, _ = _cluster(rng, B, 1024, 192, 128, 0)
        p.update(node_type=nt, node_cap=cap, node_free=free, node_backlog_us=bl, node_chunks=ch)
        _actions(rng, p, [0.8, 0.2, 0.0], cpu_median=1_000_000, cpu_sigma=1.5)
        n = B * p["N"]
        w = 1.0 / np.arange(1, n_tasks + 1) ** 1.2
        task = rng.choice(n_tasks, size=n, p=w / w.sum()).astype(np.int32)
        p["act_task"] = task
        # the task fixes elasticity class and unit mask of its actions
        task_p = np.rint(rng.uniform(0.5, 0.95, n_tasks) * 1e6).astype(np.uint32)
        task_mask_cpu = _cpu_masks(rng, n_tasks, 6)
        task_nonel = (np.arange(n_tasks) % 8) == 7
        c = p["act_type"] == TYPE_CPU
        p["act_param"][c] = task_p[task[c]]
        p["act_kmask"][c] = task_mask_cpu[task[c]]
        p["act_model"][c] = np.where(task_nonel[task[c]], MODEL_NONE, MODEL_AMDAHL)
        g = p["act_type"] == TYPE_GPU
        p["act_param"][g] = (task[g] % 3).astype(np.uint32)
        p["act_t_ori_us"][g] = _lognormal_us(rng, 1_000_000, 1.5, int(g.sum()))
        return p
    raise ValueError("snapshot configs are 1..4; config 5 is make_trace()")


def subset_problem(p, lo, hi, n_cpu_nodes=2, cap=8, seed=0):
    """Actions lo..hi of snapshot 0 on a shrunk CPU cluster so that capacity binds (brute-force cases)."""
    rng = np.random.default_rng(seed)
    N = hi - lo
    q = _base(1, N, n_cpu_nodes, p["k_list"], p["type_k"], depth=p["depth"])
    q.update(
        node_type=np.zeros(n_cpu_nodes, np.uint8),
        node_cap=np.full(n_cpu_nodes, cap, np.int32),
        node_free=np.full(n_cpu_nodes, cap, np.int32),
        node_backlog_us=rng.integers(0, 5_000_001, n_cpu_nodes).astype(np.int64),
        node_chunks=np.zeros(n_cpu_nodes * 4, np.uint8),
    )
    for k in ("act_type", "act_model", "act_t_ori_us", "act_age_us", "act_kmask", "act_param", "act_task"):
        q[k] = p[k][lo:hi].copy()
    q["act_pin_node"] = np.full(N, -1, np.int32)
    return q


def make_random_problem(seed, B=2, N=40, n_cpu=3, n_gpu=2, n_api=2, cpu_cap_hi=24,
                        k_list=(1, 2, 4, 8), depth=2, busy=True, pin_frac=0.3,
                        bad_frac=0.05, shuffle_nodes=True, t_median=2_000_000, type_probs=(0.6, 0.25, 0.15)):
    """Adversarial small problems: partly occupied nodes, fragmented GPU nodes, running
    actions (busy units), shuffled node order, pins, non-elastic and infeasible actions,
    duplicate durations (ties)."""
    rng = np.random.default_rng(seed)
    K = len(k_list)
    M = n_cpu + n_gpu + n_api
    kg = sum(1 for k in k_list if k <= 8)
    p = _base(B, N, M, list(k_list), [K, kg, 1 if n_api else 0], depth=depth, n_tasks=4)
    node_type = np.zeros((B, M), np.uint8)
    cap = np.zeros((B, M), np.int32)
    free = np.zeros((B, M), np.int32)
    backlog = np.zeros((B, M), np.int64)
    chunks = np.zeros((B, M, 4), np.uint8)
    busy_cnt = np.zeros((B, M), np.int64)
    busy_vals = []
    gpu_mask = np.zeros((B, M), np.int32)
    base_types = np.array([TYPE_CPU] * n_cpu + [TYPE_GPU] * n_gpu + [TYPE_API] * n_api, np.uint8)
    for b in range(B):
        ty = base_types.copy()
        if shuffle_nodes:
            rng.shuffle(ty)
        node_type[b] = ty
        for j in range(M):
            if ty[j] == TYPE_CPU:
                cap[b, j] = rng.integers(1, cpu_cap_hi + 1)
                free[b, j] = rng.integers(0, cap[b, j] + 1)
                backlog[b, j] = rng.integers(0, 4) * 500_000
            elif ty[j] == TYPE_GPU:
                cap[b, j] = 8
                mask = int(rng.integers(0, 256)) if rng.random() < 0.7 else 0xFF
                chunks[b, j] = _chunks_from_mask(mask)
                gpu_mask[b, j] = mask
                free[b, j] = bin(mask).count("1")
                backlog[b, j] = rng.integers(0, 3) * 250_000
            else:
                cap[b, j] = rng.integers(1, 12)
                free[b, j] = rng.integers(0, cap[b, j] + 1)
            if busy and ty[j] != TYPE_API:
                busy_cnt[b, j] = rng.integers(0, cap[b, j] - free[b, j] + 1)
                busy_vals.append(rng.integers(0, 3_000_000, busy_cnt[b, j]).astype(np.int64))
    p.update(node_type=node_type.reshape(-1), node_cap=cap.reshape(-1), node_free=free.reshape(-1),
             node_backlog_us=backlog.reshape(-1), node_chunks=chunks.reshape(-1),
             gpu_mask_=gpu_mask.reshape(-1))     # free-GPU bit masks the chunk counts were derived from
    if busy:
        off = np.zeros(B * M + 1, np.int32)
        off[1:] = np.cumsum(busy_cnt.reshape(-1))
        p["node_busy_off"] = off
        p["node_busy_rel_us"] = (np.concatenate(busy_vals) if busy_vals else np.zeros(0, np.int64)).astype(np.int64)

    n = B * N
    present = [n_cpu > 0, n_gpu > 0, n_api > 0]
    probs = np.array([type_probs[0] * present[0], type_probs[1] * present[1], type_probs[2] * present[2]])
    t = rng.choice(3, size=n, p=probs / probs.sum()).astype(np.uint8)
    # few distinct base durations so that equal costs (ties) are common
    T = (rng.integers(1, 9, n) * (t_median // 4)).astype(np.int64)
    jitter = rng.random(n) < 0.5
    T[jitter] = _lognormal_us(rng, t_median, 1.0, int(jitter.sum()))
    model = np.zeros(n, np.uint8)
    param = np.zeros(n, np.uint32)
    kmask = rng.integers(1, 1 << K, n).astype(np.uint32)
    u = rng.random(n)
    c = t == TYPE_CPU
    model[c] = np.where(u[c] < 0.2, MODEL_NONE, np.where(u[c] < 0.8, MODEL_AMDAHL, MODEL_TABLE))
    g = t == TYPE_GPU
    model[g] = np.where(u[g] < 0.2, MODEL_NONE, MODEL_TABLE)
    am = model == MODEL_AMDAHL
    param[am] = rng.choice(np.array([0, 500_000, 750_000, 900_000, 1_000_000], np.uint32), int(am.sum()))
    tb = model == MODEL_TABLE
    param[tb] = rng.integers(0, len(CLASS_ALPHA), int(tb.sum()))
    kmask[g] &= (1 << kg) - 1
    kmask[g & (kmask == 0)] = 1
    kmask[t == TYPE_API] = 1
    pin = np.full(n, -1, np.int32)
    snap = np.repeat(np.arange(B), N)
    for i in range(n):
        ids = np.flatnonzero(node_type[snap[i]] == t[i])
        if t[i] == TYPE_API or rng.random() < pin_frac:
            pin[i] = ids[rng.integers(0, ids.size)]
    bad = rng.random(n) < bad_frac
    for i in np.flatnonzero(bad):
        r = rng.integers(0, 3)
        if r == 0:
            kmask[i] = 0                               # no allowed unit count
        elif r == 1 and t[i] != TYPE_API:
            pin[i] = rng.integers(0, M)                # pin that may name a node of another type
        elif t[i] == TYPE_CPU:
            kmask[i] = 1 << (K - 1)                    # only the largest unit count
    p.update(act_type=t, act_model=model, act_t_ori_us=T,
             act_age_us=(rng.integers(0, 5, n) * 100_000).astype(np.int64),
             act_kmask=kmask, act_param=param, act_pin_node=pin,
             act_task=rng.integers(0, 4, n).astype(np.int32))
    return p


def make_trace(S=4096, A=10_000, seed=4, contended=False, rate_per_s=50.0, horizon_s=200.0,
               tick_us=100_000, max_ticks=None, cluster=None, type_probs=(0.6, 0.2, 0.2),
               pin_frac=0.25, cpu_median=2_000_000):
    """Workload 5: S independent scenarios, each with A Poisson arrivals over ``horizon_s``.

    ``cluster`` = (n_cpu, cpu_cap, n_gpu, n_api); default is workload 3's cluster
    (256x128 cores, 32x8 GPUs, 16 quotas), ``contended`` shrinks it to 4x32 cores, 2x8 GPUs.
    """
    rng = np.random.default_rng(seed)
    if cluster is None:
        cluster = (4, 32, 2, 16) if contended else (256, 128, 32, 16)
    n_cpu, cpu_cap, n_gpu, n_api = cluster
    k_list = [1, 2, 4, 8, 16]
    p = _base(S, A, 0, k_list, [5, 4, 1 if n_api else 0])
    M, nt, cap, free, _, _, rate = _cluster(rng, S, n_cpu, cpu_cap, n_gpu, n_api)
    tp = np.array(type_probs, dtype=np.float64) * np.array([n_cpu > 0, n_gpu > 0, n_api > 0])
    p.update(B=S, N=A, M=M, node_type=nt, node_cap=cap, node_free=free,
             node_backlog_us=np.zeros(S * M, np.int64), node_chunks=np.zeros(S * M * 4, np.uint8))
    _actions(rng, p, tp / tp.sum(), pin_frac=pin_frac, cpu_median=cpu_median)
    gaps = rng.exponential(1e6 / rate_per_s, (S, A))
    arr = np.minimum(np.cumsum(gaps, axis=1), horizon_s * 1e6)
    t = dict(
        S=S, A=A, M=M, K=len(k_list), n_classes=p["n_classes"], depth=2,
        k_list=p["k_list"], type_k=p["type_k"], speedup_q16=p["speedup_q16"],
        node_type=nt, node_cap=cap, quota_rate=rate,
        quota_tok0_micro=(free.astype(np.int64) * 1_000_000) * (nt == TYPE_API),
        arrival_us=np.rint(arr).astype(np.int64).reshape(-1),
        act_type=p["act_type"], act_model=p["act_model"], act_t_ori_us=p["act_t_ori_us"],
        act_kmask=p["act_kmask"], act_param=p["act_param"], act_pin_node=p["act_pin_node"],
        tick_us=int(tick_us),
        max_ticks=int(max_ticks if max_ticks is not None else 4 * int(horizon_s * 1e6 / tick_us)),
    )
    return t


def slice_problem(p, snapshots):
    """The sub-problem made of the listed snapshots (for oracle checks on samples of a big batch)."""
    B, N, M = p["B"], p["N"], p["M"]
    snapshots = list(snapshots)
    q = dict(p)
    q["B"] = len(snapshots)
    for k in PROBLEM_ARRAYS + ("gpu_mask_", "node_aux_free", "act_aux", "act_service", "node_resident", "node_core_free", "act_quota_mask"):
        v = p.get(k)
        if v is None or k in ("k_list", "type_k", "speedup_q16", "node_busy_off", "node_busy_rel_us"):
            continue
        per = len(v) // B
        q[k] = np.concatenate([v[b * per:(b + 1) * per] for b in snapshots])
    if p.get("node_busy_off") is not None:
        off, rel = p["node_busy_off"], p["node_busy_rel_us"]
        cnt = np.concatenate([np.diff(off[b * M:(b + 1) * M + 1]) for b in snapshots])
        q["node_busy_off"] = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
        q["node_busy_rel_us"] = np.concatenate([rel[off[b * M]:off[(b + 1) * M]] for b in snapshots] + [np.zeros(0, np.int64)])
    return q


def with_core_maps(p, numa_cores, seed=0):
    """Adds the core topology of the CPU nodes to a problem (in place): cores in NUMA domains of
    ``numa_cores`` consecutive ids, and per node a random bitmap (4 x uint64) of its free cores with
    exactly ``node_free`` bits below ``node_cap``.  Other nodes get an empty map."""
    rng = np.random.default_rng(seed + 4242)
    m = p["B"] * p["M"]
    maps = np.zeros((m, 4), np.uint64)
    for j in np.flatnonzero(p["node_type"] == TYPE_CPU):
        cores = rng.choice(int(p["node_cap"][j]), int(p["node_free"][j]), replace=False)
        for c in cores:
            maps[j, c // 64] |= np.uint64(1) << np.uint64(c % 64)
    p["node_core_free"] = maps.reshape(-1)
    p["numa_cores"] = int(numa_cores)
    return p


def with_extra_quotas(p, frac=0.5, seed=0, max_extra=3):
    """Adds ``act_quota_mask`` to a problem or a trace (in place): a fraction of the API actions that are pinned to a quota
    also name up to ``max_extra`` other quotas of their snapshot (by rank among its API nodes, first 64 only)."""
    rng = np.random.default_rng(seed + 515)
    B, N, M = (p["B"], p["N"], p["M"]) if "B" in p else (p["S"], p["A"], p["M"])     # a problem or a trace
    mask = np.zeros(B * N, np.uint64)
    for b in range(B):
        api = np.flatnonzero(p["node_type"][b * M:(b + 1) * M] == TYPE_API)[:64]
        if len(api) < 2:
            continue
        rank = {int(j): r for r, j in enumerate(api)}
        for i in range(N):
            g = b * N + i
            pin = int(p["act_pin_node"][g])
            if p["act_type"][g] != TYPE_API or pin not in rank or rng.random() >= frac:
                continue
            others = [r for r in range(len(api)) if r != rank[pin]]
            for r in rng.choice(others, min(len(others), int(rng.integers(1, max_extra + 1))), replace=False):
                mask[g] |= np.uint64(1) << np.uint64(int(r))
    p["act_quota_mask"] = mask
    return p


def trace_with_aux(t, seed, scarce):
    """Adds a second resource to a trace (in place): what every node has of it and what an action holds of it."""
    rng = np.random.default_rng(seed + 5)
    t["act_aux"] = rng.integers(0, 40, t["S"] * t["A"]).astype(np.int32)
    t["node_aux"] = rng.integers(40 if scarce else 400, 120 if scarce else 4000, t["S"] * t["M"]).astype(np.int32)
    return t


def trace_with_services(t, seed, n_services, slots):
    """Adds services to a trace (in place): the service of every GPU action (-1: none), restore times, cache slots."""
    rng = np.random.default_rng(seed)
    sv = rng.integers(-1, n_services, t["S"] * t["A"]).astype(np.int32)
    sv[t["act_type"] != TYPE_GPU] = -1                         # services live on GPU nodes
    t["act_service"] = sv
    t["restore_us"] = (rng.integers(0, 9, n_services) * 150_000).astype(np.int64)
    t["cache_slots"] = slots
    return t


def random_trace(seed):
    """One small trace with cluster shape, load, tick limit, pins, depth, further quotas, services (cached per node or per GPU), the
    prefix rule, a second resource, named cores, the visiting order and pooled GPUs drawn at random from ``seed``."""
    rng = np.random.default_rng(seed)
    n_cpu, n_gpu, n_api = int(rng.integers(0, 6)), int(rng.integers(0, 4)), int(rng.integers(0, 4))
    if n_cpu + n_gpu + n_api == 0:
        n_cpu = 2
    probs = np.array([0.6 * (n_cpu > 0), 0.25 * (n_gpu > 0), 0.15 * (n_api > 0)])
    t = make_trace(S=int(rng.integers(1, 5)), A=int(rng.integers(1, 600)), seed=seed,
                   cluster=(n_cpu, int(rng.choice([4, 16, 48, 128])), n_gpu, n_api),
                   type_probs=tuple((probs / probs.sum()).tolist()),
                   rate_per_s=float(rng.choice([20.0, 100.0, 500.0])), horizon_s=float(rng.choice([1.0, 5.0, 20.0])),
                   max_ticks=int(rng.choice([60, 5000, 60000])), pin_frac=float(rng.choice([0.0, 0.3, 0.8])))
    t["depth"] = int(rng.integers(1, 5))
    if n_api >= 2 and rng.random() < 0.6:
        with_extra_quotas(t, frac=float(rng.random()), seed=seed, max_extra=int(rng.integers(1, 4)))
    if n_gpu and rng.random() < 0.6:
        trace_with_services(t, seed, n_services=int(rng.choice([1, 4, 20])), slots=int(rng.choice([1, 2, 5])))
    t["queue_prefix"] = int(rng.random() < 0.3)                # one prefix of the whole queue per step
    if rng.random() < 0.4:                                     # a second resource held by the actions that chose their node
        trace_with_aux(t, seed, scarce=bool(rng.integers(0, 2)))
    if rng.random() < 0.4:                                     # CPU actions get named cores
        t["numa_cores"] = int(rng.choice([4, 8, 16, 32, 64]))
    if rng.random() < 0.35:                                    # the queue visited by least estimated ACT
        t["order_policy"] = 1
    if n_gpu and rng.random() < 0.4 and t.get("act_service") is None and t.get("node_aux") is None:
        trace_with_pooled_gpus(t)                              # the GPU nodes as one pool of chunks
    if t.get("act_service") is not None and rng.random() < 0.5:
        t["cache_per_gpu"] = 1                                 # the cache of services on every GPU instead of the node
    return t


def trace_with_pooled_gpus(t):
    """Marks a trace (in place) as one whose GPU nodes are scheduled as one pool; GPU actions lose their pins."""
    t["act_pin_node"] = np.where(t["act_type"] == TYPE_GPU, -1, t["act_pin_node"]).astype(np.int32)
    t["gpu_pooled"] = 1
    return t


NODE_ARRAYS = ("node_type", "node_cap", "node_free", "node_backlog_us", "node_chunks", "node_aux_free", "node_resident",
               "node_core_free")


def with_shared_nodes(p):
    """Two views of one problem whose snapshots all see the node table of snapshot 0: ``(shared, expanded)``.
    ``shared`` carries the table once (``nodes_shared = 1``, node arrays of M entries), ``expanded`` carries B
    copies of it.  Pins move to a node of the action's own kind in that table where it has one."""
    B, N, M = p["B"], p["N"], p["M"]
    shared, expanded = dict(p), dict(p)
    for k in NODE_ARRAYS:
        v = p.get(k)
        if v is None:
            continue
        per = len(v) // B
        shared[k] = v[:per].copy()
        expanded[k] = np.tile(v[:per], B)
    if p.get("node_busy_off") is not None:
        off, rel = p["node_busy_off"], p["node_busy_rel_us"]
        per = int(off[M])
        shared["node_busy_off"] = off[:M + 1].copy()
        shared["node_busy_rel_us"] = rel[:per].copy()
        expanded["node_busy_off"] = np.concatenate([off[:M] + b * per for b in range(B)] + [[B * per]]).astype(np.int32)
        expanded["node_busy_rel_us"] = np.tile(rel[:per], B)
    nt = p["node_type"][:M]
    pin = p["act_pin_node"].copy()
    for g in np.flatnonzero(pin >= 0):
        own = np.flatnonzero(nt == p["act_type"][g])
        if len(own) and pin[g] < M:
            pin[g] = own[pin[g] % len(own)]
    shared["act_pin_node"] = pin
    expanded["act_pin_node"] = pin.copy()
    if p.get("act_quota_mask") is not None:                       # ranks among the API nodes of the old tables: drop
        shared["act_quota_mask"] = expanded["act_quota_mask"] = None
    shared["nodes_shared"] = 1
    return shared, expanded


def with_fixed_dop(t, k):
    """Copy of a trace (or problem) in which every elastic action may only run on exactly ``k`` units
    (the fixed degree-of-parallelism baselines of the paper's scheduler ablation); actions that do not
    allow ``k`` keep their own set."""
    q = {key: (v.copy() if isinstance(v, np.ndarray) else v) for key, v in t.items()}
    bit = np.uint32(1 << [int(x) for x in t["k_list"]].index(k))
    sel = (q["act_model"] != MODEL_NONE) & ((q["act_kmask"] & bit) != 0)
    q["act_kmask"][sel] = bit
    return q
