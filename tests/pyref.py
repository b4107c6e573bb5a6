"""Independent, slow Python restatements used only to pin the CPU oracle.

Nothing here is shared with oracle/ or with the HIP library: durations use exact
rationals, the completion heap uses heapq, the dynamic programs are replaced by
exhaustive enumeration, and GPU chunks are simulated on real addresses.
"""
from __future__ import annotations

import heapq
import itertools
from fractions import Fraction

INF = (1 << 63) - 1


def duration(model, T, param, k, speedup=0):
    """Eq. 1 of the paper with E(k) from the Amdahl fraction or the fixed-point table, rounded up."""
    if model == 0:
        return T
    if model == 1:
        p = Fraction(param, 10**6)
        e = 1 / ((1 - p) * k + p)                  # E(k) in (0, 1]
    else:
        e = Fraction(speedup, 65536) / k           # E(k) k = speedup / 65536
    d = Fraction(T) / (e * k)
    c = -((-d.numerator) // d.denominator)
    return max(1, c)


def estimate(heap, ac, depth):
    """ac: list of option lists [(k, dur), ...] ascending in k.  Per-unit completion heap."""
    H = len(heap)
    ac = [[(k, d) for (k, d) in o if k <= H] for o in ac]
    ac = [o for o in ac if o]
    if not ac:
        return 0
    best = None
    for d in range(1, depth + 1):
        if len(ac[0]) < d:
            break
        h = list(heap)
        heapq.heapify(h)
        obj = 0
        for x, o in enumerate(ac):
            k, dur = o[d - 1] if x == 0 else o[0]
            popped = [heapq.heappop(h) for _ in range(k)]
            fin = max(popped) + dur
            for _ in range(k):
                heapq.heappush(h, fin)
            obj += fin
        best = obj if best is None else min(best, obj)
    return best


def best_units_exhaustive(opts, U):
    """min sum of durations over every unit vector with sum <= U.  opts[i] = [(k, dur), ...]."""
    best = None
    for combo in itertools.product(*opts):
        if sum(k for k, _ in combo) <= U:
            v = sum(d for _, d in combo)
            if best is None or v < best:
                best = v
    return best


class Buddy:
    """8-GPU buddy allocator on addresses (Sec. 5.3): best fit, lowest address, split down."""

    def __init__(self, free_mask=0xFF):
        self.mask = free_mask

    def chunks(self):
        out = []                                   # (start, size) of maximal aligned free blocks
        for lvl in (3, 2, 1, 0):
            sz = 1 << lvl
            for s in range(0, 8, sz):
                blk = ((1 << sz) - 1) << s
                if self.mask & blk != blk:
                    continue
                if any(s >= ps and s + sz <= ps + psz for ps, psz in out):
                    continue
                out.append((s, sz))
        return out

    def counts(self):
        c = [0, 0, 0, 0]
        for _, sz in self.chunks():
            c[sz.bit_length() - 1] += 1
        return tuple(c)

    def alloc(self, k):
        size = 1
        while size < k:
            size *= 2
        cands = sorted((sz, s) for s, sz in self.chunks() if sz >= size)
        if not cands:
            return None
        sz, s = cands[0]
        self.mask &= ~(((1 << size) - 1) << s)
        return s

    def free(self, s, k):
        size = 1
        while size < k:
            size *= 2
        self.mask |= ((1 << size) - 1) << s


class BuddyCluster:
    """Several 8-GPU nodes behind one allocator: the smallest free chunk of the cluster that is large
    enough, on the lowest-numbered node that has one, lowest address there."""

    def __init__(self, masks):
        self.nodes = [Buddy(m) for m in masks]

    def counts(self):
        return tuple(sum(c) for c in zip(*[b.counts() for b in self.nodes])) if self.nodes else (0, 0, 0, 0)

    def alloc(self, k):
        size = 1
        while size < k:
            size *= 2
        cands = sorted((sz, j, s) for j, b in enumerate(self.nodes) for s, sz in b.chunks() if sz >= size)
        if not cands:
            return None
        sz, j, s = cands[0]
        self.nodes[j].mask &= ~(((1 << size) - 1) << s)
        return j, s


def best_chunks_exhaustive(opts, mask):
    """min sum of durations over unit vectors that a buddy allocator can serve in order."""
    best = None
    for combo in itertools.product(*opts):
        b = Buddy(mask)
        if all(b.alloc(k) is not None for k, _ in combo):
            v = sum(d for _, d in combo)
            if best is None or v < best:
                best = v
    return best
