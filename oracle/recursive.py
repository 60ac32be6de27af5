"""Oracle for the recursive R2CCL-AllReduce: the peel plan, its alpha-beta time and the schedule.

TEST INFRASTRUCTURE ONLY.  Follows the R2CCL paper, Sec. 6 ("Recursive R2CCL-AllReduce": a global
ring at the slowest node's rate, then faster sub-rings peeled off one after the other, reductions
in parallel, broadcasts afterwards; an alpha-beta model picks the depth), built on the two-ring
analysis of Sec. 5.2.  The paper gives no pseudo-code for this part, so the concrete rules below
are this project's reading; they are chosen so that one degraded rank gives back exactly the
two-ring schedule of Sec. 5.2.  PARITY UNPINNED beyond: (1) that reduction to Sec. 5.2, (2) the
result equals a plain all-reduce up to the rounding order, (3) the structural invariants of the
plan (nested members, increasing bandwidth, shares sum to one).

The plan is computed with exact fractions; the schedule is composed from this package's own ring
and reduce-copy.  Nothing is shared with the product.
"""
from __future__ import annotations

from dataclasses import dataclass
from fractions import Fraction
from typing import List, Sequence

import numpy as np

from . import r2_oracle as o
from .split import _add, ring_factor


@dataclass
class Level:
    members: List[int]      # ranks in this level's ring, ascending
    fail_mask: int          # channels down at any member: the state the level's ring runs under
    bandwidth: int          # sum of the weights of the channels healthy under fail_mask
    increment: int          # bandwidth minus the previous level's (level 0: its bandwidth)
    share: Fraction         # fraction of the data this level's ring reduces


def own_bandwidth(weights: Sequence[int], mask: int) -> int:
    return sum(int(w) for c, w in enumerate(weights) if not (mask >> c) & 1)


def plan(weights: Sequence[int], fail_masks: Sequence[int], gpus_per_rank: int = 1,
         max_levels: int = 16) -> List[Level]:
    """Peel the slowest ranks off, level by level (Sec. 6).

    Level 0 is the ring over all ranks.  The next level drops every rank whose own remaining
    bandwidth is the smallest among the current members, as long as at least two ranks stay; a
    peel that does not raise the ring's bandwidth (the union of failed channels is unchanged) makes
    no level of its own, the peeling just goes on.  Shares make all rings finish together when
    latency is ignored: share_k is proportional to increment_k / ring_factor(participants_k),
    which for two levels is the balance point T1 = T2 of Sec. 5.2.
    """
    R = len(fail_masks)
    C = len(weights)
    full = (1 << C) - 1
    members = list(range(R))
    union = 0
    for m in fail_masks:
        union |= m & full
    bw = own_bandwidth(weights, union)
    if bw == 0:
        raise o.NoHealthyChannel(-2, "no channel is healthy at every rank")
    levels = [Level(list(members), union, bw, bw, Fraction(0))]
    while len(levels) < max_levels:
        own = {r: own_bandwidth(weights, fail_masks[r] & full) for r in members}
        lo = min(own.values())
        rest = [r for r in members if own[r] > lo]
        if len(rest) < 2:
            break
        members = rest
        union = 0
        for r in members:
            union |= fail_masks[r] & full
        bw = own_bandwidth(weights, union)
        if bw > levels[-1].bandwidth:
            levels.append(Level(list(members), union, bw, bw - levels[-1].bandwidth, Fraction(0)))
    wsum = Fraction(0)
    raw = []
    for lv in levels:
        raw.append(Fraction(lv.increment) / ring_factor(len(lv.members) * gpus_per_rank))
        wsum += raw[-1]
    for lv, x in zip(levels, raw):
        lv.share = x / wsum
    return levels


def hops(n_ranks: int, n_members: int) -> int:
    """Links the broadcast of one level crosses, one after the other: along the excluded ranks,
    into the ring, along the ring, back out, and along the excluded ranks again."""
    m = n_ranks - n_members
    return n_members + 2 * m - 1


def completion_time(levels: Sequence[Level], n_ranks: int, gpus_per_rank: int, nbytes, alpha, beta):
    """alpha-beta time of the plan: all reductions run in parallel, each on its own increment of
    bandwidth; then the broadcasts of the levels above 0 run in parallel, each at its own
    increment.  ``beta`` is bytes per second per unit of weight.  With alpha = 0 and two levels this
    is T(Y) = max(T1, T2) + T3 of Sec. 5.2."""
    red, bc = [], [0]
    for k, lv in enumerate(levels):
        p = len(lv.members) * gpus_per_rank
        t = lv.share * nbytes / (lv.increment * beta)
        red.append(2 * (p - 1) * alpha + ring_factor(p) * t)
        if k:
            bc.append(hops(n_ranks, len(lv.members)) * alpha + t)
    return max(red) + max(bc)


def select_depth(weights, fail_masks, gpus_per_rank, nbytes, alpha, beta, max_levels: int = 16):
    """Depth (number of levels minus one) with the smallest modelled time; depth 0 is the single
    balanced ring (R2CCL-Balance).  Ties go to the shallower plan."""
    full = plan(weights, fail_masks, gpus_per_rank, max_levels)
    times = []
    for depth in range(len(full)):
        lv = plan(weights, fail_masks, gpus_per_rank, depth + 1)
        times.append(completion_time(lv, len(fail_masks), gpus_per_rank, nbytes, alpha, beta))
    best = min(range(len(times)), key=lambda i: (times[i], i))
    return best, times


def segments(levels: Sequence[Level], n_ranks: int, n_elems: int, n_slabs: int, elem_bytes: int) -> List[int]:
    """Elements per level: every level above 0 gets its share of the buffer, rounded down to what
    both its own ring and the global ring can divide into whole 16-byte vectors; level 0 the rest."""
    from math import gcd

    per16 = 16 // elem_bytes
    assert n_elems % (n_slabs * n_ranks * per16) == 0
    out = [0] * len(levels)
    for k in range(len(levels) - 1, 0, -1):
        p = len(levels[k].members)
        granule = n_slabs * (p * n_ranks // gcd(p, n_ranks)) * per16
        out[k] = int(levels[k].share * n_elems) // granule * granule
    out[0] = n_elems - sum(out)
    return out


# ------------------------------------------------------------------ schedule

def chain_order(n_ranks: int, members: Sequence[int]):
    """Excluded ranks ascending; members in ring order starting after the last excluded rank."""
    mem = set(members)
    excl = [r for r in range(n_ranks) if r not in mem]
    if not excl:
        return [], list(members)
    start = excl[-1]
    order = [(start + 1 + i) % n_ranks for i in range(n_ranks)]
    return excl, [r for r in order if r in mem]


def recursive_expected(inputs: Sequence[np.ndarray], dtype: int, levels: Sequence[Level],
                       level_elems: Sequence[int], n_slabs: int) -> List[np.ndarray]:
    """What every rank must hold afterwards, by definition: per level's segment, the ring
    all-reduce of the members (in chain order) plus the running sum of the excluded ranks (in
    ascending order), every addition rounded to the buffer type."""
    R = len(inputs)
    outs = [x.copy() for x in inputs]
    lo = 0
    for lv, n in zip(levels, level_elems):
        hi = lo + n
        if n:
            excl, order = chain_order(R, lv.members)
            seg = o.expected([np.ascontiguousarray(inputs[r][lo:hi]) for r in order], dtype, n_slabs, o.PHASE_AR)[0]
            if excl:
                acc = np.ascontiguousarray(inputs[excl[0]][lo:hi])
                for r in excl[1:]:
                    acc = _add(np.ascontiguousarray(inputs[r][lo:hi]), acc, dtype)
                seg = _add(seg, acc, dtype)
            for r in range(R):
                outs[r][lo:hi] = seg
        lo = hi
    assert lo == inputs[0].size
    return outs


def recursive_sim(bufs: Sequence[np.ndarray], dtype: int, levels: Sequence[Level],
                  level_elems: Sequence[int], n_slabs: int, n_channels: int, align: int,
                  weights: Sequence[int], fail_masks: Sequence[int]):
    """The schedule step by step, in place on ``bufs``: for every level the ring over its members
    on its segment under the level's channel state, then, for the levels above 0, the broadcast
    chain.  A link between two ranks is cut by the union of their failed channels.

    Returns, per level, ``None`` (no chain) or ``(chain, tables[len(chain)-1, C+1], stage)`` with
    the ranks in the order the data visits them, the table of every link and the two stage
    parities (C buffers each) as the chain left them."""
    R = len(bufs)
    es = bufs[0].itemsize
    lo = 0
    trace = []
    for lv, n in zip(levels, level_elems):
        hi = lo + n
        trace.append(None)
        if n == 0:
            continue
        excl, order = chain_order(R, lv.members)
        segs = {r: np.ascontiguousarray(bufs[r][lo:hi]) for r in range(R)}
        o.ring_sim([segs[r] for r in order], dtype, n_slabs, n_channels, align,
                   [(0, lv.fail_mask, weights)], o.PHASE_AR)
        if excl:
            nbytes = n * es
            cap = (nbytes + 255) // 256 * 256
            stage = [[np.full(cap, 0xA5, np.uint8) for _ in range(n_channels)] for _ in range(2)]
            chain = excl + order + excl      # every rank the data visits, in order
            m, p = len(excl), len(order)

            def table(u, v):
                return o.partition(weights, fail_masks[u] | fail_masks[v], nbytes, align)

            tables = np.stack([table(chain[i], chain[i + 1]) for i in range(len(chain) - 1)])
            trace[-1] = (chain, tables, stage)
            for i, r in enumerate(chain):
                t_in = tables[i - 1] if i else None
                t_out = tables[i] if i + 1 < len(chain) else None
                s_in = stage[(i + 1) & 1] if i else None
                s_out = stage[i & 1] if i + 1 < len(chain) else None
                if i < m:                     # excluded ranks add themselves up
                    op = o.OP_SUM
                elif i < m + p - 1:           # members add the sum to their result, relay it unchanged
                    op = o.OP_SUM_FORWARD
                elif i == m + p - 1:          # the last member sends its finished result on
                    op = o.OP_SUM
                else:                         # excluded ranks take the result and pass it on
                    op = o.OP_COPY
                o.reduce_copy(segs[r], dtype, op, s_in, t_in, s_out, t_out, n_channels, cap)
        for r in range(R):
            bufs[r][lo:hi] = segs[r]
        lo = hi
    assert lo == bufs[0].size
    return trace
