"""Oracle for the recursive R2CCL-AllReduce: the peel plan, its alpha-beta time and the schedule.

TEST INFRASTRUCTURE ONLY.  Follows the R2CCL paper, Sec. 6 ("Recursive R2CCL-AllReduce": a global
ring at the slowest node's rate, then faster sub-rings peeled off one after the other, each handling
data in proportion to the bandwidth it adds, logical re-ranking applied at every level, reductions in
parallel, broadcasts afterwards; an alpha-beta model picks the depth), built on the two-ring analysis
of Sec. 5.2 and on "Topology-Aware Logical Re-ranking" (Sec. 6, Appendix D Algorithm 1).  The paper
gives no pseudo-code for this part, so the concrete rules below are this project's reading; they are
chosen so that one degraded rank gives back exactly the two-ring schedule of Sec. 5.2.

What pins it: (1) that reduction to Sec. 5.2 (shares, time, bits); (2) the result equals a plain
all-reduce up to the rounding order; (3) the shares minimise the modelled completion time, which is
checked by brute force over a grid of share vectors; (4) every level's ring runs at the bandwidth of its
narrowest link after re-ranking, never below the rails its members all share; (5) the structural
invariants of the plan (nested members, growing bandwidth, shares sum to one).  PARITY UNPINNED: the
peel rule (which ranks leave together), the order of the broadcast chain and its relay rule.

The plan is computed with exact fractions; the schedule is composed from this package's own ring
with per-link tables, re-ranking and reduce-copy.  Nothing is shared with the product.
"""
from __future__ import annotations

from dataclasses import dataclass
from fractions import Fraction
from typing import List, Sequence

import numpy as np

from . import r2_oracle as o
from . import rails as rl
from .rerank import bridge_rerank
from .split import _add, ring_factor


@dataclass
class Level:
    members: List[int]      # ranks in this level's ring, ascending
    fail_mask: int          # channels down at any member (informational: the ring runs link by link)
    bandwidth: int          # the ring's bandwidth: that of its narrowest link, in its re-ranked order
    increment: int          # bandwidth minus the previous level's (level 0: its bandwidth)
    share: Fraction         # fraction of the data this level's ring reduces
    order: List[int]        # the members in the order the ring visits them


def own_bandwidth(weights: Sequence[int], mask: int) -> int:
    return sum(int(w) for c, w in enumerate(weights) if not (mask >> c) & 1)


def ring_order(n_ranks: int, n_channels: int, fail_masks: Sequence[int], members: Sequence[int]) -> List[int]:
    """A level's ring: its members in rank order, starting after the highest-numbered rank that is
    left out (level 0: from rank 0), then re-ranked (Sec. 6: re-ranking at every level, because
    skipping the slower nodes puts nodes next to each other that lost different rails)."""
    mem = set(members)
    excl = [r for r in range(n_ranks) if r not in mem]
    start = excl[-1] + 1 if excl else 0
    base = [(start + i) % n_ranks for i in range(n_ranks) if (start + i) % n_ranks in mem]
    rails = {r: {c for c in range(n_channels) if not (fail_masks[r] >> c) & 1} for r in base}
    return bridge_rerank(base, rails)[0]


def level_bandwidth(weights: Sequence[int], fail_masks: Sequence[int], order: Sequence[int]) -> int:
    """A ring moves data at the rate of its narrowest link; a link carries what both ends still have."""
    return rl.ring_bandwidth(weights, [fail_masks[r] for r in order])


def optimal_shares(increments: Sequence[int], participants: Sequence[int]) -> List[Fraction]:
    """Shares that minimise the completion time with latency ignored, given that every level is used.

    With u_k = share_k / increment_k (the time level k needs per unit of ring factor) the time is
    max_k f_k u_k + max_{k>=1} u_k, f_k = 2(p_k - 1)/p_k, the generalisation of T(Y) = max(T1, T2) + T3
    of Sec. 5.2.  It is piecewise linear in the shares, so its minimum over the simplex lies where the
    lower levels' rings finish together and the levels from some j on have one and the same u (their
    shares are then exactly proportional to the bandwidth they add, the paper's wording): u_k = tau/f_k
    for k <= j, u_k = tau/f_j for k >= j.  The best j is found by trying them all; ties go to the
    smallest.  For two levels this is the balance point T1 = T2."""
    L = len(increments)
    if L == 1:
        return [Fraction(1)]
    f = [ring_factor(p) for p in participants]
    best = None
    for j in range(1, L):
        u = [1 / f[k] if k <= j else 1 / f[j] for k in range(L)]        # in units of tau
        tau = 1 / sum(Fraction(increments[k]) * u[k] for k in range(L))
        t = tau * (1 + 1 / f[j])
        if best is None or t < best[0]:
            best = (t, [Fraction(increments[k]) * u[k] * tau for k in range(L)])
    return best[1]


def plan(weights: Sequence[int], fail_masks: Sequence[int], gpus_per_rank: int = 1,
         max_levels: int = 16) -> List[Level]:
    """Peel the slowest ranks off, level by level (Sec. 6).

    Level 0 is the ring over all ranks.  The next level drops every rank whose own remaining
    bandwidth is the smallest among the current members, as long as at least two ranks stay.  Every
    level's ring is re-ranked and runs link by link; its bandwidth is its narrowest link's.  A peel
    that does not raise the bandwidth makes no level of its own, the peeling just goes on.
    """
    R = len(fail_masks)
    C = len(weights)
    full = (1 << C) - 1
    masks = [m & full for m in fail_masks]

    def level(members, prev_bw):
        order = ring_order(R, C, masks, members)
        union = 0
        for r in members:
            union |= masks[r]
        bw = level_bandwidth(weights, masks, order)
        return Level(list(members), union, bw, bw - prev_bw, Fraction(0), order)

    members = list(range(R))
    levels = [level(members, 0)]
    if levels[0].bandwidth == 0:
        raise o.NoHealthyChannel(-2, "a link of the global ring is left without a channel")
    while len(levels) < max_levels:
        own = {r: own_bandwidth(weights, masks[r]) for r in members}
        lo = min(own.values())
        rest = [r for r in members if own[r] > lo]
        if len(rest) < 2:
            break
        members = rest
        cand = level(members, levels[-1].bandwidth)
        if cand.increment > 0:
            levels.append(cand)
    shares = optimal_shares([lv.increment for lv in levels], [len(lv.members) * gpus_per_rank for lv in levels])
    for lv, x in zip(levels, shares):
        lv.share = x
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

def excluded_of(n_ranks: int, members: Sequence[int]) -> List[int]:
    mem = set(members)
    return [r for r in range(n_ranks) if r not in mem]


def chain_visits(n_ranks: int, n_channels: int, fail_masks: Sequence[int], level: Level):
    """The ranks a level's broadcast visits, in order, as (rank, role) pairs.

    The ranks left out add their segments up one after the other in ascending order ("gather"); the
    sum then goes round the ring's members in the ring's order, each adding it to its ring result and
    passing it on unchanged ("member"; the last one passes its finished result on instead); the ranks
    left out take the result in ascending order ("take").  Where two consecutive ranks of that walk
    have no channel in common -- they lost complementary rails -- the hop goes through a third rank
    that has a channel in common with both and forwards the data untouched ("relay"): the first such
    rank among the ring's members in ring order, then among the ranks left out in ascending order.
    No such rank: NoHealthyChannel."""
    full = (1 << n_channels) - 1
    excl = excluded_of(n_ranks, level.members)
    if not excl:
        return []
    walk = [(r, "gather") for r in excl] + [(r, "member") for r in level.order] + [(r, "take") for r in excl]

    def linked(a, b):
        return ((fail_masks[a] | fail_masks[b]) & full) != full

    visits = [walk[0]]
    for nxt in walk[1:]:
        u, v = visits[-1][0], nxt[0]
        if not linked(u, v):
            for w in list(level.order) + excl:
                if w not in (u, v) and linked(u, w) and linked(w, v):
                    visits.append((w, "relay"))
                    break
            else:
                raise o.NoHealthyChannel(-2, f"no path from rank {u} to rank {v}")
        visits.append(nxt)
    return visits


def recursive_expected(inputs: Sequence[np.ndarray], dtype: int, levels: Sequence[Level],
                       level_elems: Sequence[int], n_slabs: int) -> List[np.ndarray]:
    """What every rank must hold afterwards, by definition: per level's segment, the ring
    all-reduce of the members (in the ring's order) plus the running sum of the excluded ranks (in
    ascending order), every addition rounded to the buffer type."""
    R = len(inputs)
    outs = [x.copy() for x in inputs]
    lo = 0
    for lv, n in zip(levels, level_elems):
        hi = lo + n
        if n:
            excl = excluded_of(R, lv.members)
            seg = o.expected([np.ascontiguousarray(inputs[r][lo:hi]) for r in lv.order], dtype, n_slabs, o.PHASE_AR)[0]
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
    """The schedule step by step, in place on ``bufs``: for every level the ring over its members, in
    the level's order and link by link (a link carries what both its ends still have), on its
    segment; then, for the levels above 0, the broadcast chain.  A link between two ranks is cut by the
    union of their failed channels.

    Returns, per level, ``None`` (no data) or ``(ring_tables, visits, tables, stage)``: the ring's
    per-link tables [p, S*(J-1), C+1]; for levels with a chain the (rank, role) pairs in the order the
    data visits them, the table of every hop and the two stage parities (C buffers each) as the
    chain left them (``None`` each for level 0)."""
    R = len(bufs)
    es = bufs[0].itemsize
    lo = 0
    trace = []
    for lv, n in zip(levels, level_elems):
        hi = lo + n
        trace.append(None)
        if n == 0:
            continue
        segs = {r: np.ascontiguousarray(bufs[r][lo:hi]) for r in range(R)}
        ring_tables, _ = rl.ring_rails_sim([segs[r] for r in lv.order], dtype, n_slabs, n_channels, align,
                                           rl.static_epochs(weights, [fail_masks[r] for r in lv.order]), o.PHASE_AR)
        visits = chain_visits(R, n_channels, fail_masks, lv)
        trace[-1] = (ring_tables, None, None, None)
        if visits:
            nbytes = n * es
            cap = (nbytes + 255) // 256 * 256
            stage = [[np.full(cap, 0xA5, np.uint8) for _ in range(n_channels)] for _ in range(2)]
            tables = np.stack([o.partition(weights, fail_masks[visits[i][0]] | fail_masks[visits[i + 1][0]], nbytes, align)
                               for i in range(len(visits) - 1)])
            trace[-1] = (ring_tables, visits, tables, stage)
            last_member = max(i for i, (_, role) in enumerate(visits) if role == "member")
            for i, (r, role) in enumerate(visits):
                t_in = tables[i - 1] if i else None
                t_out = tables[i] if i + 1 < len(visits) else None
                s_in = stage[(i + 1) & 1] if i else None
                s_out = stage[i & 1] if i + 1 < len(visits) else None
                local = segs[r]
                if role == "gather":          # the ranks left out add themselves up
                    op = o.OP_SUM
                elif role == "member":        # members add the sum to their result and relay it unchanged;
                    op = o.OP_SUM if i == last_member else o.OP_SUM_FORWARD   # the last sends its result on
                elif role == "take":          # the ranks left out take the result and pass it on
                    op = o.OP_COPY
                else:                         # a relay forwards what it gets; its own data is not involved
                    op = o.OP_COPY
                    local = np.empty_like(segs[r])
                o.reduce_copy(local, dtype, op, s_in, t_in, s_out, t_out, n_channels, cap)
        for r in range(R):
            bufs[r][lo:hi] = segs[r]
        lo = hi
    assert lo == bufs[0].size
    return trace
