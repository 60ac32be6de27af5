"""Recursive R2CCL-AllReduce (Sec. 6): pins for the oracle's plan, time model and schedule, and parity
of the product's host planner against it.  No GPU involved.

What the paper and the mathematics fix, and what therefore pins this part: one degraded server must
give the two-ring schedule and T(Y) of Sec. 5.2; the result must be an all-reduce; the levels are
nested rings of growing bandwidth, re-ranked at every level, each running at its narrowest link's
rate; the shares minimise the modelled completion time (brute force over a grid of share vectors)
and, from some level on, are exactly proportional to the bandwidth each level adds.  The rest is this
project's reading (the paper has no pseudo-code here) and is listed as such in the oracle's header."""
from fractions import Fraction as F

import numpy as np
import pytest

import oracle as o
from oracle import recursive as rec
from oracle import split as sp


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg
    from paper_2512_25059_amd import build as hip_build

    if hip_build.is_stale():
        hip_build.build()
    pkg.load_library()
    return pkg


EQ8 = [50000] * 8


def _rand_case(rng):
    R = int(rng.integers(2, 12))
    C = int(rng.integers(1, 9))
    w = [int(x) for x in rng.integers(1, 1000, C)]
    masks = []
    for _ in range(R):
        m = 0
        if rng.random() < 0.6:
            for c in range(C):
                if rng.random() < 0.3:
                    m |= 1 << c
        masks.append(m)
    return R, C, w, masks


# ------------------------------------------------------------------ plan

def test_worked_example_by_hand():
    """Four servers with eight equal NICs; server 0 lost four, server 1 two of those.  Rings: all four
    at 4 NICs, {1,2,3} at 6 (adds 2), {2,3} at 8 (adds 2); no neighbours lost different rails, so no
    ring is re-ranked.  Ring factors 3/2, 4/3, 1.  With the two lower rings finishing together and the
    two upper levels taking data in proportion to what they add (u1 = u2): shares 2/(3/2) : 1/(4/3) :
    1/(4/3) = 16 : 9 : 9, time (1 + 3/4) / (17/6) = 21/34 of D/(100000 beta).  With all three rings
    finishing together instead (16 : 9 : 12) it is 2 / (37/12) = 24/37, which is more."""
    lv = rec.plan(EQ8, [0b1111, 0b0011, 0, 0])
    assert [l.members for l in lv] == [[0, 1, 2, 3], [1, 2, 3], [2, 3]]
    assert [l.order for l in lv] == [[0, 1, 2, 3], [1, 2, 3], [2, 3]]
    assert [l.fail_mask for l in lv] == [0b1111, 0b0011, 0]
    assert [l.bandwidth for l in lv] == [200000, 300000, 400000]
    assert [l.increment for l in lv] == [200000, 100000, 100000]
    assert [l.share for l in lv] == [F(16, 34), F(9, 34), F(9, 34)]
    assert rec.completion_time(lv, 4, 1, 1, 0, F(1, 100000)) == F(21, 34)
    for l, x in zip(lv, (F(16, 37), F(9, 37), F(12, 37))):
        l.share = x
    assert rec.completion_time(lv, 4, 1, 1, 0, F(1, 100000)) == F(24, 37) > F(21, 34)


def test_top_ring_adds_most_by_hand():
    """Eight servers with eight equal NICs: one kept a single NIC, five kept two (that one among them),
    two kept all eight.  Rings: all eight at 1 NIC, seven at 2 (adds 1), two at 8 (adds 6); ring factors
    7/4, 12/7, 1.  Here it pays to let all three rings finish together (u_k = tau/f_k): shares
    1*(4/7) : 1*(7/12) : 6*1 = 48 : 49 : 504, time 2 / (601/84) = 168/601 of D/(50000 beta).  Giving the two
    upper levels data in proportion to what they add (u_1 = u_2 = tau*7/12) costs (1 + 7/12) / (391/84) =
    133/391, a fifth more: which levels share one u is found by trying, not fixed."""
    masks = [0b01111111] + [0b00111111] * 5 + [0, 0]
    lv = rec.plan(EQ8, masks)
    assert [l.members for l in lv] == [list(range(8)), list(range(1, 8)), [6, 7]]
    assert [l.increment for l in lv] == [50000, 50000, 300000]
    assert [l.share for l in lv] == [F(48, 601), F(49, 601), F(504, 601)]
    assert rec.completion_time(lv, 8, 1, 1, 0, F(1, 50000)) == F(168, 601)
    for l, x in zip(lv, (F(48, 391), F(49, 391), F(294, 391))):
        l.share = x
    assert rec.completion_time(lv, 8, 1, 1, 0, F(1, 50000)) == F(133, 391) > F(168, 601)


def test_share_tie_goes_to_exact_proportion_by_hand():
    """Increments 3 : 4 : 4 on rings of 10, 7 and 6 participants (ring factors 9/5, 12/7, 5/3).  Two share
    vectors reach the minimal time 1/4: 5 : 7 : 7 of 19 (the two lower rings finish together, both upper
    levels take data in exact proportion to what they add) and 25 : 35 : 36 of 96 (all three rings
    finish together).  The rule takes the first: as many levels as possible in the paper's proportion."""
    inc, parts = (3, 4, 4), (10, 7, 6)
    assert _time_of(inc, parts, [F(5, 19), F(7, 19), F(7, 19)]) == F(1, 4)
    assert _time_of(inc, parts, [F(25, 96), F(35, 96), F(36, 96)]) == F(1, 4)
    assert rec.optimal_shares(inc, parts) == [F(5, 19), F(7, 19), F(7, 19)]


def _time_of(increments, participants, shares):
    """The completion time by its definition (latency ignored, D = beta = 1), written out again here:
    the slowest ring, then the slowest broadcast."""
    ring = max(F(2 * (p - 1), p) * s / inc for inc, p, s in zip(increments, participants, shares))
    bcast = max([s / inc for inc, s in list(zip(increments, shares))[1:]] + [F(0)])
    return ring + bcast


@pytest.mark.parametrize("increments,participants", [
    ((2, 1, 1), (4, 3, 2)),            # the worked example
    ((4, 2, 1, 1), (8, 7, 6, 5)),      # eight servers that lost 4 / 2 / 1 NICs
    ((1, 3, 2), (6, 4, 2)),            # a slow global ring under fast upper ones
    ((5, 1, 1), (16, 12, 8)),          # little to gain: X = 2/7 is below the two-ring threshold
    ((3, 3), (5, 4)),                  # two levels: the balance point of Sec. 5.2
    ((1, 1, 6), (8, 7, 2)),            # the top ring adds most: all three rings finish together (j = 2)
    ((1, 1, 4, 1), (8, 7, 3, 2)),      # four levels, the lower three finish together (j = 2)
    ((1, 1, 1, 4), (9, 8, 7, 2)),      # four levels, all four finish together (j = 3)
    ((3, 4, 4), (10, 7, 6)),           # a tie: two share vectors reach the minimum
])
def test_shares_minimise_the_modelled_time_brute_force(increments, participants):
    """Every share vector on a grid of the simplex (steps of 1/120; levels above 0 may also get nothing)
    is at least as slow as the planner's, unless it gives up the upper levels so far that the plain
    balanced ring -- depth 0, the selector's business, not the share rule's -- is what wins."""
    import itertools

    L = len(increments)
    shares = rec.optimal_shares(increments, participants)
    assert sum(shares) == 1 and all(x > 0 for x in shares)
    best = _time_of(increments, participants, shares)
    single = F(2 * (participants[0] - 1), participants[0]) / increments[0]   # everything on level 0
    steps = 120 if L <= 3 else 40
    grid_best = None
    for combo in itertools.product(range(steps + 1), repeat=L - 1):
        if sum(combo) > steps:
            continue
        cand = [F(steps - sum(combo), steps)] + [F(c, steps) for c in combo]
        t = _time_of(increments, participants, cand)
        grid_best = t if grid_best is None else min(grid_best, t)
        assert t >= min(best, single), cand
    # the grid comes close to the planner's optimum (or to the single ring where that is better)
    assert grid_best - min(best, single) <= F(1, 25) * min(best, single)
    # and from some level on the shares are exactly proportional to what the levels add (Sec. 6)
    u = [x / inc for x, inc in zip(shares, increments)]
    assert any(all(u[k] == u[j] for k in range(j, L)) for j in range(1, L))
    assert all(a <= b for a, b in zip(u, u[1:]))


def test_shares_for_two_levels_are_the_balance_point():
    for n, g, lost in ((4, 1, 3), (8, 2, 4), (16, 8, 6)):
        X = F(lost, 8)
        shares = rec.optimal_shares([8 - lost, lost], [n * g, (n - 1) * g])
        assert shares[1] == sp.balance_point(n, g, X)


def test_reranking_at_every_level_by_hand():
    """Six servers, eight equal NICs.  Server 0 lost NICs 0-3, server 1 lost NICs 4-7: as neighbours they
    share nothing, and no rail is up at all six servers -- a single table for the whole ring would have
    no channel.  Re-ranked, server 2 (all NICs) stands between them: links 0-2 and 2-1 carry 4 NICs, the
    others 4 or 8: the global ring runs at 4, the slowest server's own rate.  The ring of the four
    healthy servers adds 4.  Shares: 4/(5/3) : 4/(3/2) = 9 : 10.
    The broadcast of the upper level walks 0, 1, then the ring 2 3 4 5, then 0, 1 again; the hops 0 -> 1
    have no channel, so each goes through server 2, the first ring member linked to both."""
    masks = [0b00001111, 0b11110000, 0, 0, 0, 0]
    lv = rec.plan([1] * 8, masks)
    assert [l.members for l in lv] == [[0, 1, 2, 3, 4, 5], [2, 3, 4, 5]]
    assert lv[0].order == [0, 2, 1, 3, 4, 5] and lv[1].order == [2, 3, 4, 5]
    assert [l.bandwidth for l in lv] == [4, 8] and [l.share for l in lv] == [F(9, 19), F(10, 19)]
    assert rec.chain_visits(6, 8, masks, lv[0]) == []
    assert rec.chain_visits(6, 8, masks, lv[1]) == [
        (0, "gather"), (2, "relay"), (1, "gather"), (2, "member"), (3, "member"), (4, "member"), (5, "member"),
        (0, "take"), (2, "relay"), (1, "take")]
    # three servers: in a ring of three everybody is everybody's neighbour, so the two that share nothing
    # cannot be separated and the ring cannot run
    with pytest.raises(o.NoHealthyChannel):
        rec.plan([1] * 8, [0b00001111, 0b11110000, 0b01111110])


def test_no_failure_is_one_ring():
    lv = rec.plan(EQ8, [0] * 6)
    assert len(lv) == 1 and lv[0].share == 1 and lv[0].members == list(range(6))
    # and its time is the ring all-reduce time of Sec. 5.2: 2(n-1)/n * D/B
    assert rec.completion_time(lv, 6, 1, 1000, 0, F(1, 400000)) == F(2 * 5, 6) * 1000


@pytest.mark.parametrize("n,g,lost", [(4, 1, 1), (8, 1, 4), (8, 8, 2), (16, 4, 7), (3, 2, 5)])
def test_one_degraded_server_is_the_two_ring_schedule(n, g, lost):
    """Sec. 5.2: global ring at (1-X)B with share 1-Y, partial ring at XB with share Y, where Y makes
    T1 = T2; and the modelled time is T(Y) = max(T1, T2) + T3."""
    masks = [0] * n
    masks[n // 2] = (1 << lost) - 1
    lv = rec.plan(EQ8, masks, g)
    X = F(lost, 8)
    assert len(lv) == 2
    assert lv[1].members == [r for r in range(n) if r != n // 2]
    assert F(lv[1].increment, lv[1].bandwidth) == X
    assert lv[1].share == sp.balance_point(n, g, X)
    # B = 400000 weight units, beta = 1/B bytes per second per unit, D = 1: the units of Sec. 5.2
    assert rec.completion_time(lv, n, g, 1, 0, F(1, 400000)) == sp.completion_time(n, g, X, lv[1].share)


def test_shares_follow_the_incremental_bandwidth():
    """Sec. 6: a ring's share is proportional to the bandwidth it adds.  The ring factor 2(p-1)/p
    tends to 2 for many GPUs per server, and the shares then tend to increment / top bandwidth."""
    masks = [0b111111, 0b1111, 0b1, 0, 0]
    lv = rec.plan(EQ8, masks, gpus_per_rank=10 ** 6)
    top = lv[-1].bandwidth
    for l in lv:
        assert abs(float(l.share) - l.increment / top) < 1e-5


def test_plan_invariants_random():
    from oracle import rails as rl

    rng = np.random.default_rng(77)
    seen_multi = seen_reranked = 0
    for _ in range(400):
        R, C, w, masks = _rand_case(rng)
        try:
            lv = rec.plan(w, masks)
        except o.NoHealthyChannel:
            # then no order of the global ring that this project's re-ranking finds has a channel on
            # every link; in particular the given order has a dead link
            assert rl.ring_bandwidth(w, masks) == 0
            continue
        seen_multi += len(lv) > 2
        assert lv[0].members == list(range(R))
        assert sum(l.share for l in lv) == 1 and all(l.share > 0 for l in lv)
        assert sum(l.increment for l in lv) == lv[-1].bandwidth
        for a, b in zip(lv, lv[1:]):
            assert set(b.members) < set(a.members) and len(b.members) >= 2
            assert b.bandwidth > a.bandwidth and (b.fail_mask & ~a.fail_mask) == 0
            # the ranks left out are slower than every rank kept
            slow = max(rec.own_bandwidth(w, masks[r]) for r in set(a.members) - set(b.members))
            assert slow < min(rec.own_bandwidth(w, masks[r]) for r in b.members)
        for l in lv:
            union = 0
            for r in l.members:
                union |= masks[r]
            assert l.fail_mask == union and sorted(l.order) == l.members
            # a ring runs at its narrowest link's rate: at least what all members share, at most what
            # its slowest member has left; and re-ranking never made it slower than the plain order
            links = [rec.own_bandwidth(w, masks[a] | masks[b]) for a, b in zip(l.order, l.order[1:] + l.order[:1])]
            assert l.bandwidth == min(links)
            assert rec.own_bandwidth(w, union) <= l.bandwidth <= min(rec.own_bandwidth(w, masks[r]) for r in l.members)
            excl = [r for r in range(R) if r not in l.members]
            start = excl[-1] + 1 if excl else 0
            base = [(start + i) % R for i in range(R) if (start + i) % R in l.members]
            seen_reranked += base != l.order
        # the lower rings finish together, nobody finishes later, and the time per unit of added
        # bandwidth does not fall from level to level
        t = [sp.ring_factor(len(l.members)) * l.share / l.increment for l in lv]
        u = [l.share / l.increment for l in lv]
        assert t[0] == max(t) and (len(lv) == 1 or t[1] == t[0])
        assert all(a <= b for a, b in zip(u, u[1:]))
        # a truncated peel is a prefix in members, and depth 0 is the single ring
        for d in range(1, len(lv) + 1):
            cut = rec.plan(w, masks, 1, d)
            assert [l.members for l in cut] == [l.members for l in lv[:d]]
    assert seen_multi > 20 and seen_reranked > 5


# ------------------------------------------------------------------ selector

def test_selector_follows_the_papers_threshold_for_one_failure():
    """Appendix A: with latency ignored, splitting wins iff the lost fraction X exceeds
    ng/(3ng-2) (a little above 1/3).  Checked on both sides of it for eight servers."""
    n = 8
    for lost, want in ((1, 0), (2, 0), (3, 1), (4, 1), (6, 1)):
        masks = [0] * n
        masks[5] = (1 << lost) - 1
        assert (F(lost, 8) > sp.threshold(n, 1)) == bool(want)
        depth, times = rec.select_depth(EQ8, masks, 1, 1 << 30, 0, 1)
        assert depth == want, (lost, times)


def test_latency_terms_by_hand():
    """One ring of p participants is the textbook ring all-reduce: 2(p-1) steps of latency alpha each and
    2(p-1)/p of the data over the ring's bandwidth.  The worked example of four servers (rings of 4, 3, 2)
    with no data at all is latency only: the longest reduction, 2*3 steps, then the longest broadcast --
    the top level's, which walks two servers left out, two members and the two left out again: 5 hops."""
    for n, g in ((4, 1), (8, 8), (5, 3)):
        lv = rec.plan(EQ8, [0] * n, g)
        assert len(lv) == 1
        p = n * g
        assert rec.completion_time(lv, n, g, F(10**9), F(3, 10**6), F(7)) == \
            2 * (p - 1) * F(3, 10**6) + F(2 * (p - 1), p) * F(10**9) / (400000 * 7)
    lv = rec.plan(EQ8, [0b1111, 0b0011, 0, 0])
    assert rec.completion_time(lv, 4, 1, 0, 1, 1) == 6 + 5
    assert rec.completion_time(lv, 4, 2, 0, 1, 1) == 14 + 5      # two GPUs per server: rings of 8, 6, 4


def test_selector_prefers_balance_for_small_messages():
    """Sec. 8 (AllReduce performance): for small messages R2CCL-Balance is faster, because the split
    schedule's extra steps cost latency; for large ones the split schedule is."""
    masks = [0] * 8
    masks[0] = 0b1111
    alpha, beta = 5e-6, 1e3  # 5 us per hop; 50000 units * 1e3 = 50 MB/s... the ratio is what matters
    small, _ = rec.select_depth(EQ8, masks, 1, 1 << 10, alpha, beta)
    large, _ = rec.select_depth(EQ8, masks, 1, 1 << 34, alpha, beta)
    assert (small, large) == (0, 1)


def test_selector_ties_go_to_the_shallower_plan():
    """Nothing to move and no latency: every depth takes time 0; the plain balanced ring is chosen."""
    depth, times = rec.select_depth(EQ8, [0b1111, 0b11, 0, 0], 1, 0, 0, 1)
    assert times == [0, 0, 0] and depth == 0


def test_time_is_monotone_in_alpha_and_bytes():
    lv = rec.plan(EQ8, [0b1111, 0b11, 0, 0])
    t = lambda b, a: rec.completion_time(lv, 4, 1, b, a, F(1, 1000))
    assert t(1000, 0) < t(2000, 0) and t(1000, 0) < t(1000, F(1, 10))
    assert t(2000, 0) == 2 * t(1000, 0)


# ------------------------------------------------------------------ schedule

def _inputs(rng, R, N, dtype):
    xs = []
    for _ in range(R):
        x = rng.standard_normal(N).astype(np.float32)
        if dtype == o.BF16:
            x = np.array([o.f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
        xs.append(x)
    return xs


def _elems(levels, unit):
    """Segment sizes that divide into every level's ring: the more the higher the share (roughly)."""
    return [unit * len(l.members) * max(1, int(4 * l.share)) for l in levels]


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_schedule_matches_definition_and_is_an_allreduce(dtype):
    rng = np.random.default_rng(5 + dtype)
    per16 = 4 if dtype == o.F32 else 8
    w = [3, 5, 7, 11]
    for masks in ([0b0001, 0b0011, 0, 0b0001, 0], [0b1000, 0, 0, 0], [0b0110, 0b0010, 0b0100, 0, 0, 0],
                  [0, 0b0001, 0b0011, 0b0111, 0]):
        R = len(masks)
        lv = rec.plan(w, masks)
        assert len(lv) >= 2
        elems = _elems(lv, per16 * 3)
        xs = _inputs(rng, R, sum(elems), dtype)
        want = rec.recursive_expected(xs, dtype, lv, elems, 1)
        bufs = [x.copy() for x in xs]
        rec.recursive_sim(bufs, dtype, lv, elems, 1, len(w), 16, w, masks)
        for r in range(R):
            assert bufs[r].tobytes() == want[r].tobytes()
            assert bufs[r].tobytes() == bufs[0].tobytes()
        # an all-reduce: equal to the exact sum within the rounding of R-1 additions
        wide = (lambda a: (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)) if dtype == o.BF16 \
            else (lambda a: a.astype(np.float64))
        exact = np.sum([wide(x) for x in xs], axis=0)
        mag = np.sum([np.abs(wide(x)) for x in xs], axis=0)
        u = 2.0 ** -24 if dtype == o.F32 else 2.0 ** -8
        assert np.all(np.abs(wide(bufs[0]) - exact) <= (R - 1) * u * mag * 1.01 + 1e-30)


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_one_degraded_rank_reproduces_the_split_schedule(dtype):
    """Sec. 5.2 is the two-level case: same bits as the split schedule's oracle."""
    rng = np.random.default_rng(9)
    per16 = 4 if dtype == o.F32 else 8
    R, d, C = 5, 3, 4
    w = [50000] * C
    masks = [0] * R
    masks[d] = 0b0101
    lv = rec.plan(w, masks)
    assert len(lv) == 2 and lv[0].order == list(range(R))
    ng, npart = R * 2 * per16 * 5, (R - 1) * 3 * per16 * 3
    xs = _inputs(rng, R, ng + npart, dtype)
    a = [x.copy() for x in xs]
    trace = rec.recursive_sim(a, dtype, lv, [ng, npart], 1, C, 32, w, masks)
    b = [x.copy() for x in xs]
    t_two, stage = sp.split_sim(b, dtype, d, npart, 1, 1, C, 32, w, masks[d])
    for r in range(R):
        assert a[r].tobytes() == b[r].tobytes()
    # the broadcast's links and stage buffers too: links that touch d are cut by d's channel state
    assert trace[0][1] is None
    _, visits, tables, st = trace[1]
    assert [r for r, _ in visits] == [d] + [(d + 1 + i) % R for i in range(R - 1)] + [d]
    assert [role for _, role in visits] == ["gather"] + ["member"] * (R - 1) + ["take"]
    for i in range(len(visits) - 1):
        touches_d = d in (visits[i][0], visits[i + 1][0])
        assert tables[i].tolist() == t_two[0 if touches_d else 1].tolist()
    for par in range(2):
        for c in range(C):
            assert st[par][c].tobytes() == stage[par][c].tobytes()


def test_links_are_cut_by_both_ends():
    """A link's table is the partition under the failed channels of BOTH its ends: a channel that either
    end has lost carries nothing; by hand for the rings and one chain with two excluded ranks.  Rank 0
    has rails {2,3}, rank 1 rails {0,1,3}: as neighbours they share one rail, fewer than rank 0 could
    sustain (2), so the global ring is re-ranked: rank 2 goes between them, 0 2 1 3."""
    w = [1, 1, 1, 1]
    masks = [0b0011, 0b0100, 0, 0]           # own bandwidth 2, 3, 4, 4
    lv = rec.plan(w, masks)
    assert [l.members for l in lv] == [[0, 1, 2, 3], [1, 2, 3], [2, 3]]
    assert [l.order for l in lv] == [[0, 2, 1, 3], [1, 2, 3], [2, 3]]
    assert [l.bandwidth for l in lv] == [2, 3, 4]   # one table for all would leave the global ring rail 3 alone
    elems = [4 * 16, 3 * 16, 2 * 32]
    xs = _inputs(np.random.default_rng(3), 4, sum(elems), o.F32)
    trace = rec.recursive_sim([x.copy() for x in xs], o.F32, lv, elems, 1, 4, 16, w, masks)
    # level 0's ring, chunks of 16 elements = 64 bytes = 4 units: link 0 -> 2 has rails 2 and 3
    ring_tables = trace[0][0]
    assert ring_tables.shape == (4, 6, 5)
    assert ring_tables[0, 0].tolist() == [0, 0, 0, 32, 64]       # 0 -> 2: rails 2, 3
    assert ring_tables[1, 0].tolist() == [0, 16, 32, 32, 64]     # 2 -> 1: rails 0, 1, 3: floor(4/3), floor(8/3) units
    assert ring_tables[2, 0].tolist() == [0, 16, 32, 32, 64]     # 1 -> 3
    assert ring_tables[3, 0].tolist() == [0, 0, 0, 32, 64]       # 3 -> 0
    _, visits, tables, _ = trace[2]
    assert [r for r, _ in visits] == [0, 1, 2, 3, 0, 1]
    nbytes = elems[2] * 4                     # 256 bytes
    # link 0 -> 1: channels 0, 1 (rank 0) and 2 (rank 1) are down: everything rides on channel 3
    assert tables[0].tolist() == [0, 0, 0, 0, nbytes]
    # link 1 -> 2: only channel 2 is down: thirds of 256 in units of 16 bytes: 5, 5 and 6 units
    assert tables[1].tolist() == [0, 80, 160, 160, nbytes]
    # link 2 -> 3: nothing down: quarters
    assert tables[2].tolist() == [0, 64, 128, 192, nbytes]
    # link 3 -> 0: rank 0's state
    assert tables[3].tolist() == [0, 0, 0, 128, nbytes]


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_relays_between_ranks_that_share_no_rail(dtype):
    """The case re-ranking and the relay rule exist for: two servers that lost complementary halves of
    their NICs are left out of the upper ring and must still add their data up and get the result.  The
    schedule runs, every rank ends with the same bits, they are the definition's, and the relay's own
    data is untouched by what it forwards (it shows in the result only through its own additions)."""
    per16 = 4 if dtype == o.F32 else 8
    w = [1] * 8
    masks = [0b00001111, 0b11110000, 0, 0, 0, 0]
    lv = rec.plan(w, masks)
    elems = [6 * per16 * 3, 4 * per16 * 5]
    xs = _inputs(np.random.default_rng(21), 6, sum(elems), dtype)
    want = rec.recursive_expected(xs, dtype, lv, elems, 1)
    bufs = [x.copy() for x in xs]
    trace = rec.recursive_sim(bufs, dtype, lv, elems, 1, 8, 16, w, masks)
    for r in range(6):
        assert bufs[r].tobytes() == want[r].tobytes()
    _, visits, tables, _ = trace[1]
    assert [role for _, role in visits].count("relay") == 2
    nbytes = elems[1] * xs[0].itemsize
    assert tables[0].tolist() == o.partition(w, 0b00001111, nbytes, 16).tolist()   # 0 -> relay 2: rank 0's rails
    assert tables[1].tolist() == o.partition(w, 0b11110000, nbytes, 16).tolist()   # relay 2 -> 1: rank 1's rails


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_relay_on_the_way_in_only_by_hand(dtype):
    """Four servers, eight equal NICs: server 0 kept NICs 0-1, server 1 lost exactly those.  The global
    ring is re-ranked to 0 2 1 3; the upper ring 1 2 3 adds 4 to its 2.  Its broadcast starts at server 0,
    whose first stop, server 1, shares nothing with it: the hop goes through server 2 -- before server 2's
    own turn as a member.  The way back, 3 -> 0, needs no relay, so nothing ever repairs what the relay
    would have damaged: server 2's own result must come out of forwarding untouched."""
    per16 = 4 if dtype == o.F32 else 8
    w, masks = [1] * 8, [0b11111100, 0b00000011, 0, 0]
    lv = rec.plan(w, masks, max_levels=2)
    assert [l.members for l in lv] == [[0, 1, 2, 3], [1, 2, 3]]
    assert [l.order for l in lv] == [[0, 2, 1, 3], [1, 2, 3]]
    assert [l.bandwidth for l in lv] == [2, 6]
    assert rec.chain_visits(4, 8, masks, lv[1]) == [
        (0, "gather"), (2, "relay"), (1, "member"), (2, "member"), (3, "member"), (0, "take")]
    elems = [4 * per16 * 3, 3 * per16 * 4]
    xs = _inputs(np.random.default_rng(33), 4, sum(elems), dtype)
    bufs = [x.copy() for x in xs]
    rec.recursive_sim(bufs, dtype, lv, elems, 1, 8, 16, w, masks)
    want = rec.recursive_expected(xs, dtype, lv, elems, 1)
    for r in range(4):
        assert bufs[r].tobytes() == want[r].tobytes()


def test_relay_is_the_first_member_linked_to_both_ends_by_hand():
    """Five servers, eight equal NICs.  Servers 0, 1, 2 kept NICs {0,1}, {2,3}, {1,2}; server 3 lost NICs 2-3;
    server 4 lost nothing.  The three slow servers leave together; the upper ring is 3 4.  Servers 0 and 1
    share nothing.  Of the ring's members, server 3 is linked to 0 but not to 1, server 4 to both; server 2,
    which is left out too, is linked to both as well.  The rule asks the members first, in ring order, and
    wants a link to both ends: server 4 relays, on the way in and on the way out."""
    keep = lambda *nics: 0xFF & ~sum(1 << c for c in nics)
    masks = [keep(0, 1), keep(2, 3), keep(1, 2), 0b00001100, 0]
    lv = rec.plan([1] * 8, masks)
    assert [l.members for l in lv] == [[0, 1, 2, 3, 4], [3, 4]]
    assert lv[0].order == [0, 4, 1, 2, 3] and lv[1].order == [3, 4]
    assert [l.bandwidth for l in lv] == [1, 6]
    assert rec.chain_visits(5, 8, masks, lv[1]) == [
        (0, "gather"), (4, "relay"), (1, "gather"), (2, "gather"), (3, "member"), (4, "member"),
        (0, "take"), (4, "relay"), (1, "take"), (2, "take")]


def test_chain_visits():
    full = [0] * 6
    lv = rec.plan([1] * 4, [0, 0, 0, 0b1, 0])
    assert [l.order for l in lv] == [[0, 1, 2, 3, 4], [4, 0, 1, 2]]
    assert rec.chain_visits(5, 4, [0, 0, 0, 0b1, 0], lv[0]) == []
    assert [r for r, _ in rec.chain_visits(5, 4, [0, 0, 0, 0b1, 0], lv[1])] == [3, 4, 0, 1, 2, 3]
    lv = rec.plan([1] * 4, [0b1, 0b1, 0, 0b1, 0b1, 0])
    assert lv[1].order == [5, 2]
    assert [r for r, _ in rec.chain_visits(6, 4, [0b1, 0b1, 0, 0b1, 0b1, 0], lv[1])] == [0, 1, 3, 4, 5, 2, 0, 1, 3, 4]
    assert rec.hops(5, 4) == 5 and rec.hops(6, 2) == 9 and full == [0] * 6


# ------------------------------------------------------------------ product's host planner vs oracle

def test_host_planner_matches_oracle(r2):
    rng = np.random.default_rng(78)
    n_multi = 0
    for _ in range(300):
        R, C, w, masks = _rand_case(rng)
        g = int(rng.integers(1, 9))
        try:
            want = rec.plan(w, masks, g)
        except o.NoHealthyChannel:
            with pytest.raises(r2.R2Error) as e:
                r2.r2_recursive_plan(w, masks, g)
            assert e.value.code == -2
            continue
        got = r2.r2_recursive_plan(w, masks, g)
        assert len(got) == len(want)
        for a, b in zip(got, want):
            assert a.ranks() == b.members and a.fail_mask == b.fail_mask
            assert r2.r2_recursive_ring_order(C, masks, a.members) == b.order
            assert (a.bandwidth, a.increment) == (b.bandwidth, b.increment)
            assert a.share == pytest.approx(float(b.share), rel=1e-13)
        n_multi += len(want) > 1
        for d in range(1, len(want) + 1):
            assert [l.members for l in r2.r2_recursive_plan(w, masks, g, d)] == [l.members for l in got[:d]]
        nbytes, alpha, beta = float(rng.integers(1, 1 << 34)), float(rng.random() * 1e-5), float(rng.random() + 0.1)
        t = r2.r2_recursive_time(R, g, got, nbytes, alpha, beta)
        assert t == pytest.approx(float(rec.completion_time(want, R, g, F(nbytes), F(alpha), F(beta))), rel=1e-12)
        depth, times = r2.r2_select_strategy(w, masks, g, nbytes, alpha, beta)
        odepth, otimes = rec.select_depth(w, masks, g, F(nbytes), F(alpha), F(beta))
        assert len(times) == len(otimes)
        assert times == pytest.approx([float(x) for x in otimes], rel=1e-12)
        # the choice may differ only where two depths tie to rounding
        assert depth == odepth or abs(times[depth] - times[odepth]) <= 1e-12 * times[odepth]
    assert n_multi > 100


def _masks_for(increments, participants):
    """A failure pattern (equal NICs, one GPU per server) whose plan has these increments and ring sizes:
    the servers that leave before level k keep the first sum(increments[:k]) NICs."""
    C = sum(increments)
    masks = []
    for k in range(1, len(increments)):
        kept = sum(increments[:k])
        masks += [((1 << C) - 1) & ~((1 << kept) - 1)] * (participants[k - 1] - participants[k])
    return C, masks + [0] * participants[-1]


def test_host_planner_on_the_share_rules_corner_cases(r2):
    """The plans in which a later balance level wins, and every exact tie between two balance levels that
    small increments and ring sizes produce (the product compares in doubles, where an exact tie is a
    matter of rounding unless it is handled): shares as the oracle's."""
    import itertools

    cases = [((2, 1, 1), (4, 3, 2)), ((1, 1, 6), (8, 7, 2)), ((1, 1, 4, 1), (8, 7, 3, 2)), ((1, 1, 1, 4), (9, 8, 7, 2))]
    n_ties = 0
    for parts in itertools.combinations(range(12, 1, -1), 3):
        for inc in itertools.product(range(1, 9), repeat=3):
            f = [F(2 * (p - 1), p) for p in parts]
            t1 = (1 + 1 / f[1]) / (inc[0] / f[0] + (inc[1] + inc[2]) / f[1])
            t2 = (1 + 1 / f[2]) / sum(i / x for i, x in zip(inc, f))
            if t1 == t2:
                cases.append((inc, parts))
                n_ties += 1
    assert n_ties > 50
    for inc, parts in cases:
        C, masks = _masks_for(inc, parts)
        want = rec.plan([1000] * C, masks)
        assert [l.increment for l in want] == [1000 * i for i in inc] and [len(l.members) for l in want] == list(parts)
        got = r2.r2_recursive_plan([1000] * C, masks, 1)
        assert [l.ranks() for l in got] == [l.members for l in want]
        for a, b in zip(got, want):
            assert a.share == pytest.approx(float(b.share), rel=1e-13), (inc, parts)


def _masks_for(increments, participants):
    """A failure pattern (equal NICs, one GPU per server) whose plan has these increments and ring sizes:
    the servers that leave before level k keep the first sum(increments[:k]) NICs."""
    C = sum(increments)
    masks = []
    for k in range(1, len(increments)):
        kept = sum(increments[:k])
        masks += [((1 << C) - 1) & ~((1 << kept) - 1)] * (participants[k - 1] - participants[k])
    return C, masks + [0] * participants[-1]


def test_host_planner_on_the_share_rules_corner_cases(r2):
    """The plans in which a later balance level wins, and every exact tie between two balance levels that
    small increments and ring sizes produce (the product compares in doubles, where an exact tie is a
    matter of rounding unless it is handled): shares as the oracle's."""
    import itertools

    cases = [((2, 1, 1), (4, 3, 2)), ((1, 1, 6), (8, 7, 2)), ((1, 1, 4, 1), (8, 7, 3, 2)), ((1, 1, 1, 4), (9, 8, 7, 2))]
    n_ties = 0
    for parts in itertools.combinations(range(12, 1, -1), 3):
        for inc in itertools.product(range(1, 9), repeat=3):
            f = [F(2 * (p - 1), p) for p in parts]
            t1 = (1 + 1 / f[1]) / (inc[0] / f[0] + (inc[1] + inc[2]) / f[1])
            t2 = (1 + 1 / f[2]) / sum(i / x for i, x in zip(inc, f))
            if t1 == t2:
                cases.append((inc, parts))
                n_ties += 1
    assert n_ties > 50
    for inc, parts in cases:
        C, masks = _masks_for(inc, parts)
        want = rec.plan([1000] * C, masks)
        assert [l.increment for l in want] == [1000 * i for i in inc] and [len(l.members) for l in want] == list(parts)
        got = r2.r2_recursive_plan([1000] * C, masks, 1)
        assert [l.ranks() for l in got] == [l.members for l in want]
        for a, b in zip(got, want):
            assert a.share == pytest.approx(float(b.share), rel=1e-13), (inc, parts)


def test_segments_follow_the_shares_and_fit_the_rings(r2):
    """Every segment divides into its ring in whole 16-byte vectors, level 0's into the global ring; the
    upper levels get their share rounded down by less than one granule, level 0 the rest; the host
    routine agrees with the oracle (a share in doubles may fall one granule short at an exact multiple)."""
    from math import gcd

    rng = np.random.default_rng(79)
    checked = planned = 0
    for _ in range(300):
        R, C, w, masks = _rand_case(rng)
        try:
            lv = rec.plan(w, masks)
        except o.NoHealthyChannel:
            continue
        planned += 1
        es = (2, 4)[int(rng.integers(0, 2))]
        S = int(rng.integers(1, 4))
        per16 = 16 // es
        N = S * R * per16 * int(rng.integers(1, 1 << int(rng.integers(1, 20))))
        seg = rec.segments(lv, R, N, S, es)
        assert sum(seg) == N and all(n >= 0 for n in seg)
        for k, (l, n) in enumerate(zip(lv, seg)):
            p = len(l.members)
            assert n % (S * p * per16) == 0 and (n * es) % 16 == 0
            if k:
                granule = S * (p * R // gcd(p, R)) * per16
                assert n <= l.share * N < n + granule
        assert seg[0] >= lv[0].share * N
        desc = r2.RecursiveDesc(R, C, 16, N, r2.F32 if es == 4 else r2.BF16, len(lv), S)
        got = r2.r2_recursive_segments(desc, r2.r2_recursive_plan(w, masks))
        assert sum(got) == N
        for k, (a, b, l) in enumerate(zip(got, seg, lv)):
            p = len(l.members)
            granule = S * (p * R // gcd(p, R)) * per16
            assert a == b or (k and abs(a - b) == granule) or (k == 0 and abs(a - b) % (S * R * per16) == 0)
        checked += got == seg
    assert planned > 150 and checked >= 0.95 * planned, (checked, planned)
    with pytest.raises(r2.R2Error):  # the buffer does not divide into the global ring
        r2.r2_recursive_segments(r2.RecursiveDesc(4, 8, 16, 4 * 4 * 3 + 4, r2.F32, 1), [r2.Level(0b1111, 0, 8, 8, 1.0)])


def test_segments_by_hand():
    """The worked example (shares 16 : 9 : 9 of 34), fp32, one slab, 4 ranks: granules are
    lcm(3, 4) * 4 = 48 and lcm(2, 4) * 4 = 16 elements; 34 * 1600 elements."""
    lv = rec.plan(EQ8, [0b1111, 0b0011, 0, 0])
    N = 34 * 1600
    assert rec.segments(lv, 4, N, 1, 4) == [N - 14400 - 14400, 14400, 14400]  # 9 * 1600 = 14400 = 300 * 48 = 900 * 16
    assert rec.segments(lv, 4, 16 * 34, 1, 4) == [256, 144, 144]                 # exact: 144 = 3 * 48 = 9 * 16
    # 640 elements: 9/34 of them is 169.4 -> 144 (3 * 48) for level 1, 160 (10 * 16) for level 2, the rest to level 0
    assert rec.segments(lv, 4, 640, 1, 4) == [336, 144, 160]


def test_host_selector_ties_go_to_the_shallower_plan(r2):
    depth, times = r2.r2_select_strategy(EQ8, [0b1111, 0b11, 0, 0], 1, 0.0, 0.0, 1.0)
    assert times == [0.0, 0.0, 0.0] and depth == 0


def test_host_planner_rejects_bad_arguments(r2):
    with pytest.raises(r2.R2Error):
        r2.r2_recursive_plan(EQ8, [0])  # one rank
    with pytest.raises(r2.R2Error):
        r2.r2_recursive_plan(EQ8, [0, 0], 0)  # no GPUs
    with pytest.raises(r2.R2Error):
        r2.r2_recursive_plan(EQ8, [0, 0], 1, 0)  # no levels
    with pytest.raises(r2.R2Error):
        r2.r2_recursive_plan(EQ8, [0, 0], 1, 17)
    assert r2.r2_recursive_time(4, 1, [r2.Level(0b1111, 0, 8, 0, 1.0)], 1.0, 0.0, 1.0) < 0  # increment 0
    assert r2.r2_recursive_time(4, 1, [r2.Level(0b1111, 0, 8, 8, 1.0)], 1.0, 0.0, 0.0) < 0  # beta 0
