"""Recursive R2CCL-AllReduce (Sec. 6): pins for the oracle's plan, time model and schedule, and parity
of the product's host planner against it.  No GPU involved.

What the paper fixes, and what therefore pins this part: one degraded server must give the two-ring
schedule and T(Y) of Sec. 5.2; the result must be an all-reduce; the levels are nested rings of
growing bandwidth whose shares follow the bandwidth each adds.  Everything else is this project's
reading (the paper has no pseudo-code here) and is listed as such in the oracle's header."""
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
    at 4 NICs, {1,2,3} at 6 (adds 2), {2,3} at 8 (adds 2).  Equal finishing times need shares in the
    ratio 4/(2*3/4) : 2/(2*2/3) : 2/(2*1/2) = 16 : 9 : 12."""
    lv = rec.plan(EQ8, [0b1111, 0b0011, 0, 0])
    assert [l.members for l in lv] == [[0, 1, 2, 3], [1, 2, 3], [2, 3]]
    assert [l.fail_mask for l in lv] == [0b1111, 0b0011, 0]
    assert [l.bandwidth for l in lv] == [200000, 300000, 400000]
    assert [l.increment for l in lv] == [200000, 100000, 100000]
    assert [l.share for l in lv] == [F(16, 37), F(9, 37), F(12, 37)]


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
    rng = np.random.default_rng(77)
    seen_multi = 0
    for _ in range(400):
        R, C, w, masks = _rand_case(rng)
        try:
            lv = rec.plan(w, masks)
        except o.NoHealthyChannel:
            union = 0
            for m in masks:
                union |= m
            assert union == (1 << C) - 1
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
            assert l.fail_mask == union and l.bandwidth == rec.own_bandwidth(w, union)
        # all rings finish together when latency is ignored
        t = [sp.ring_factor(len(l.members)) * l.share / l.increment for l in lv]
        assert all(x == t[0] for x in t)
        # a truncated peel is a prefix in members, and depth 0 is the single ring
        for d in range(1, len(lv) + 1):
            cut = rec.plan(w, masks, 1, d)
            assert [l.members for l in cut] == [l.members for l in lv[:d]]
    assert seen_multi > 20


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
    assert len(lv) == 2
    ng, npart = R * 2 * per16 * 5, (R - 1) * 3 * per16 * 3
    xs = _inputs(rng, R, ng + npart, dtype)
    a = [x.copy() for x in xs]
    trace = rec.recursive_sim(a, dtype, lv, [ng, npart], 1, C, 32, w, masks)
    b = [x.copy() for x in xs]
    t_two, stage = sp.split_sim(b, dtype, d, npart, 1, 1, C, 32, w, masks[d])
    for r in range(R):
        assert a[r].tobytes() == b[r].tobytes()
    # the broadcast's links and stage buffers too: links that touch d are cut by d's channel state
    assert trace[0] is None
    chain, tables, st = trace[1]
    assert chain == [d] + [(d + 1 + i) % R for i in range(R - 1)] + [d]
    for i in range(len(chain) - 1):
        touches_d = d in (chain[i], chain[i + 1])
        assert tables[i].tolist() == t_two[0 if touches_d else 1].tolist()
    for par in range(2):
        for c in range(C):
            assert st[par][c].tobytes() == stage[par][c].tobytes()


def test_links_are_cut_by_both_ends():
    """A link's table is the partition under the failed channels of BOTH its ends: a channel that either
    end has lost carries nothing; by hand for one link of a chain with two excluded ranks."""
    w = [1, 1, 1, 1]
    masks = [0b0011, 0b0100, 0, 0]           # own bandwidth 2, 3, 4, 4
    lv = rec.plan(w, masks)
    assert [l.members for l in lv] == [[0, 1, 2, 3], [1, 2, 3], [2, 3]]
    elems = [4 * 16, 3 * 16, 2 * 32]
    xs = _inputs(np.random.default_rng(3), 4, sum(elems), o.F32)
    trace = rec.recursive_sim([x.copy() for x in xs], o.F32, lv, elems, 1, 4, 16, w, masks)
    chain, tables, _ = trace[2]
    assert chain == [0, 1, 2, 3, 0, 1]
    nbytes = elems[2] * 4                     # 256 bytes
    # link 0 -> 1: channels 0, 1 (rank 0) and 2 (rank 1) are down: everything rides on channel 3
    assert tables[0].tolist() == [0, 0, 0, 0, nbytes]
    # link 1 -> 2: only channel 2 is down: thirds of 256 in units of 16 bytes: 5, 5 and 6 units
    assert tables[1].tolist() == [0, 80, 160, 160, nbytes]
    # link 2 -> 3: nothing down: quarters
    assert tables[2].tolist() == [0, 64, 128, 192, nbytes]
    # link 3 -> 0: rank 0's state
    assert tables[3].tolist() == [0, 0, 0, 128, nbytes]


def test_chain_order():
    assert rec.chain_order(5, [0, 1, 2, 3, 4]) == ([], [0, 1, 2, 3, 4])
    assert rec.chain_order(5, [0, 1, 2, 4]) == ([3], [4, 0, 1, 2])
    assert rec.chain_order(6, [2, 5]) == ([0, 1, 3, 4], [5, 2])
    assert rec.hops(5, 4) == 5 and rec.hops(6, 2) == 9


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
    """The worked example (shares 16 : 9 : 12 of 37), fp32, one slab, 4 ranks: granules are
    lcm(3, 4) * 4 = 48 and lcm(2, 4) * 4 = 16 elements; 37 * 1600 elements."""
    lv = rec.plan(EQ8, [0b1111, 0b0011, 0, 0])
    N = 37 * 1600
    assert rec.segments(lv, 4, N, 1, 4) == [N - 14400 - 19200, 14400, 19200]  # 9 * 1600 = 14400 = 300 * 48
    assert rec.segments(lv, 4, 16 * 37, 1, 4) == [256, 144, 192]                 # exact: 144 = 3 * 48, 192 = 12 * 16
    # 640 elements: 9/37 of them is 155.7 -> 144 (3 * 48), 12/37 is 207.6 -> 192 (12 * 16), the rest to level 0
    assert rec.segments(lv, 4, 640, 1, 4) == [304, 144, 192]


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
