"""Pins for the oracle of R2CCL-AllReduce (CPU only): the planner's closed forms of Sec. 5.2 /
Appendix A against exact algebra and brute-force minimisation, the one number the paper prints
(Fig. 4: 2D becomes 1.75D), and the split schedule against the plain definition of an all-reduce.
Also the product's host-side planner against the oracle (no GPU needed)."""
from fractions import Fraction as F

import numpy as np
import pytest
import torch

from oracle import split

F32, BF16 = 0, 1


def test_fig4_workload_of_the_degraded_server():
    """Fig. 4: with a quarter of the data on the partial path the bottleneck server moves 1.75 D
    instead of the 2 D of a plain ring all-reduce."""
    assert split.degraded_server_volume(F(0)) == 2
    assert split.degraded_server_volume(F(1, 4)) == F(7, 4)


@pytest.mark.parametrize("n,g", [(2, 2), (2, 8), (3, 4), (4, 8), (16, 8), (64, 8)])
def test_printed_y_star_is_the_balance_point(n, g):
    """Appendix A, Step 1: the printed closed form equals the exact solution of T1 = T2."""
    for X in (F(1, 100), F(1, 8), F(1, 4), F(1, 3), F(1, 2), F(3, 4), F(99, 100)):
        assert split.y_star_paper(n, g, X) == split.balance_point(n, g, X)
        y = split.y_star_paper(n, g, X)
        assert 0 < y < 1 and y > X  # slightly more than the lost fraction goes the partial way


@pytest.mark.parametrize("n,g", [(2, 2), (2, 8), (4, 8), (8, 1), (16, 8)])
def test_threshold_and_minimiser_by_brute_force(n, g):
    """Appendix A, Step 3: below the threshold T(Y) is smallest at Y = 0 (plain ring); above it the
    minimum sits at Y*.  Checked by evaluating T on a fine grid of exact rationals."""
    thr = split.threshold(n, g)
    grid = [F(k, 2000) for k in range(2001)]
    for X in (thr / 2, thr - F(1, 1000), thr + F(1, 1000), (thr + 1) / 2, F(9, 10)):
        ts = [split.completion_time(n, g, X, y) for y in grid]
        best = grid[min(range(len(grid)), key=lambda k: ts[k])]
        ystar = split.y_star_paper(n, g, X)
        if X <= thr:
            assert best == 0
            assert split.completion_time(n, g, X, 0) <= split.completion_time(n, g, X, ystar)
        else:
            assert abs(best - ystar) <= F(1, 2000)
            assert split.completion_time(n, g, X, ystar) < split.completion_time(n, g, X, 0)
            assert all(split.completion_time(n, g, X, ystar) <= t for t in ts)
    assert F(1, 3) < thr <= F(1, 2)  # "in practice 1/3": the exact threshold is just above it


def test_plain_ring_time_at_y_zero():
    """T(0) is the ring all-reduce time 2(ng-1)/(ng) at the degraded bandwidth (1-X)."""
    assert split.completion_time(2, 8, F(1, 8), 0) == F(2 * 15, 16) / F(7, 8)


def test_product_planner_matches_oracle():
    import paper_2512_25059_amd as r2
    from paper_2512_25059_amd import build as hip_build

    if hip_build.is_stale():
        hip_build.build()
    for n, g in [(2, 2), (2, 8), (3, 1), (4, 8), (16, 8), (2, 1)]:
        for X in (0.01, 0.125, 0.25, 1 / 3, 0.34, 0.35, 0.4, 0.5, 0.75, 0.99):
            use, y, thr = r2.r2_split_plan(n, g, X)
            assert thr == pytest.approx(float(split.threshold(n, g)), rel=1e-14)
            assert y == pytest.approx(float(split.y_star_paper(n, g, F(X))), rel=1e-12)
            assert use == (X > float(split.threshold(n, g)) and (n - 1) * g >= 2)
            for yy in (0.0, 0.1, y, 0.9, 1.0):
                assert r2.r2_split_time(n, g, X, yy) == pytest.approx(float(split.completion_time(n, g, F(X), F(yy))), rel=1e-12)
    for bad in [(1, 8, 0.5), (2, 0, 0.5), (2, 8, 0.0), (2, 8, 1.0), (2, 8, -0.1)]:
        with pytest.raises(r2.R2Error):
            r2.r2_split_plan(*bad)


def test_partial_elems_follow_the_share_and_fit_both_rings():
    """The tail for share Y: both parts divide into their rings in whole 16-byte vectors, the tail is Y of
    the buffer rounded down by less than one granule.  By hand: 8 ranks, bf16, one slab each: granule
    lcm(8, 7) * 8 = 448 elements; Y = 0.5052 of 2^26 elements is 33 903 398.1 -> 75 677 * 448."""
    import paper_2512_25059_amd as r2
    from math import gcd

    assert r2.r2_split_partial_elems(8, 1, 1, r2.BF16, 1 << 26, 0.5052) == 75677 * 448
    rng = np.random.default_rng(13)
    for _ in range(300):
        R, Sg, Sp = int(rng.integers(3, 65)), int(rng.integers(1, 5)), int(rng.integers(1, 5))
        dt, per16 = ((r2.F32, 4), (r2.BF16, 8))[int(rng.integers(0, 2))]
        N = Sg * R * per16 * int(rng.integers(1, 1 << 16))
        y = float(rng.random())
        n = r2.r2_split_partial_elems(R, Sg, Sp, dt, N, y)
        granule = (Sg * R) * (Sp * (R - 1)) // gcd(Sg * R, Sp * (R - 1)) * per16
        assert n % (Sp * (R - 1) * per16) == 0 and (N - n) % (Sg * R * per16) == 0
        assert n <= y * N < n + granule + 1
    assert r2.r2_split_partial_elems(8, 1, 1, r2.BF16, (1 << 26) + 8, 0.5) == 0   # does not divide into the global ring
    assert r2.r2_split_partial_elems(2, 1, 1, r2.BF16, 1 << 20, 0.5) == 0         # no partial ring with one healthy rank
    assert r2.r2_split_partial_elems(8, 1, 1, 5, 1 << 20, 0.5) == 0 and r2.r2_split_partial_elems(8, 1, 1, r2.F32, 1 << 20, 1.5) == 0


# ------------------------------------------------------------------ schedule

def _inputs(rng, R, N, dtype, ints=False):
    xs = []
    for _ in range(R):
        x = rng.integers(-9, 10, size=N).astype(np.float32) if ints else rng.standard_normal(N).astype(np.float32)
        if dtype == BF16:
            x = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        xs.append(x)
    return xs


def _f64(dtype, a):
    return a.astype(np.float64) if dtype == F32 else (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_split_schedule_equals_its_definition_and_sums_everything(oracle, dtype):
    rng = np.random.default_rng(77 + dtype)
    es = 4 if dtype == F32 else 2
    for R in (3, 4, 6):
        for d in range(R):
            for Sg, Sp, Eg, Ep in ((1, 1, 8, 8), (2, 1, 4, 24), (1, 3, 12, 8)):
                ng, npart = Sg * R * Eg * (16 // es), Sp * (R - 1) * Ep * (16 // es)
                xs = _inputs(rng, R, ng + npart, dtype)
                bufs = [x.copy() for x in xs]
                split.split_sim(bufs, dtype, d, npart, Sg, Sp, 4, 16, (5, 3, 7, 1), 0b0100)
                want = split.split_expected(xs, dtype, d, npart, Sg, Sp)
                for r in range(R):
                    assert bufs[r].tobytes() == want[r].tobytes(), (R, d, r)
                    assert bufs[r].tobytes() == bufs[0].tobytes()  # everybody holds the same bits
                exact = sum(_f64(dtype, x) for x in xs)
                absum = sum(np.abs(_f64(dtype, x)) for x in xs)
                u = 2.0 ** -24 if dtype == F32 else 2.0 ** -8
                assert np.all(np.abs(_f64(dtype, bufs[0]) - exact) <= (R - 1) * u * absum * 1.01)
    # small integers: the split must give exactly the integer sum, like any all-reduce
    xs = _inputs(rng, 5, 5 * 8 * 4 + 4 * 8 * 4, dtype, ints=True)
    bufs = [x.copy() for x in xs]
    split.split_sim(bufs, dtype, 2, 4 * 8 * 4, 1, 1, 3, 16, (1, 1, 1), 0b001)
    total = sum(_f64(dtype, x) for x in xs)
    for b in bufs:
        assert np.array_equal(_f64(dtype, b), total)


def test_each_ring_is_cut_by_its_own_channel_state_by_hand(oracle):
    """Sec. 5.2: the global ring runs through the degraded server and is throttled to what that server has
    left; the partial ring runs among the healthy servers at full width.  Four ranks, fp32, four equal
    channels, rank 1 lost channels 0 and 1.  Head: 4 ring chunks of 64 bytes, every one of the 6
    transmissions cut over channels 2 and 3 alone (32 bytes each).  Tail: 3 ring chunks of 128 bytes,
    every one of the 4 transmissions cut into quarters.  Broadcast hops that touch rank 1 carry the
    384-byte tail on channels 2 and 3, the others on all four."""
    rng = np.random.default_rng(12)
    ng, npart = 4 * 16, 3 * 32
    xs = _inputs(rng, 4, ng + npart, F32)
    bufs = [x.copy() for x in xs]
    logs = {}
    tables, _ = split.split_sim(bufs, F32, 1, npart, 1, 1, 4, 16, (7, 7, 7, 7), 0b0011, ring_logs=logs)
    assert logs["global"].tolist() == [[0, 0, 0, 32, 64]] * 6
    assert logs["partial"].tolist() == [[0, 32, 64, 96, 128]] * 4
    assert tables.tolist() == [[0, 0, 0, 192, 384], [0, 96, 192, 288, 384]]
    want = split.split_expected(xs, F32, 1, npart, 1, 1)
    for r in range(4):
        assert bufs[r].tobytes() == want[r].tobytes()


def test_split_with_nothing_partial_is_the_plain_ring(oracle):
    rng = np.random.default_rng(5)
    xs = _inputs(rng, 4, 4 * 32, F32)
    bufs = [x.copy() for x in xs]
    split.split_sim(bufs, F32, 1, 0, 1, 1, 2, 16, (1, 1), 0b01)
    want = oracle.expected(xs, F32, 1, oracle.PHASE_AR)
    for a, b in zip(bufs, want):
        assert a.tobytes() == b.tobytes()


def test_relay_step_forwards_the_incoming_data(oracle):
    """R2_OP_SUM_FORWARD of the oracle: local gets the sum, the next stage the untouched incoming."""
    rng = np.random.default_rng(6)
    n, C = 64, 2
    inc, loc = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    off = oracle.partition([1, 1], 0, n * 4, 16)
    cap = n * 4
    ins = [np.full(cap, 0xA5, np.uint8) for _ in range(C)]
    raw = inc.view(np.uint8)
    for k in range(C):
        a, b = int(off[k]), int(off[k + 1])
        ins[k][:b - a] = raw[a:b]
    outs = [np.full(cap, 0xA5, np.uint8) for _ in range(C)]
    local = loc.copy()
    oracle.reduce_copy(local, F32, oracle.OP_SUM_FORWARD, ins, off, outs, off, C, cap)
    assert np.array_equal(local, inc + loc)
    got = np.concatenate([outs[k][:int(off[k + 1] - off[k])] for k in range(C)]).view(np.float32)
    assert np.array_equal(got, inc)
