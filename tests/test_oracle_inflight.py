"""Pins for the oracle of a ring run with failures in flight (CPU only).

Paper: Sec. 4.3 Technique II (rewind to the first chunk without a completion, retransmit it over the
NICs that are left; completed chunks stay), Sec. 5.1 (shares in proportion to bandwidth), Sec. 8.2
(lossless whatever the failure timing).  The hand-worked cases A and B of golden/rollback_cases.txt
are the tables of the first two benchmark configurations: 1 MiB chunks over four equal channels with
channel 2 down, and 16 MiB chunks over eight equal channels where channels 2 and 5 fail.
"""
import os

import numpy as np
import pytest

import workloads as wl
from inflight_util import random_case as _random_case
from oracle import inflight

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rollback_cases.txt")


def _golden(name):
    for line in open(GOLDEN):
        if line.startswith(name + " |"):
            _, w, mb, ma, align, off, rows, _ = [s.strip() for s in line.split("|")]
            want = {}
            for part in rows.split(";"):
                f, vals = part.split(":")
                want[int(f)] = [int(x) for x in vals.split()]
            return [int(x) for x in w.split()], int(mb, 16), int(ma, 16), int(align), [int(x) for x in off.split()], want
    raise KeyError(name)


def _codes(oracle, w):
    return (oracle.F32 if w.dtype == "f32" else oracle.BF16,
            {"ar": oracle.PHASE_AR, "rs": oracle.PHASE_RS, "ag": oracle.PHASE_AG}[w.phases])


def test_hand_case_A_first_configuration(oracle):
    """cfg1 (4 ranks, fp32, 1 MiB chunks, channel 2 down from the start); channel 0 fails during
    transmission 2.  Transmissions 0..2 keep the table 0 349440 698880 698880 1048576; the plan shares
    channel 0's 349440 bytes as 174592 to channel 1 and the rest to channel 3; transmissions 3..5 are
    cut over channels 1 and 3 alone."""
    weights, mb, ma, align, off, want = _golden("A")
    w = wl.cfg1()
    assert w.chunk_bytes == off[-1] and w.epochs[0][1] == mb and list(w.epochs[0][2]) == weights
    epochs = [w.epochs[0], (2, ma, tuple(weights))]
    xs = wl.make_inputs(w)
    odt, oph = _codes(oracle, w)
    bufs = [x.copy() for x in xs]
    log, _, plans = inflight.ring_sim_inflight(bufs, odt, w.S, w.C, align, epochs, [False, True], oph)
    for t in (0, 1, 2):
        assert log[t].tolist() == off
    half = 1048576 // 256 // 2 * 256
    for t in (3, 4, 5):
        assert log[t].tolist() == [0, 0, half, half, 1048576]
    assert sorted(plans) == [1]
    for f in range(w.C):
        assert plans[1][f].tolist() == want.get(f, [0] * (w.C + 1))
    for got, exp in zip(bufs, oracle.expected(xs, odt, w.S, oph)):
        assert got.tobytes() == exp.tobytes()


def test_hand_case_B_second_configuration(oracle):
    """cfg2 (8 ranks, bf16, 16 MiB chunks, 8 equal channels): channels 2 and 5 fail during
    transmission 3.  Rows 0..3 are the even split, rows 4.. are cut over the six survivors, and each
    failed 2 MiB slice is shared out as the golden rows say."""
    weights, mb, ma, align, off, want = _golden("B")
    w = wl.cfg2()
    assert w.chunk_bytes == off[-1] and w.epochs[0][1] == mb and w.epochs[1][:2] == (3, ma)
    xs = wl.make_inputs(w)
    odt, oph = _codes(oracle, w)
    bufs = [x.copy() for x in xs]
    log, _, plans = inflight.ring_sim_inflight(bufs, odt, w.S, w.C, align, list(w.epochs), [False, True], oph, cap=w.chunk_bytes)
    for t in range(4):
        assert log[t].tolist() == off
    survivors = oracle.partition(weights, ma, w.chunk_bytes, align).tolist()
    assert survivors[2] == survivors[3] and survivors[5] == survivors[6]
    for t in range(4, log.shape[0]):
        assert log[t].tolist() == survivors
    for f in range(w.C):
        assert plans[1][f].tolist() == want.get(f, [0] * (w.C + 1))
    for got, exp in zip(bufs, oracle.expected(xs, odt, w.S, oph)):
        assert got.tobytes() == exp.tobytes()


def test_plan_shares_by_the_weights_the_failure_leaves_by_hand(oracle):
    """Two ranks, fp32, one 4 KiB chunk per rank half, four channels, 256-byte units.  Equal weights cut
    the chunk at 1024, 2048, 3072.  Channel 0 fails during transmission 1 and the state it leaves rates
    channels 1, 2, 3 at 3 : 1 : 0.  The struck transmission keeps the even table; channel 0's four units
    are re-carried three by channel 1 and one by channel 2, none by channel 3 (healthy, weight 0) --
    with the old, equal weights it would have been 1 : 1 : 2 units."""
    rng = np.random.default_rng(8)
    xs = [rng.standard_normal(2048).astype(np.float32) for _ in range(2)]
    epochs = [(0, 0, (1, 1, 1, 1)), (1, 0b0001, (5, 3, 1, 0))]
    bufs = [x.copy() for x in xs]
    log, _, plans = inflight.ring_sim_inflight(bufs, oracle.F32, 1, 4, 256, epochs, [False, True], oracle.PHASE_AR)
    assert log.tolist() == [[0, 1024, 2048, 3072, 4096]] * 2
    assert sorted(plans) == [1]
    assert plans[1].tolist() == [[0, 0, 768, 1024, 1024]] + [[0] * 5] * 3
    for got, exp in zip(bufs, oracle.expected(xs, oracle.F32, 1, oracle.PHASE_AR)):
        assert got.tobytes() == exp.tobytes()


def test_invariants_random(oracle):
    """What must hold whatever the rounding: the result is the plain definition's (lossless whatever
    the failure timing); the transmission a failure strikes in keeps the table of the state before it
    and every later one has the new state's; the bytes re-carried are exactly the newly failed slices,
    each byte by exactly one channel that is still up; channels that did not newly fail have no plan."""
    rng = np.random.default_rng(20251)
    n_plans = 0
    for _ in range(300):
        w, flags, T = _random_case(rng)
        xs = wl.make_inputs(w)
        odt, oph = _codes(oracle, w)
        bufs = [x.copy() for x in xs]
        log, stage, plans = inflight.ring_sim_inflight(bufs, odt, w.S, w.C, w.align, list(w.epochs), flags, oph)
        for got, exp in zip(bufs, oracle.expected(xs, odt, w.S, oph)):
            assert got.tobytes() == exp.tobytes()
        for t in range(T):
            # the state whose table transmission t has: the last epoch that started before t, or at t
            # unless it struck in flight
            cur = w.epochs[0]
            for e, fl in zip(w.epochs, flags):
                if e[0] < t or (e[0] == t and not fl):
                    cur = e
            assert log[t].tolist() == oracle.partition(cur[2], cur[1], w.chunk_bytes, w.align).tolist(), t
        for i, fl in enumerate(flags):
            k = w.epochs[i][0]
            assert (i in plans) == (fl and k < T)
            if i not in plans:
                continue
            n_plans += 1
            before, after = w.epochs[i - 1][1], w.epochs[i][1]
            newly = after & ~before
            row = log[k].astype(object)
            carried = 0
            for f in range(w.C):
                p = plans[i][f].astype(object)
                length = row[f + 1] - row[f]
                if not (newly >> f) & 1 or length == 0:
                    assert not p.any()
                    continue
                assert p[0] == 0 and p[-1] == length and all(p[c] <= p[c + 1] for c in range(w.C))
                for c in range(w.C):
                    if (after >> c) & 1:
                        assert p[c + 1] == p[c]  # a channel that is down carries nothing
                carried += int(p[-1])
            assert carried == sum(int(row[f + 1] - row[f]) for f in range(w.C) if (newly >> f) & 1)
    assert n_plans > 100


def test_without_flags_it_is_the_plain_ring(oracle):
    rng = np.random.default_rng(7)
    for _ in range(40):
        w, flags, _ = _random_case(rng)
        xs = wl.make_inputs(w)
        odt, oph = _codes(oracle, w)
        a, b = [x.copy() for x in xs], [x.copy() for x in xs]
        log1, stage1 = oracle.ring_sim(a, odt, w.S, w.C, w.align, list(w.epochs), oph)
        log2, stage2, plans = inflight.ring_sim_inflight(b, odt, w.S, w.C, w.align, list(w.epochs),
                                                         [False] * len(flags), oph)
        assert not plans and log1.tolist() == log2.tolist() and stage1.tobytes() == stage2.tobytes()
        assert all(x.tobytes() == y.tobytes() for x, y in zip(a, b))


def test_corner_cases(oracle):
    """By hand, 2 ranks x 2 slabs all-reduce (T = 4), 3 channels of weights 1:1:2, 64 bytes per chunk,
    alignment 16: the even state cuts 0 16 32 64.  (a) A failure of channel 2 in the last transmission
    changes no table and shares channel 2's 32 bytes 16/16.  (b) Failures in transmissions 1 and 2, one
    after the other: row 1 old, row 2 under the first failure (channel 0 down: U = 4 units, weight in
    front of the channels (0, 0, 1) of W = 3, floor(4*1/3) = 1 unit to channel 1: 0 0 16 64), row 3 under
    both (only channel 2 left).  (c) A failure in flight at transmission 1 followed by an ordinary epoch at
    transmission 2: its state never cuts a table, but its plan exists.  (d) Beyond the run: no effect."""
    from dataclasses import replace

    wts = (1, 1, 2)
    base = replace(wl.cfg1(), name="corner", R=2, dtype="f32", N=2 * 2 * 16, S=2, C=3, align=16, phases="ar",
                   sigma=1.0, seed=5)
    odt, oph = oracle.F32, oracle.PHASE_AR

    def run(epochs, flags):
        w = replace(base, epochs=tuple(epochs))
        bufs = [x.copy() for x in wl.make_inputs(w)]
        log, _, plans = inflight.ring_sim_inflight(bufs, odt, w.S, w.C, w.align, list(epochs), flags, oph)
        return log.tolist(), {i: p.tolist() for i, p in plans.items()}

    even = [0, 16, 32, 64]
    log, plans = run([(0, 0, wts), (3, 0b100, wts)], [False, True])
    assert log == [even] * 4
    assert plans == {1: [[0] * 4, [0] * 4, [0, 16, 32, 32]]}

    log, plans = run([(0, 0, wts), (1, 0b001, wts), (2, 0b011, wts)], [False, True, True])
    assert log == [even, even, [0, 0, 16, 64], [0, 0, 0, 64]]
    assert plans == {1: [[0, 0, 0, 16], [0] * 4, [0] * 4],      # 16 bytes = 1 unit: floor(1*1/3) = 0 -> all to channel 2
                     2: [[0] * 4, [0, 0, 0, 16], [0] * 4]}      # channel 1's 16 bytes of row 2 go to channel 2

    log, plans = run([(0, 0, wts), (1, 0b001, wts), (2, 0, (1, 1, 1))], [False, True, False])
    assert log == [even, even, [0, 16, 32, 64], [0, 16, 32, 64]]  # weights 1:1:1: floor(4/3) = 1, floor(8/3) = 2 units
    assert plans == {1: [[0, 0, 0, 16], [0] * 4, [0] * 4]}

    log, plans = run([(0, 0, wts), (4, 0b001, wts)], [False, True])
    assert log == [even] * 4 and plans == {}


def test_rejects_recovery_in_flight_and_first_epoch(oracle):
    w = wl.scaled(wl.cfg1(), 4 * 64)
    bufs = [x.copy() for x in wl.make_inputs(w)]
    with pytest.raises(oracle.OracleError):
        inflight.ring_sim_inflight(bufs, oracle.F32, 1, 4, 16, [(0, 0b0100, (1, 1, 1, 1)), (2, 0b0001, (1, 1, 1, 1))],
                                   [False, True], oracle.PHASE_AR)
    with pytest.raises(AssertionError):
        inflight.table_epochs([(0, 0, (1,))], [True])
