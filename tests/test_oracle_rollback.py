"""Pins for the oracle's in-flight failover plan (CPU only).

Paper: Sec. 4.3 (live migration; buffers intact until completion, every NIC registered on every
buffer) and Sec. 5.1 (the failed NIC's portion goes to the healthy NICs in proportion to bandwidth).
What must hold whatever the rounding rule: every byte of a newly failed slice is carried by exactly
one healthy NIC, nothing is given to a NIC that is down, shares are proportional to within one
alignment unit, and nothing else is touched.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rollback_cases.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, w, mb, ma, align, off, rows, status = [s.strip() for s in line.split("|")]
        want = {}
        for part in rows.split(";"):
            part = part.strip()
            if part:
                f, vals = part.split(":")
                want[int(f)] = [int(x) for x in vals.split()]
        out.append((name, [int(x) for x in w.split()], int(mb, 16), int(ma, 16), int(align),
                    [int(x) for x in off.split()], want, int(status)))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_worked_examples(oracle, case):
    _, w, mb, ma, align, off, want, status = case
    C = len(w)
    if status != 0:
        with pytest.raises(oracle.NoHealthyChannel):
            oracle.rollback_plan(off, w, mb, ma, align)
        return
    plan = oracle.rollback_plan(off, w, mb, ma, align)
    for f in range(C):
        assert plan[f].tolist() == want.get(f, [0] * (C + 1)), f


def test_invariants_random(oracle):
    rng = np.random.default_rng(4242)
    done = 0
    while done < 1500:
        C = int(rng.integers(2, 17))
        w = [int(x) for x in rng.integers(0, 1000, size=C)]
        mb = int(rng.integers(0, 1 << C))
        ma = mb | int(rng.integers(0, 1 << C))
        align = int(rng.choice([16, 256, 4096]))
        nbytes = int(rng.integers(0, 1 << 26))
        if sum(0 if (mb >> c) & 1 else w[c] for c in range(C)) == 0:
            continue
        off = [int(x) for x in oracle.partition(w, mb, nbytes, align)]
        alive = [0 if (ma >> c) & 1 else w[c] for c in range(C)]
        W = sum(alive)
        newly = [f for f in range(C) if (ma >> f) & 1 and not (mb >> f) & 1 and off[f + 1] > off[f]]
        if W == 0 and newly:
            with pytest.raises(oracle.NoHealthyChannel):
                oracle.rollback_plan(off, w, mb, ma, align)
            done += 1
            continue
        plan = oracle.rollback_plan(off, w, mb, ma, align)
        moved = 0
        for f in range(C):
            row = [int(x) for x in plan[f]]
            if f not in newly:
                assert row == [0] * (C + 1)
                continue
            length = off[f + 1] - off[f]
            assert row[0] == 0 and row[C] == length
            assert all(row[c] <= row[c + 1] for c in range(C))
            U, tail = length // align, length % align
            last = max(c for c in range(C) if alive[c])
            for c in range(C):
                got = row[c + 1] - row[c]
                if alive[c] == 0:
                    assert got == 0  # nothing to a NIC that is down, the failed one included
                    continue
                if c == last:
                    got -= tail
                assert got % align == 0
                assert abs(Fraction(got, align) - Fraction(U * alive[c], W)) < 1
            moved += row[C]
        assert moved == sum(off[f + 1] - off[f] for f in newly)  # exactly the failed slices, once
        done += 1


def test_no_failure_no_plan(oracle):
    off = oracle.partition([1, 2, 3], 0, 6000, 16)
    assert not oracle.rollback_plan(off, [1, 2, 3], 0, 0, 16).any()
    assert not oracle.rollback_plan(off, [1, 2, 3], 0b010, 0b010, 16).any()


def test_single_survivor_takes_everything(oracle):
    """Hot repair (Sec. 5, opening paragraph): with one NIC left it carries the whole failed slice."""
    w = [5, 5, 5, 5]
    off = [int(x) for x in oracle.partition(w, 0, 1 << 20, 256)]
    plan = oracle.rollback_plan(off, w, 0, 0b1101, 256)  # only channel 1 survives
    for f in (0, 2, 3):
        length = off[f + 1] - off[f]
        assert plan[f].tolist() == [0, 0, length, length, length]
    assert not plan[1].any()


def test_recovery_is_rejected(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.rollback_plan([0, 16, 32], [1, 1], 0b01, 0b10, 16)  # channel 0 came back: not a rollback
