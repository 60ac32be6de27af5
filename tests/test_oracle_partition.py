"""Pins for the oracle's channel partition (CPU only).

The paper (Sec. 5.1, R2CCL-Balance and "Overhead Analysis"; Appendix C for the
"one healthy NIC must remain" boundary) fixes what a partition must satisfy:
healthy NICs only, shares proportional to bandwidth, volumes unchanged.  Each
test below checks the oracle against something that is not the oracle: worked
examples, invariants, exact rational arithmetic, brute force written in a
different shape, and textbook special cases.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "partition_cases.txt")


def _golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, w, mask, nbytes, align, off = [s.strip() for s in line.split("|")]
            cases.append((name, [int(x) for x in w.split()], int(mask, 16), int(nbytes), int(align),
                          [int(x) for x in off.split()]))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_worked_examples(oracle, case):
    _, w, mask, nbytes, align, want = case
    got = oracle.partition(w, mask, nbytes, align)
    assert got.tolist() == want


def _alive(w, mask):
    return [0 if (mask >> c) & 1 else int(w[c]) for c in range(len(w))]


def _check_invariants(off, w, mask, nbytes, align):
    C = len(w)
    e = _alive(w, mask)
    W = sum(e)
    off = [int(x) for x in off]
    # coverage: every byte in exactly one slice (volumes unchanged)
    assert off[0] == 0 and off[C] == nbytes
    assert all(off[c] <= off[c + 1] for c in range(C))
    # nothing is routed to a failed (or zero-bandwidth) channel
    for c in range(C):
        if e[c] == 0:
            assert off[c + 1] == off[c]
    # interior boundaries are whole alignment units
    for c in range(1, C):
        assert off[c] % align == 0 or off[c] == nbytes
    # proportionality: each healthy channel is within one unit of its exact share
    U = nbytes // align
    tail = nbytes - U * align
    last_alive = max(c for c in range(C) if e[c])
    for c in range(C):
        length = off[c + 1] - off[c]
        if c == last_alive:
            length -= tail
        assert length % align == 0
        exact_units = Fraction(U * e[c], W)
        assert abs(Fraction(length, align) - exact_units) < 1


def test_invariants_random(oracle):
    rng = np.random.default_rng(20251)
    for _ in range(3000):
        C = int(rng.integers(1, 65))
        kind = rng.integers(0, 3)
        if kind == 0:
            w = rng.integers(0, 5, size=C)
        elif kind == 1:
            w = rng.integers(1, 400001, size=C)
        else:
            w = rng.integers(0, 2 ** 32, size=C, dtype=np.uint64)
        mask = int(rng.integers(0, 2 ** 63)) & ((1 << C) - 1)
        if rng.integers(0, 4) == 0:
            mask = 0
        align = int(rng.choice([1, 2, 4, 16, 256, 4096]))
        nbytes = int(rng.choice([0, 1, 100, 2 ** 20, 2 ** 24 + 48, int(rng.integers(0, 2 ** 40))]))
        if sum(_alive(w, mask)) == 0:
            with pytest.raises(oracle.NoHealthyChannel):
                oracle.partition(w, mask, nbytes, align)
            continue
        off = oracle.partition(w, mask, nbytes, align)
        _check_invariants(off, w, mask, nbytes, align)


def test_huge_values_no_overflow(oracle):
    """64 channels at the largest weight and a byte count near 2^64: exact arithmetic must hold."""
    C = 64
    w = [2 ** 32 - 1] * C
    nbytes = 2 ** 64 - 1 - 255
    off = oracle.partition(w, 0, nbytes, 256)
    U = nbytes // 256
    for c in range(C):
        assert int(off[c]) == 256 * ((U * c) // C)
    assert int(off[C]) == nbytes


def _unit_owner_bruteforce(w, mask, U):
    """Unit u belongs to the channel whose cumulative-share interval (P_c/W, P_{c+1}/W]
    contains the unit's right edge (u+1)/U -- exact rationals, one unit at a time."""
    e = _alive(w, mask)
    W = sum(e)
    owners = []
    for u in range(U):
        edge = Fraction(u + 1, U)
        lo = Fraction(0)
        owner = None
        for c in range(len(e)):
            hi = lo + Fraction(e[c], W)
            if lo < edge <= hi:
                owner = c
                break
            lo = hi
        assert owner is not None
        owners.append(owner)
    return owners


def test_bruteforce_all_tiny(oracle):
    """Every weight vector in {0..3}^C, every mask, C <= 4, U <= 12 (+ a ragged tail)."""
    align = 4
    for C in range(1, 5):
        for w in itertools.product(range(4), repeat=C):
            for mask in range(1 << C):
                e = _alive(w, mask)
                if sum(e) == 0:
                    with pytest.raises(oracle.NoHealthyChannel):
                        oracle.partition(w, mask, 8, align)
                    continue
                for U in (0, 1, 2, 3, 5, 8, 12):
                    for tail in (0, 3):
                        nbytes = U * align + tail
                        off = [int(x) for x in oracle.partition(w, mask, nbytes, align)]
                        owners = _unit_owner_bruteforce(w, mask, U)
                        last_alive = max(c for c in range(C) if e[c])
                        want_len = [owners.count(c) * align for c in range(C)]
                        want_len[last_alive] += tail
                        got_len = [off[c + 1] - off[c] for c in range(C)]
                        assert got_len == want_len, (w, mask, U, tail)
                        # units are handed out in channel order
                        assert owners == sorted(owners)
                        assert off[0] == 0 and off[C] == nbytes


def test_equal_split_textbook(oracle):
    """Equal bandwidth, no failure, size divisible: the plain even split."""
    for C in (1, 2, 4, 8, 64):
        nbytes = 256 * C * 37
        off = oracle.partition([50000] * C, 0, nbytes, 256)
        assert off.tolist() == [c * (nbytes // C) for c in range(C + 1)]


def test_failed_share_redistributed_in_proportion(oracle):
    """Sec. 5.1 says the failed NIC's portion is spread over the healthy NICs in
    proportion to their bandwidth.  Starting from the no-failure shares w_c/W_all and
    adding to each survivor its proportional part of the failed share must give,
    within one alignment unit, the slice lengths the oracle produces."""
    rng = np.random.default_rng(7)
    for _ in range(300):
        C = int(rng.integers(2, 9))
        w = [int(x) for x in rng.integers(1, 100001, size=C)]
        f = int(rng.integers(0, C))
        U = int(rng.integers(C, 100000))
        align = 256
        off = [int(x) for x in oracle.partition(w, 1 << f, U * align, align)]
        W_all = sum(w)
        W_rem = W_all - w[f]
        for c in range(C):
            units = Fraction(off[c + 1] - off[c], align)
            if c == f:
                assert units == 0
                continue
            share = Fraction(w[c], W_all) + Fraction(w[f], W_all) * Fraction(w[c], W_rem)
            assert abs(units - U * share) < 1


def test_scale_invariance_of_weights(oracle):
    """Only bandwidth ratios matter: multiplying every weight by k changes nothing."""
    rng = np.random.default_rng(11)
    for _ in range(200):
        C = int(rng.integers(1, 17))
        w = rng.integers(0, 1000, size=C)
        mask = int(rng.integers(0, 1 << C))
        if sum(_alive(w, mask)) == 0:
            continue
        nbytes = int(rng.integers(0, 2 ** 30))
        a = oracle.partition(w, mask, nbytes, 256)
        b = oracle.partition(w * 4093, mask, nbytes, 256)
        assert a.tolist() == b.tolist()


def test_failed_equals_zero_weight(oracle):
    """A failed channel and a zero-bandwidth channel are the same thing to the split."""
    rng = np.random.default_rng(13)
    for _ in range(200):
        C = int(rng.integers(1, 17))
        w = rng.integers(1, 1000, size=C)
        mask = int(rng.integers(0, (1 << C) - 1))
        wz = w.copy()
        for c in range(C):
            if (mask >> c) & 1:
                wz[c] = 0
        nbytes = int(rng.integers(0, 2 ** 30))
        assert oracle.partition(w, mask, nbytes, 256).tolist() == oracle.partition(wz, 0, nbytes, 256).tolist()


def test_invalid_arguments(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.partition([1, 2], 0, 100, 0)  # align 0
    with pytest.raises(oracle.OracleError):
        oracle.partition([1] * 65, 0, 100, 16)  # too many channels
