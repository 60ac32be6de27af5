"""Broadcast, Reduce and All-to-All under R2CCL-Balance (Sec. 5: table of strategies; Sec. 5.1
"Overhead Analysis"): pins for the oracle.  Each result has a plain definition that does not depend
on the channel schedule; the step-by-step oracle must reach it under any schedule, its stage slices
must be the data cut at the table, and failed channels must carry nothing."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as o
from oracle import collectives as col
from oracle.sendrecv import state_at


def _bufs(rng, R, N, dtype, ints=False):
    if ints:  # small integers: every partial sum is exact in fp32 and in bf16 (|sum| <= 64*3 < 256)
        vals = [rng.integers(-3, 4, N).astype(np.float32) for _ in range(R)]
    else:
        vals = [rng.standard_normal(N).astype(np.float32) for _ in range(R)]
    if dtype == o.F32:
        return vals
    return [torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy() for v in vals]


def _as_f64(x, dtype):
    if dtype == o.F32:
        return x.astype(np.float64)
    return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _schedule(rng, C, n_tx):
    w = [int(x) for x in rng.integers(1, 100, C)]
    epochs = [(0, int(rng.integers(0, (1 << C) - 1)), w)]
    for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, 3))):
        epochs.append((t, int(rng.integers(0, (1 << C) - 1)), [int(x) for x in rng.integers(1, 100, C)]))
    return epochs


def _check_stage(log, stage_of, chunk_of, epochs, nbytes, C, align):
    """log rows follow the epoch in force; slices reassemble to the chunk; the rest is untouched."""
    for t in range(log.shape[0]):
        _, mask, ws = state_at(epochs, t)
        assert log[t].tolist() == o.partition(ws, mask, nbytes, align).tolist()
        for c in range(C):
            if (mask >> c) & 1:
                assert log[t][c + 1] == log[t][c]
    for (t, bufs), raw in zip(stage_of, chunk_of):
        got = b"".join(bufs[c][: int(log[t][c + 1] - log[t][c])].tobytes() for c in range(C))
        assert got == raw


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_broadcast_everyone_gets_the_roots_bytes(dtype):
    rng = np.random.default_rng(21)
    for _ in range(25):
        R, S, C = int(rng.integers(2, 7)), int(rng.integers(1, 5)), int(rng.integers(1, 7))
        E, root = int(rng.integers(1, 150)), int(rng.integers(0, R))
        epochs = _schedule(rng, C, S * (R - 1))
        bufs = _bufs(rng, R, S * E, dtype)
        keep = [b.copy() for b in bufs]
        log, stage = col.broadcast_sim(bufs, dtype, root, S, C, 16, epochs)
        for r in range(R):
            assert bufs[r].tobytes() == keep[root].tobytes()
        assert [b.tobytes() for b in col.broadcast_expected(keep, root)] == [keep[root].tobytes()] * R
        # every hop carries the root's chunk; the last rank of the chain stages nothing
        stages, chunks = [], []
        for l in range(S):
            for j in range(R - 1):
                r = (root + j) % R
                stages.append((l * (R - 1) + j, [stage[j & 1, r, l, c] for c in range(C)]))
                chunks.append(keep[root][l * E:(l + 1) * E].tobytes())
        _check_stage(log, stages, chunks, epochs, E * bufs[0].itemsize, C, 16)
        last = (root + R - 1) % R
        assert np.all(stage[:, last] == 0xA5)


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_reduce_root_gets_the_fold_and_nobody_else_changes(dtype):
    rng = np.random.default_rng(22)
    for _ in range(25):
        R, S, C = int(rng.integers(2, 7)), int(rng.integers(1, 5)), int(rng.integers(1, 7))
        E, root = int(rng.integers(1, 150)), int(rng.integers(0, R))
        epochs = _schedule(rng, C, S * (R - 1))
        bufs = _bufs(rng, R, S * E, dtype)
        keep = [b.copy() for b in bufs]
        col.reduce_sim(bufs, dtype, root, S, C, 16, epochs)
        want = col.reduce_expected(keep, dtype, root)
        for r in range(R):
            assert bufs[r].tobytes() == want[r].tobytes()
            if r != root:
                assert bufs[r].tobytes() == keep[r].tobytes()
        # an independent fold in the chain's order with torch's rounding
        tt = torch.float32 if dtype == o.F32 else torch.bfloat16
        as_t = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).view(tt)
        acc = as_t(keep[(root + 1) % R]).clone()
        for k in range(2, R + 1):
            acc = (acc.float() + as_t(keep[(root + k) % R]).float()).to(tt)
        raw = acc.view(torch.int16).numpy().tobytes() if dtype == o.BF16 else acc.numpy().tobytes()
        assert bufs[root].tobytes() == raw
        # and within R-1 roundings of the exact sum
        exact = sum(_as_f64(k, dtype) for k in keep)
        bound = (R - 1) * 2.0 ** (-24 if dtype == o.F32 else -8) * sum(np.abs(_as_f64(k, dtype)) for k in keep)
        assert np.all(np.abs(_as_f64(bufs[root], dtype) - exact) <= bound * 1.01 + 1e-30)


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_reduce_of_small_integers_is_exact_and_matches_the_ring_allreduce(dtype):
    """Integer data sums exactly in any order, so the reduce (chain order), the ring all-reduce (ring
    order per chunk) and Python's integers must agree; a broadcast of the reduced buffer then gives
    every rank what the all-reduce gives it."""
    rng = np.random.default_rng(23)
    for R in (2, 3, 5, 8):
        S, C, E, root = 2, 4, 8 * R, int(rng.integers(0, R))
        bufs = _bufs(rng, R, S * E, dtype, ints=True)
        keep = [b.copy() for b in bufs]
        total = sum(_as_f64(k, dtype) for k in keep)
        col.reduce_sim(bufs, dtype, root, S, C, 16, [(0, 0b0010, [5, 7, 9, 11])])
        assert np.array_equal(_as_f64(bufs[root], dtype), total)
        col.broadcast_sim(bufs, dtype, root, S, C, 16, [(0, 0b0100, [5, 7, 9, 11]), (2, 0, [1, 1, 1, 1])])
        ring = o.expected(keep, dtype, S, o.PHASE_AR)
        for r in range(R):
            assert bufs[r].tobytes() == ring[r].tobytes()


def test_reduce_two_ranks_is_one_addition():
    x = [np.array([1.5, -2.25, 1e-8, 3e38], np.float32), np.array([0.25, 2.25, 1.0, 3e38], np.float32)]
    keep = [b.copy() for b in x]
    col.reduce_sim(x, o.F32, 0, 1, 2, 16, [(0, 0, [1, 1])])
    with np.errstate(over="ignore"):
        assert x[0].tolist() == (keep[0] + keep[1]).tolist()  # incl. the overflow to inf
    assert x[1].tolist() == keep[1].tolist()


def test_reduce_stage_carries_the_running_sum():
    """The hop rank root+1+j sends is the fold of the first j+1 ranks of the chain, cut at the table."""
    rng = np.random.default_rng(24)
    R, S, C, E, root = 5, 3, 4, 40, 3
    epochs = [(0, 0b0001, [3, 1, 4, 1]), (5, 0b1010, [3, 1, 4, 1]), (9, 0, [2, 7, 1, 8])]
    bufs = _bufs(rng, R, S * E, o.BF16)
    keep = [b.copy() for b in bufs]
    log, stage = col.reduce_sim(bufs, o.BF16, root, S, C, 16, epochs)
    stages, chunks = [], []
    for l in range(S):
        acc = keep[(root + 1) % R][l * E:(l + 1) * E].copy()
        for j in range(R - 1):
            r = (root + 1 + j) % R
            if j:
                acc = col._add(acc, keep[r][l * E:(l + 1) * E], o.BF16)
            stages.append((l * (R - 1) + j, [stage[j & 1, r, l, c] for c in range(C)]))
            chunks.append(acc.tobytes())
    _check_stage(log, stages, chunks, epochs, E * 2, C, 16)
    assert np.all(stage[:, root] == 0xA5)  # the root sends nothing


@pytest.mark.parametrize("dtype", [o.F32, o.BF16])
def test_alltoall_is_a_block_transpose(dtype):
    rng = np.random.default_rng(25)
    for _ in range(20):
        R, S, C = int(rng.integers(2, 7)), int(rng.integers(1, 4)), int(rng.integers(1, 7))
        E = int(rng.integers(1, 60))
        B = S * E
        epochs = _schedule(rng, C, (R - 1) * S)
        send = _bufs(rng, R, R * B, dtype)
        keep = [b.copy() for b in send]
        recv = [np.zeros_like(b) for b in send]
        log, stage = col.alltoall_sim(send, recv, dtype, S, C, 16, epochs)
        want = col.alltoall_expected(keep)
        for r in range(R):
            assert send[r].tobytes() == keep[r].tobytes()  # send buffers are only read
            assert recv[r].tobytes() == want[r].tobytes()
            for q in range(R):  # the definition, block by block
                assert recv[r][q * B:(q + 1) * B].tobytes() == keep[q][r * B:(r + 1) * B].tobytes()
        # twice is the identity
        back = [np.zeros_like(b) for b in send]
        col.alltoall_sim(recv, back, dtype, S, C, 16, epochs)
        for r in range(R):
            assert back[r].tobytes() == keep[r].tobytes()
        stages, chunks = [], []
        for k in range(1, R):
            for l in range(S):
                t = (k - 1) * S + l
                for r in range(R):
                    dst = (r + k) % R
                    stages.append((t, [stage[r, t, c] for c in range(C)]))
                    chunks.append(keep[r][dst * B + l * E: dst * B + (l + 1) * E].tobytes())
        _check_stage(log, stages, chunks, epochs, E * send[0].itemsize, C, 16)


def test_alltoall_two_ranks_by_hand():
    send = [np.array([10, 11, 12, 13], np.float32), np.array([20, 21, 22, 23], np.float32)]
    recv = [np.zeros(4, np.float32), np.zeros(4, np.float32)]
    log, _ = col.alltoall_sim(send, recv, o.F32, 1, 2, 16, [(0, 0b01, [1, 1])])
    assert recv[0].tolist() == [10, 11, 20, 21]
    assert recv[1].tolist() == [12, 13, 22, 23]
    assert log.tolist() == [[0, 0, 8]]  # one transmission of 8 bytes, all on channel 1


def test_balance_keeps_the_volume_and_shares_it_in_proportion():
    """Sec. 5.1: the bytes a rank must send do not change with a failure; they are spread over the
    healthy NICs in proportion to bandwidth (within one alignment unit per channel)."""
    R, S, C, E = 4, 1, 4, 4096
    w = [50, 25, 100, 25]
    for mask in (0, 0b0001, 0b0110):
        bufs = [np.full(E, r, np.float32) for r in range(R)]
        log, _ = col.broadcast_sim(bufs, o.F32, 1, S, C, 256, [(0, mask, w)])
        alive = sum(x for c, x in enumerate(w) if not (mask >> c) & 1)
        for row in log:
            assert row[-1] == E * 4
            for c in range(C):
                share = Fraction(0) if (mask >> c) & 1 else Fraction(w[c] * E * 4, alive)
                assert abs(Fraction(int(row[c + 1] - row[c])) - share) <= 256
