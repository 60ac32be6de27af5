"""Oracle for the other collectives R2CCL-Balance covers: Broadcast, Reduce and All-to-All.

TEST INFRASTRUCTURE ONLY.  R2CCL paper, Sec. 5 (the table of strategies: Balance serves
ReduceScatter, AllGather, Broadcast, Reduce and point-to-point incl. All-to-All) and Sec. 5.1
("Overhead Analysis": the collective's own schedule is kept -- in a ring Broadcast the root sends
the whole buffer and every other rank receives it -- and only the cut of each transmission over
the healthy NICs changes).  Composed from this package's own partition and reduce-copy; nothing is
shared with the product.

What each computes has a plain definition, written out in the ``*_expected`` functions:
  broadcast   every rank ends with the root's bytes;
  reduce      the root ends with the left fold x_{root+1} + x_{root+2} + ... + x_{root} taken along
              the ring (the chain that ends at the root), rounded to the buffer type after every
              addition; all other buffers are unchanged;
  all-to-all  block q of rank r's receive buffer is block r of rank q's send buffer.
The ``*_sim`` functions take the steps one by one with explicit stage buffers: a rank buffer is S
message chunks (all-to-all: R blocks of S chunks), every hop of every chunk is one transmission,
cut by the channel state in force at its index.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import r2_oracle as o
from .sendrecv import state_at


def _cap(nbytes: int) -> int:
    return (max(nbytes, 1) + 255) // 256 * 256


# ------------------------------------------------------------------ broadcast

def broadcast_expected(bufs: Sequence[np.ndarray], root: int) -> List[np.ndarray]:
    return [bufs[root].copy() for _ in bufs]


def broadcast_sim(bufs: Sequence[np.ndarray], dtype: int, root: int, n_slabs: int, n_channels: int,
                  align: int, epochs: Sequence[o.Epoch], stage_fill: int = 0xA5):
    """Ring broadcast, in place: chunk l travels root -> root+1 -> ... -> root+R-1; the hop that
    rank root+j sends is transmission l*(R-1) + j and uses stage parity j & 1.
    Returns (offsets_log[S*(R-1), C+1], stage[2, R, S, C, cap])."""
    R, N = len(bufs), bufs[0].size
    assert N % n_slabs == 0
    E = N // n_slabs
    nbytes = E * bufs[0].itemsize
    cap = _cap(nbytes)
    log = np.zeros((n_slabs * (R - 1), n_channels + 1), dtype=np.uint64)
    stage = np.full((2, R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    for l in range(n_slabs):
        for j in range(R):
            r = (root + j) % R
            t = l * (R - 1) + j
            chunk = np.ascontiguousarray(bufs[r][l * E:(l + 1) * E])
            s_in = t_in = s_out = t_out = None
            if j > 0:
                s_in = [stage[(j - 1) & 1, (r - 1) % R, l, c] for c in range(n_channels)]
                t_in = log[t - 1]
            if j < R - 1:
                _, mask, weights = state_at(epochs, t)
                log[t] = o.partition(weights, mask, nbytes, align)
                s_out = [stage[j & 1, r, l, c] for c in range(n_channels)]
                t_out = log[t]
            o.reduce_copy(chunk, dtype, o.OP_COPY, s_in, t_in, s_out, t_out, n_channels, cap)
            bufs[r][l * E:(l + 1) * E] = chunk
    return log, stage


# ------------------------------------------------------------------ reduce

def _add(a: np.ndarray, b: np.ndarray, dtype: int) -> np.ndarray:
    """One hop of the reduction: a + b in fp32, rounded to the buffer type."""
    if dtype == o.F32:
        return (a + b).astype(np.float32)
    wa = (a.astype(np.uint32) << 16).view(np.float32)
    wb = (b.astype(np.uint32) << 16).view(np.float32)
    s = (wa + wb).astype(np.float32)
    return np.array([o.f32_to_bf16(float(v)) for v in s], dtype=np.uint16)


def reduce_expected(bufs: Sequence[np.ndarray], dtype: int, root: int) -> List[np.ndarray]:
    R = len(bufs)
    outs = [b.copy() for b in bufs]
    acc = bufs[(root + 1) % R].copy()
    for k in range(2, R + 1):
        acc = _add(acc, bufs[(root + k) % R], dtype)
    outs[root] = acc
    return outs


def reduce_sim(bufs: Sequence[np.ndarray], dtype: int, root: int, n_slabs: int, n_channels: int,
               align: int, epochs: Sequence[o.Epoch], stage_fill: int = 0xA5):
    """Ring reduce towards the root, in place on the root's buffer only: rank root+1 sends chunk l,
    every rank after it sends on (incoming + its own chunk) and keeps its own buffer as it was, the
    root adds the last incoming into its buffer.  The hop sent at step j (by rank root+1+j) is
    transmission l*(R-1) + j, stage parity j & 1.
    Returns (offsets_log[S*(R-1), C+1], stage[2, R, S, C, cap])."""
    R, N = len(bufs), bufs[0].size
    assert N % n_slabs == 0
    E = N // n_slabs
    nbytes = E * bufs[0].itemsize
    cap = _cap(nbytes)
    log = np.zeros((n_slabs * (R - 1), n_channels + 1), dtype=np.uint64)
    stage = np.full((2, R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    for l in range(n_slabs):
        for j in range(R):
            r = (root + 1 + j) % R
            t = l * (R - 1) + j
            own = np.ascontiguousarray(bufs[r][l * E:(l + 1) * E])
            s_in = t_in = s_out = t_out = None
            if j > 0:
                s_in = [stage[(j - 1) & 1, (r - 1) % R, l, c] for c in range(n_channels)]
                t_in = log[t - 1]
            if j < R - 1:
                _, mask, weights = state_at(epochs, t)
                log[t] = o.partition(weights, mask, nbytes, align)
                s_out = [stage[j & 1, r, l, c] for c in range(n_channels)]
                t_out = log[t]
            work = own.copy()  # a rank that passes the sum on does not keep it
            o.reduce_copy(work, dtype, o.OP_SUM, s_in, t_in, s_out, t_out, n_channels, cap)
            if j == R - 1:
                bufs[r][l * E:(l + 1) * E] = work
    return log, stage


# ------------------------------------------------------------------ all-to-all

def alltoall_expected(send: Sequence[np.ndarray]) -> List[np.ndarray]:
    R = len(send)
    B = send[0].size // R
    outs = []
    for r in range(R):
        outs.append(np.concatenate([send[q][r * B:(r + 1) * B] for q in range(R)]))
    return outs


def alltoall_sim(send: Sequence[np.ndarray], recv: Sequence[np.ndarray], dtype: int, n_slabs: int,
                 n_channels: int, align: int, epochs: Sequence[o.Epoch], stage_fill: int = 0xA5):
    """Pairwise exchange in R-1 rounds: in round k = 1..R-1 rank r sends its block for rank r+k, in
    S chunks, and receives rank r-k's block for it; chunk l of round k is transmission
    (k-1)*S + l, the same for every rank.  A rank's own block is copied without touching a
    channel.  Returns (offsets_log[(R-1)*S, C+1], stage[R, (R-1)*S, C, cap])."""
    R, N = len(send), send[0].size
    assert N % (R * n_slabs) == 0
    B = N // R
    E = B // n_slabs
    nbytes = E * send[0].itemsize
    cap = _cap(nbytes)
    n_tx = (R - 1) * n_slabs
    log = np.zeros((n_tx, n_channels + 1), dtype=np.uint64)
    stage = np.full((R, n_tx, n_channels, cap), stage_fill, dtype=np.uint8)
    for r in range(R):
        recv[r][r * B:(r + 1) * B] = send[r][r * B:(r + 1) * B]
    for k in range(1, R):
        for l in range(n_slabs):
            t = (k - 1) * n_slabs + l
            _, mask, weights = state_at(epochs, t)
            log[t] = o.partition(weights, mask, nbytes, align)
            for r in range(R):
                dst = (r + k) % R
                chunk = np.ascontiguousarray(send[r][dst * B + l * E: dst * B + (l + 1) * E])
                bufs = [stage[r, t, c] for c in range(n_channels)]
                o.reduce_copy(chunk, dtype, o.OP_SUM, None, None, bufs, log[t], n_channels, cap)
            for r in range(R):
                src = (r - k) % R
                out = np.empty(E, dtype=send[0].dtype)
                bufs = [stage[src, t, c] for c in range(n_channels)]
                o.reduce_copy(out, dtype, o.OP_COPY, bufs, log[t], None, None, n_channels, cap)
                recv[r][src * B + l * E: src * B + (l + 1) * E] = out
    return log, stage
