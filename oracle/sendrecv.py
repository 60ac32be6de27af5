"""Oracle for point-to-point transfers under R2CCL-Balance (Sec. 5.1; Sec. 8 and Appendix E measure
SendRecv).  TEST INFRASTRUCTURE ONLY; composed from this package's own partition and reduce-copy.

Every rank sends its buffer to its ring successor in ``n_slabs`` message chunks; chunk l is
transmission l and is cut over the channels by the state in force then.  By definition the receiver
ends up with the sender's bytes, whatever the channel schedule.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import r2_oracle as o


def state_at(epochs: Sequence[o.Epoch], t: int):
    """The last epoch whose t_start is <= t."""
    cur = epochs[0]
    for e in epochs:
        if e[0] <= t:
            cur = e
    return cur


def sendrecv_expected(send: Sequence[np.ndarray]) -> List[np.ndarray]:
    R = len(send)
    return [send[(r - 1) % R].copy() for r in range(R)]


def sendrecv_sim(send: Sequence[np.ndarray], recv: Sequence[np.ndarray], dtype: int, n_slabs: int,
                 n_channels: int, align: int, epochs: Sequence[o.Epoch], stage_fill: int = 0xA5):
    """Chunk by chunk: the sender stages its chunk under the table of transmission l, the receiver
    copies it out with the same table.  Returns (offsets_log[S, C+1], stage[R, S, C, cap])."""
    R = len(send)
    N = send[0].size
    assert N % n_slabs == 0
    E = N // n_slabs
    nbytes = E * send[0].itemsize
    cap = (max(nbytes, 1) + 255) // 256 * 256
    log = np.zeros((n_slabs, n_channels + 1), dtype=np.uint64)
    stage = np.full((R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    for l in range(n_slabs):
        _, mask, weights = state_at(epochs, l)
        table = o.partition(weights, mask, nbytes, align)
        log[l] = table
        for r in range(R):
            chunk = np.ascontiguousarray(send[r][l * E:(l + 1) * E])
            bufs = [stage[r, l, c] for c in range(n_channels)]
            o.reduce_copy(chunk, dtype, o.OP_SUM, None, None, bufs, table, n_channels, cap)
        for r in range(R):
            out = np.empty(E, dtype=send[0].dtype)
            bufs = [stage[(r - 1) % R, l, c] for c in range(n_channels)]
            o.reduce_copy(out, dtype, o.OP_COPY, bufs, table, None, None, n_channels, cap)
            recv[r][l * E:(l + 1) * E] = out
    return log, stage
