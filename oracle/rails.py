"""Oracle for a ring whose servers have lost different NICs (rails).

TEST INFRASTRUCTURE ONLY.  R2CCL paper, Sec. 6 ("Topology-Aware Logical Re-ranking": when node u
loses rail r and its neighbour v loses rail r', the bandwidth they share drops to the rails that
survive at both; re-ranking puts a bridge node between such neighbours) on top of the ring of
Sec. 5.2 and the proportional shares of Sec. 5.1.  Composed from this package's own partition and
reduce-copy; nothing is shared with the product.

Reading: every rank (a server) has a channel schedule of its own -- which of its NICs are down
from which transmission on, and how fast each is.  The link from rank r to its ring successor
carries a transmission of rank r over the channels that are up at both ends at that moment, in
proportion to the slower end's weight per channel; the link's bandwidth is the sum of those
weights and the ring's is the smallest link's.  What the ring computes does not depend on any of
this: it is the all-reduce (or reduce-scatter / all-gather) of its definition.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import r2_oracle as o
from .sendrecv import state_at


def link_masks(fail_masks: Sequence[int]) -> List[int]:
    """Channels unusable on the link r -> r+1: down at either end."""
    R = len(fail_masks)
    return [fail_masks[r] | fail_masks[(r + 1) % R] for r in range(R)]


def link_bandwidth(weights: Sequence[int], fail_masks: Sequence[int]) -> List[int]:
    return [sum(int(w) for c, w in enumerate(weights) if not (m >> c) & 1) for m in link_masks(fail_masks)]


def ring_bandwidth(weights: Sequence[int], fail_masks: Sequence[int]) -> int:
    return min(link_bandwidth(weights, fail_masks))


def static_epochs(weights: Sequence[int], fail_masks: Sequence[int]) -> List[List[o.Epoch]]:
    """Per-rank channel schedules for ranks whose state does not change during the run."""
    return [[(0, int(m), list(weights))] for m in fail_masks]


def link_state(rank_epochs: Sequence[Sequence[o.Epoch]], r: int, t: int):
    """(fail mask, weights) of the link r -> r+1 at transmission t: a channel is down if either end
    has it down, and as fast as the slower of its two ends."""
    R = len(rank_epochs)
    _, m0, w0 = state_at(rank_epochs[r], t)
    _, m1, w1 = state_at(rank_epochs[(r + 1) % R], t)
    return m0 | m1, [min(int(a), int(b)) for a, b in zip(w0, w1)]


def link_tables(rank_epochs: Sequence[Sequence[o.Epoch]], n_tx: int, nbytes: int, align: int) -> np.ndarray:
    """tables[r, t]: how the link r -> r+1 cuts transmission t."""
    R = len(rank_epochs)
    rows = []
    for r in range(R):
        for t in range(n_tx):
            mask, w = link_state(rank_epochs, r, t)
            rows.append(o.partition(w, mask, nbytes, align))
    return np.stack(rows).reshape(R, n_tx, -1)


def ring_rails_sim(bufs: Sequence[np.ndarray], dtype: int, n_slabs: int, n_channels: int, align: int,
                   rank_epochs: Sequence[Sequence[o.Epoch]], phases: int, stage_fill: int = 0xA5):
    """The ring step by step, in place on ``bufs`` (given in ring order): at step j of slab l rank r
    works on ring chunk (r - j) mod R [all-gather alone: (r + 1 - j) mod R], reads what rank r-1
    staged at step j-1 with the table of the link r-1 -> r for that transmission and stages onward
    with the table of its own link for transmission l*(J-1) + j.  Every rank has a channel schedule
    of its own (an epoch list over the transmission index).
    Returns (tables[R, S*(J-1), C+1], stage[2, R, S, C, cap])."""
    R, N = len(bufs), bufs[0].size
    assert N % (n_slabs * R) == 0
    E = N // (n_slabs * R)
    nbytes = E * bufs[0].itemsize
    cap = (max(nbytes, 1) + 255) // 256 * 256
    J = o.num_steps(R, phases)
    T = J - 1
    tables = link_tables(rank_epochs, n_slabs * T, nbytes, align)
    stage = np.full((2, R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    first = 1 if phases == o.PHASE_AG else 0
    for l in range(n_slabs):
        for j in range(J):
            t = l * T + j
            for r in range(R):
                c = (r + first - j) % R
                peer = (r - 1) % R
                lo = (l * R + c) * E
                chunk = np.ascontiguousarray(bufs[r][lo:lo + E])
                if phases == o.PHASE_AG:
                    op = o.OP_COPY
                elif phases == o.PHASE_RS:
                    op = o.OP_SUM
                else:
                    op = o.OP_SUM if j <= R - 1 else o.OP_COPY
                s_in = [stage[(j - 1) & 1, peer, l, k] for k in range(n_channels)] if j > 0 else None
                s_out = [stage[j & 1, r, l, k] for k in range(n_channels)] if j < J - 1 else None
                o.reduce_copy(chunk, dtype, op, s_in, tables[peer, t - 1] if j > 0 else None,
                              s_out, tables[r, t] if j < J - 1 else None, n_channels, cap)
                bufs[r][lo:lo + E] = chunk
    return tables, stage
