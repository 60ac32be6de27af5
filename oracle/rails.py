"""Oracle for a ring whose servers have lost different NICs (rails).

TEST INFRASTRUCTURE ONLY.  R2CCL paper, Sec. 6 ("Topology-Aware Logical Re-ranking": when node u
loses rail r and its neighbour v loses rail r', the bandwidth they share drops to the rails that
survive at both; re-ranking puts a bridge node between such neighbours) on top of the ring of
Sec. 5.2 and the proportional shares of Sec. 5.1.  Composed from this package's own partition and
reduce-copy; nothing is shared with the product.

Reading: the link from rank r to its ring successor carries every transmission of rank r over
the channels that are up at both ends, in proportion to their weights; the link's bandwidth is
the sum of those weights and the ring's is the smallest link's.  What the ring computes does not
depend on any of this: it is the all-reduce (or reduce-scatter / all-gather) of its definition.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import r2_oracle as o


def link_masks(fail_masks: Sequence[int]) -> List[int]:
    """Channels unusable on the link r -> r+1: down at either end."""
    R = len(fail_masks)
    return [fail_masks[r] | fail_masks[(r + 1) % R] for r in range(R)]


def link_bandwidth(weights: Sequence[int], fail_masks: Sequence[int]) -> List[int]:
    return [sum(int(w) for c, w in enumerate(weights) if not (m >> c) & 1) for m in link_masks(fail_masks)]


def ring_bandwidth(weights: Sequence[int], fail_masks: Sequence[int]) -> int:
    return min(link_bandwidth(weights, fail_masks))


def link_tables(weights: Sequence[int], fail_masks: Sequence[int], nbytes: int, align: int) -> np.ndarray:
    return np.stack([o.partition(weights, m, nbytes, align) for m in link_masks(fail_masks)])


def ring_rails_sim(bufs: Sequence[np.ndarray], dtype: int, n_slabs: int, n_channels: int, align: int,
                   weights: Sequence[int], fail_masks: Sequence[int], phases: int, stage_fill: int = 0xA5):
    """The ring step by step, in place on ``bufs`` (given in ring order): at step j rank r works on
    ring chunk (r - j) mod R [all-gather alone: (r + 1 - j) mod R], reads what rank r-1 staged at
    step j-1 with the table of the link r-1 -> r and stages onward with the table of its own link.
    Returns (tables[R, C+1], stage[2, R, S, C, cap])."""
    R, N = len(bufs), bufs[0].size
    assert N % (n_slabs * R) == 0
    E = N // (n_slabs * R)
    nbytes = E * bufs[0].itemsize
    cap = (max(nbytes, 1) + 255) // 256 * 256
    tables = link_tables(weights, fail_masks, nbytes, align)
    stage = np.full((2, R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    J = o.num_steps(R, phases)
    first = 1 if phases == o.PHASE_AG else 0
    for l in range(n_slabs):
        for j in range(J):
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
                o.reduce_copy(chunk, dtype, op, s_in, tables[peer] if j > 0 else None,
                              s_out, tables[r] if j < J - 1 else None, n_channels, cap)
                bufs[r][lo:lo + E] = chunk
    return tables, stage
