"""Oracle for a ring run in which a channel fails while a transmission is in flight.

TEST INFRASTRUCTURE ONLY; composed from this package's own ring and failover plan.

R2CCL paper, Sec. 4.3, Technique II: a failure may strike in the middle of a chunk transfer.  Send
buffers stay intact until completion and every NIC is registered on every buffer (Technique I), so
the sender rewinds to the first chunk without a completion and retransmits it over the NICs that are
left; chunks already completed are untouched and later chunks use the new state (Sec. 5.1).

In the run's terms: an epoch (t_start = k, fail_mask, weights) marked "in flight" says that its
failures strike during transmission k, not before it.  Then
  * transmission k was staged with the table of the state in force before the epoch (the epoch
    before it in the list) and stays staged that way: the receiver's layout does not change;
  * the slices of the channels that newly failed are re-carried by the channels still healthy, shared
    out by the failover plan (the epoch's weights and mask; same alignment);
  * transmissions after k are cut by the epoch's own state, as for an ordinary epoch.
Readings: an in-flight epoch only adds failures to the state before it (recoveries are found by
re-probing between transmissions, Sec. 4.2, and come as ordinary epochs); the first epoch cannot be in
flight (there is no table before it); an in-flight epoch that starts beyond the run has no effect.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import r2_oracle as o


def table_epochs(epochs: Sequence[o.Epoch], in_flight: Sequence[bool]) -> List[o.Epoch]:
    """The epoch list as the tables see it: an in-flight epoch governs from the transmission after the
    one it strikes in; an epoch that another one overtakes that way never governs a table."""
    assert len(epochs) == len(in_flight) and not in_flight[0]
    shifted = [(t0 + 1 if fl else t0, mask, w) for (t0, mask, w), fl in zip(epochs, in_flight)]
    return [e for i, e in enumerate(shifted) if i + 1 == len(shifted) or e[0] < shifted[i + 1][0]]


def ring_sim_inflight(bufs: Sequence[np.ndarray], dtype: int, n_slabs: int, n_channels: int, align: int,
                      epochs: Sequence[o.Epoch], in_flight: Sequence[bool], phases: int,
                      cap: Optional[int] = None, stage_fill: int = 0xA5):
    """The ring step by step, in place on ``bufs``, with failures in flight.

    Returns ``(offsets_log, stage, plans)``: the first two as ``ring_sim``; ``plans[i]`` is the
    failover plan [C, C+1] of in-flight epoch i (only epochs that are in flight and strike within the
    run have an entry)."""
    for i, fl in enumerate(in_flight):
        if fl and (epochs[i - 1][1] & ~epochs[i][1]):
            raise o.OracleError(-1, "an in-flight epoch may only add failures")
    log, stage = o.ring_sim(bufs, dtype, n_slabs, n_channels, align, table_epochs(epochs, in_flight), phases,
                            cap=cap, stage_fill=stage_fill)
    plans: Dict[int, np.ndarray] = {}
    for i, fl in enumerate(in_flight):
        k = epochs[i][0]
        if fl and k < log.shape[0]:
            plans[i] = o.rollback_plan(log[k], epochs[i][2], epochs[i - 1][1], epochs[i][1], align)
    return log, stage, plans
