"""Oracle for R2CCL-AllReduce: the planner's closed forms and the split schedule.

TEST INFRASTRUCTURE ONLY.  Follows the R2CCL paper, Sec. 5.2 (partial all-reduce, the two-stage
R2CCL-AllReduce, "Data Partition Analysis") and Appendix A (optimal share Y*, threshold on the lost
bandwidth X).  The schedule is composed from this package's own ring and reduce-copy; nothing is
shared with the product.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import r2_oracle as o


# ------------------------------------------------------------------ planner (Sec. 5.2, Appendix A)

def ring_factor(p: int) -> Fraction:
    """Ring all-reduce over p participants moves 2(p-1)/p of the data per participant."""
    return Fraction(2 * (p - 1), p)


def completion_time(n: int, g: int, X, Y):
    """T(Y) = max(T1, T2) + T3 with B = D = 1 (Sec. 5.2, Data Partition Analysis)."""
    a, b = ring_factor(n * g), ring_factor((n - 1) * g)
    t1 = a * (1 - Y) / (1 - X)      # global all-reduce, throttled to (1-X)B
    t2 = b * Y / X                  # partial all-reduce among the healthy servers
    t3 = Y / X                      # the broadcast
    return max(t1, t2) + t3


def balance_point(n: int, g: int, X) -> Fraction:
    """The Y at which global and partial all-reduce take equally long (T1 = T2), solved exactly."""
    a, b = ring_factor(n * g), ring_factor((n - 1) * g)
    X = Fraction(X)
    return a * X / (a * X + b * (1 - X))


def y_star_paper(n: int, g: int, X) -> Fraction:
    """The closed form as printed in Appendix A, Step 1 / Step 3."""
    X = Fraction(X)
    return X + X * (1 - X) / (X + (g * (n - 1) - 1) * n)


def threshold(n: int, g: int) -> Fraction:
    """Lost-bandwidth fraction above which splitting beats the plain ring (Appendix A, Step 2)."""
    return Fraction(n * g, 3 * n * g - 2)


def degraded_server_volume(Y):
    """Data the degraded server sends (or receives), in units of D: about 2(1-Y) in the global
    all-reduce plus Y in the broadcast (Fig. 4's caption: 2D becomes 1.75D for Y = 1/4)."""
    return 2 * (1 - Y) + Y


# ------------------------------------------------------------------ schedule

def split_expected(inputs: Sequence[np.ndarray], dtype: int, d: int, n_partial: int,
                   slabs_global: int, slabs_partial: int) -> List[np.ndarray]:
    """What every rank must hold afterwards, by definition: the head is the ring all-reduce of all
    ranks; the tail is the ring all-reduce of the healthy ranks (in ring order after d) plus the
    degraded rank's own tail, rounded to the buffer type after every addition."""
    R = len(inputs)
    N = inputs[0].size
    ng = N - n_partial
    outs = [x.copy() for x in inputs]
    if ng:
        head = o.expected([np.ascontiguousarray(x[:ng]) for x in inputs], dtype, slabs_global, o.PHASE_AR)
        for r in range(R):
            outs[r][:ng] = head[r]
    if n_partial:
        order = [(d + 1 + i) % R for i in range(R - 1)]
        tails = o.expected([np.ascontiguousarray(inputs[r][ng:]) for r in order], dtype, slabs_partial, o.PHASE_AR)
        xd = np.ascontiguousarray(inputs[d][ng:])
        total = _add(tails[0], xd, dtype)
        for r in range(R):
            outs[r][ng:] = total
    return outs


def _add(a: np.ndarray, b: np.ndarray, dtype: int) -> np.ndarray:
    """a + b in fp32, rounded to the buffer type: one hop of the reduction."""
    if dtype == o.F32:
        return (a + b).astype(np.float32)
    wa = (a.astype(np.uint32) << 16).view(np.float32)
    wb = (b.astype(np.uint32) << 16).view(np.float32)
    s = (wa + wb).astype(np.float32)
    return np.array([o.f32_to_bf16(float(v)) for v in s], dtype=np.uint16)


def split_sim(bufs: Sequence[np.ndarray], dtype: int, d: int, n_partial: int, slabs_global: int,
              slabs_partial: int, n_channels: int, align: int, weights: Sequence[int],
              degraded_mask: int, ring_logs: Optional[dict] = None) -> Tuple[np.ndarray, List[np.ndarray]]:
    """The schedule step by step, in place on ``bufs``.  Returns the two broadcast tables and the
    final contents of the two broadcast stage parities (C buffers each).  ``ring_logs``, if given,
    receives the table of every transmission of the two rings under "global" and "partial"."""
    R = len(bufs)
    N = bufs[0].size
    ng = N - n_partial
    es = bufs[0].itemsize
    if ng:
        heads = [np.ascontiguousarray(b[:ng]) for b in bufs]
        log, _ = o.ring_sim(heads, dtype, slabs_global, n_channels, align, [(0, degraded_mask, weights)], o.PHASE_AR)
        if ring_logs is not None:
            ring_logs["global"] = log
        for b, h in zip(bufs, heads):
            b[:ng] = h
    if not n_partial:
        return np.zeros((2, n_channels + 1), np.uint64), []
    order = [(d + 1 + i) % R for i in range(R - 1)]
    tails = [np.ascontiguousarray(bufs[r][ng:]) for r in order]
    log, _ = o.ring_sim(tails, dtype, slabs_partial, n_channels, align, [(0, 0, weights)], o.PHASE_AR)
    if ring_logs is not None:
        ring_logs["partial"] = log

    nbytes = n_partial * es
    t_deg = o.partition(weights, degraded_mask, nbytes, align)
    t_ok = o.partition(weights, 0, nbytes, align)
    cap = (max(nbytes, 1) + 255) // 256 * 256
    stage = [[np.full(cap, 0xA5, np.uint8) for _ in range(n_channels)] for _ in range(2)]
    d_tail = np.ascontiguousarray(bufs[d][ng:])
    o.reduce_copy(d_tail, dtype, o.OP_SUM, None, None, stage[0], t_deg, n_channels, cap)          # d sends
    for k in range(1, R):                                                                          # healthy ranks
        last = k == R - 1
        o.reduce_copy(tails[k - 1], dtype, o.OP_SUM if last else o.OP_SUM_FORWARD,
                      stage[(k + 1) & 1], t_deg if k == 1 else t_ok,
                      stage[k & 1], t_deg if last else t_ok, n_channels, cap)
    o.reduce_copy(d_tail, dtype, o.OP_COPY, stage[(R + 1) & 1], t_deg, None, None, n_channels, cap)  # d receives
    for r, t in zip(order, tails):
        bufs[r][ng:] = t
    bufs[d][ng:] = d_tail
    return np.stack([t_deg, t_ok]), stage
