"""Helpers of the GPU parity tests: run a workload through the C ABI and through the oracle."""
from __future__ import annotations

import sys

import numpy as np
import torch

import workloads as wl

FILL = 0xA5


def say(msg: str) -> None:
    """Name the case before its GPU work starts, so a fault can be attributed."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def codes(r2, oracle, w: wl.Workload):
    dt = r2.F32 if w.dtype == "f32" else r2.BF16
    ph = {"ar": r2.PHASE_AR, "rs": r2.PHASE_RS, "ag": r2.PHASE_AG}[w.phases]
    odt = oracle.F32 if w.dtype == "f32" else oracle.BF16
    oph = {"ar": oracle.PHASE_AR, "rs": oracle.PHASE_RS, "ag": oracle.PHASE_AG}[w.phases]
    return dt, ph, odt, oph


def to_device(x: np.ndarray) -> torch.Tensor:
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def to_host(t: torch.Tensor, like: np.ndarray) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(like.dtype)


def run_gpu_sim(r2, w: wl.Workload, xs, fill_stage: bool = False, stepwise: bool = False, window: int = 0,
                schedule: int = 0):
    """Returns (rank buffers as numpy, offsets log [T, C+1] uint64, workspace tensor, desc)."""
    dt = r2.F32 if w.dtype == "f32" else r2.BF16
    ph = {"ar": r2.PHASE_AR, "rs": r2.PHASE_RS, "ag": r2.PHASE_AG}[w.phases]
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, dt, ph, window, schedule)
    bufs = [to_device(x) for x in xs]
    ws_bytes = r2.r2_sim_workspace_bytes(desc)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    if fill_stage:
        ws.fill_(FILL)
    T = r2.r2_sim_num_transmissions(desc)
    log = torch.full((max(T, 1), w.C + 1), -1, dtype=torch.int64, device="cuda")
    if stepwise:
        r2.r2_sim_prepare(desc, w.epochs, ws, log)
        for p in range(r2.r2_sim_num_passes(desc)):
            for j in range(r2.r2_sim_num_steps(desc)):
                r2.r2_sim_step(desc, bufs, p, j, ws)
    else:
        r2.r2_ring_allreduce_sim(desc, bufs, w.epochs, ws, log)
    torch.cuda.synchronize()
    outs = [to_host(b, x) for b, x in zip(bufs, xs)]
    return outs, log.cpu().numpy().view(np.uint64)[:T], ws, desc


def expected_log(oracle, w: wl.Workload) -> np.ndarray:
    T = w.S * w.transmissions_per_slab
    rows = []
    for t in range(T):
        ep = [e for e in w.epochs if e[0] <= t][-1]
        rows.append(oracle.partition(ep[2], ep[1], w.chunk_bytes, w.align))
    return np.array(rows, dtype=np.uint64).reshape(T, w.C + 1)


def windows_around(points, total: int, radius: int, unit: int = 1):
    """Merged, sorted index ranges [a, b) within [0, total) that cover `radius` on either side of every
    point (a point at `total` gives the tail).  Bounds are multiples of `unit`, except `total` itself."""
    spans = []
    for p in points:
        a = max(0, (int(p) - radius) // unit * unit)
        b = min(total, (int(p) + radius + unit - 1) // unit * unit)
        if a < b:
            spans.append((a, b))
    spans.sort()
    merged = []
    for a, b in spans:
        if merged and a <= merged[-1][1]:
            merged[-1] = (merged[-1][0], max(merged[-1][1], b))
        else:
            merged.append((a, b))
    return merged


def assert_same_stage(got: np.ndarray, want: np.ndarray, what: str = "stage area") -> None:
    """Stage areas [..., capacity] of the product and of an oracle that sizes its channel buffers to the
    rounded chunk: the product's buffers may be longer (r2_sim_stage_capacity: chunks of 1 MiB and more
    get a pad); what both have must be the same bytes, and the rest must never have been written."""
    got = got.reshape(want.shape[:-1] + (-1,))
    cap = want.shape[-1]
    assert got.shape[-1] >= cap
    assert got[..., :cap].tobytes() == want.tobytes(), what
    assert np.all(got[..., cap:] == FILL), what + ": bytes behind the chunk's capacity were written"

