"""Seeded synthetic workloads shared by the tests and the benchmark.

Holds shapes, channel-state schedules and random inputs only; none of the
method's arithmetic (no partition rule, no reduction) lives here.  Both the
HIP path and the CPU oracle are fed from these generators so that they see
the same bits.

The five workloads stand in for the traffic the paper measures (Sec. 8:
Megatron-LM data-parallel gradient all-reduce, vLLM tensor-parallel
all-reduce, NCCL-tests size sweeps with one injected NIC failure); the real
models and clusters are not available, so only the message shapes are kept.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import List, Tuple

import numpy as np
import torch

Epoch = Tuple[int, int, Tuple[int, ...]]  # (t_start, fail_mask, weights)

GBPS = 1000  # weights are integers in MB/s: 50 GB/s -> 50000


@dataclass(frozen=True)
class Workload:
    name: str
    R: int                 # simulated ranks
    dtype: str             # "f32" | "bf16"
    N: int                 # elements per rank
    S: int                 # slabs (pipeline iterations); ring chunk = N/(S*R) elements
    C: int                 # NIC channels
    align: int             # partition alignment in bytes
    phases: str            # "ar" | "rs" | "ag"
    sigma: float           # inputs ~ N(0, sigma)
    seed: int
    epochs: Tuple[Epoch, ...]
    note: str = ""

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def steps_per_slab(self) -> int:
        return 2 * self.R - 1 if self.phases == "ar" else self.R

    @property
    def transmissions_per_slab(self) -> int:
        return self.steps_per_slab - 1

    @property
    def chunk_elems(self) -> int:
        return self.N // (self.S * self.R)

    @property
    def chunk_bytes(self) -> int:
        return self.chunk_elems * self.elem_bytes

    @property
    def algorithmic_bytes(self) -> int:
        """Bytes the method itself must move, summed over the R ranks.

        Per rank and slab, in ring-chunk units: copy-send 2, each reducing step
        4 (two reads, two writes), each forwarding all-gather step 3, a final
        step without stage write one less."""
        R = self.R
        if self.phases == "ar":
            units = 2 + 4 * (R - 1) + 3 * (R - 2) + 2
        elif self.phases == "rs":
            units = 2 + 4 * (R - 2) + 3
        else:
            units = 2 + 3 * (R - 2) + 2
        return units * self.N * self.elem_bytes


def _equal(C: int, gbps: int = 50) -> Tuple[int, ...]:
    return tuple([gbps * GBPS] * C)


def _lognormal_weights(n_draws: int, C: int, seed: int) -> List[Tuple[int, ...]]:
    """Bandwidths ~ lognormal(mu = ln 50 GB/s, sigma = 0.3), as integers in MB/s (>= 1)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    z = torch.randn(n_draws, C, generator=g, dtype=torch.float64).numpy()
    out = []
    for row in z:
        out.append(tuple(max(1, int(math.floor(GBPS * math.exp(math.log(50.0) + 0.3 * float(v)) + 0.5)))
                         for v in row))
    return out


def cfg1(N: int = 1 << 20) -> Workload:
    C = 4
    return Workload("cfg1", R=4, dtype="f32", N=N, S=1, C=C, align=256, phases="ar", sigma=1.0, seed=1,
                    epochs=((0, 1 << 2, _equal(C)),),
                    note="channel 2 failed from t=0")


def cfg2(N: int = 1 << 26) -> Workload:
    C = 8
    return Workload("cfg2", R=8, dtype="bf16", N=N, S=1, C=C, align=256, phases="ar", sigma=0.02, seed=2,
                    epochs=((0, 0, _equal(C)), (3, (1 << 2) | (1 << 5), _equal(C))),
                    note="channels 2 and 5 fail at reduce-scatter step 3")


def cfg3(N: int = 1 << 26, S: int = 4) -> Workload:
    C, R = 8, 16
    ws = _lognormal_weights(S, C, seed=33)
    epochs = tuple((l * (R - 1), 0, ws[l]) for l in range(S))
    return Workload("cfg3", R=R, dtype="f32", N=N, S=S, C=C, align=256, phases="rs", sigma=1.0, seed=3,
                    epochs=epochs, note="lognormal weights redrawn per 64 MiB slab; reduce-scatter only")


def cfg4(N: int = 1 << 25, S: int = 32) -> Workload:
    C, R = 8, 8
    T_total = S * (2 * R - 2)
    epochs = tuple((t0, (1 << 3) if (t0 // 16) % 2 == 1 else 0, _equal(C)) for t0 in range(0, T_total, 16))
    return Workload("cfg4", R=R, dtype="bf16", N=N, S=S, C=C, align=256, phases="ar", sigma=0.02, seed=4,
                    epochs=epochs, note="channel 3 is down while floor(t/16) is odd")


def cfg5(tokens: int = 16, hidden: int = 8192) -> Workload:
    C = 8
    return Workload(f"cfg5_tok{tokens}", R=8, dtype="bf16", N=hidden * tokens, S=1, C=C, align=256,
                    phases="ar", sigma=0.02, seed=5, epochs=((0, 1, _equal(C)),),
                    note="tensor-parallel all-reduce, channel 0 failed")


CFG5_TOKENS = (1, 16, 64, 256)


def scaled(w: Workload, N: int) -> Workload:
    """Same structure at another size (N must stay a multiple of S*R)."""
    assert N % (w.S * w.R) == 0
    return replace(w, N=N, name=f"{w.name}_N{N}")


def make_inputs(w: Workload) -> List[np.ndarray]:
    """R rank buffers: float32 arrays, or uint16 bf16 bit patterns."""
    g = torch.Generator(device="cpu").manual_seed(w.seed)
    out = []
    for _ in range(w.R):
        x = torch.randn(w.N, generator=g, dtype=torch.float32)
        if w.sigma != 1.0:
            x.mul_(w.sigma)
        if w.dtype == "bf16":
            out.append(x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
        else:
            out.append(x.numpy())
    return out


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns, for error measurements."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
