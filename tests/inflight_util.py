"""Seeded random ring runs with failures in flight, for the CPU pins and the GPU parity test alike
(shapes and channel schedules only; no arithmetic of the method)."""
from dataclasses import replace

import workloads as wl


def random_case(rng, vectors_only=False):
    R = int(rng.integers(2, 7))
    S = int(rng.integers(1, 4))
    C = int(rng.integers(2, 9))
    dtype = "f32" if rng.integers(0, 2) else "bf16"
    phases = ["ar", "rs", "ag"][int(rng.integers(0, 3))]
    E = int(rng.integers(1, 400))
    if vectors_only:
        E = (E + 7) // 8 * 8  # ring chunks of whole 16-byte vectors (what fused columns need)
    align = int(rng.choice([16, 32, 256]))
    T = S * ((2 * R - 2) if phases == "ar" else (R - 1))
    weights = tuple(int(x) for x in rng.integers(1, 50, size=C))
    starts = sorted(set(int(x) for x in rng.integers(1, T + 2, size=int(rng.integers(1, 5)))))
    epochs, flags, mask = [(0, 0, weights)], [False], 0
    for t0 in starts:
        fl = bool(rng.integers(0, 2))
        if fl:
            free = [c for c in range(C) if not (mask >> c) & 1]
            if len(free) < 2:
                fl = False
            else:
                mask |= 1 << int(rng.choice(free[:-1]))  # at least one channel stays up
        if not fl:
            keep = int(rng.integers(0, C))
            mask = int(rng.integers(0, 1 << C)) & ~(1 << keep)
        weights = tuple(int(x) for x in rng.integers(1, 50, size=C))
        epochs.append((t0, mask, weights))
        flags.append(fl)
    w = replace(wl.cfg1(), name="inflight_rand", R=R, dtype=dtype, N=R * S * E, S=S, C=C, align=align,
                phases=phases, sigma=1.0, seed=int(rng.integers(0, 1 << 30)), epochs=tuple(epochs))
    return w, flags, T
