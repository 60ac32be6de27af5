"""GPU parity: the ring all-reduce simulation through the C ABI vs the oracle.

Small sizes: rank buffers, offsets log and the whole stage area are compared byte for byte with the
step-by-step oracle.  Full sizes (the five benchmark configurations, in the launch configuration the
benchmark times): every element of every rank buffer is compared with the oracle's plain-definition
result, and the offsets log with the oracle's partition of the state in force.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import FILL, codes, expected_log, run_gpu_sim, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _stage_of(ws: torch.Tensor, r2, desc, w):
    off = r2.r2_sim_stage_offset(desc)
    cap = r2.r2_sim_stage_capacity(desc)
    n = 2 * w.R * w.S * w.C * cap
    return ws[off:off + n].cpu().numpy().reshape(2, w.R, w.S, w.C, cap), cap


def _full_compare_small(r2, oracle, w, stepwise=False, window=0, check_stage=True, schedule=1):
    _, _, odt, oph = codes(r2, oracle, w)
    xs = wl.make_inputs(w)
    say(f"sim small {w.name} R={w.R} N={w.N} S={w.S} C={w.C} {w.dtype} {w.phases} stepwise={stepwise} "
        f"window={window} schedule={schedule}")
    outs, log, ws, desc = run_gpu_sim(r2, w, xs, fill_stage=True, stepwise=stepwise, window=window,
                                      schedule=schedule)
    stage, cap = _stage_of(ws, r2, desc, w)
    o_bufs = [x.copy() for x in xs]
    o_log, o_stage = oracle.ring_sim(o_bufs, odt, w.S, w.C, w.align, list(w.epochs), oph, cap=cap, stage_fill=FILL)
    for r in range(w.R):
        assert outs[r].tobytes() == o_bufs[r].tobytes(), f"{w.name}: rank {r} buffer"
    assert log.tolist() == o_log.tolist(), f"{w.name}: offsets log"
    if check_stage:
        assert stage.tobytes() == o_stage.tobytes(), f"{w.name}: stage area"
    want = oracle.expected(xs, odt, w.S, oph)
    for r in range(w.R):
        assert outs[r].tobytes() == want[r].tobytes()


SMALL = [
    lambda: wl.scaled(wl.cfg1(), 4 * 4096 * 3 + 4 * 8),        # several tiles + tail, fp32
    lambda: wl.scaled(wl.cfg1(), 4 * 5),                        # chunk of 20 B: not a multiple of 16
    lambda: wl.scaled(wl.cfg2(), 8 * 8192 * 2 + 8 * 24),        # bf16, failure at t=3
    lambda: wl.scaled(wl.cfg2(), 8 * 3),                        # 6-byte chunks, element path only
    lambda: wl.scaled(wl.cfg3(S=4), 16 * 4 * 5000),             # R=16 reduce-scatter only, 4 slabs
    lambda: wl.scaled(wl.cfg4(S=32), 8 * 32 * 1100),            # flapping channel, 32 slabs
    lambda: wl.cfg5(1),
    lambda: wl.cfg5(16),
]


@pytest.mark.parametrize("make", SMALL, ids=lambda f: f().name)
def test_sim_small_full_state(r2, oracle, make):
    _full_compare_small(r2, oracle, make())


# sizes whose ring chunks are whole 16-byte vectors: the fused-column schedule applies
SMALL_FUSED = [
    lambda: wl.scaled(wl.cfg1(), 4 * 4096 * 3 + 4 * 8),        # 3.0 columns of 2 KiB... plus a ragged one
    lambda: wl.scaled(wl.cfg1(), 4 * 4),                        # one 16-byte vector per chunk
    lambda: wl.scaled(wl.cfg2(), 8 * 8192 * 2 + 8 * 24),        # state change at t=3: two launches
    lambda: wl.scaled(wl.cfg3(S=4), 16 * 4 * 5000),             # 16 ranks = 16 waves, epochs at slab starts
    lambda: wl.scaled(wl.cfg4(S=32), 8 * 32 * 1104),            # flapping: a cut at almost every step
    lambda: wl.cfg5(1),
    lambda: wl.cfg5(16),
    lambda: wl.cfg5(64),
]


@pytest.mark.parametrize("make", SMALL_FUSED, ids=lambda f: f().name)
def test_sim_fused_schedule_full_state(r2, oracle, make):
    """One launch takes every 2 KiB column through all steps between two channel-state changes:
    buffers, log and the whole stage area still match the oracle byte for byte."""
    _full_compare_small(r2, oracle, make(), schedule=2)


@pytest.mark.parametrize("phases", ["rs", "ag", "ar"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("R", [2, 3, 5, 16, 23])
def test_sim_fused_phases_and_ring_sizes(r2, oracle, phases, dtype, R):
    """More ranks than the 16 waves of a workgroup, odd ring sizes, all three phase sets."""
    from dataclasses import replace

    S, C, E = 2, 5, 776  # 776 elements: fp32 3104 B, bf16 1552 B, both multiples of 16
    T = S * ((2 * R - 2) if phases == "ar" else (R - 1))
    eps = [(0, 0b00010, (3, 9, 1, 0, 4))]
    if T > 2:
        eps.append((T // 2, 0b01001, (3, 9, 1, 7, 4)))
        eps.append((T - 1, 0, (1, 1, 1, 1, 100)))
    w = replace(wl.cfg1(), name=f"fused_R{R}_{dtype}_{phases}", R=R, dtype=dtype, N=R * S * E, S=S, C=C,
                align=32, phases=phases, sigma=1.0, seed=R, epochs=tuple(eps))
    _full_compare_small(r2, oracle, w, schedule=2)


def test_sim_fused_many_columns_state_changes(r2, oracle):
    """More columns than the GPU holds at once, so that columns really drift apart in time, with
    channel states that change mid-slab (the launch boundaries around a change are what keeps a
    column that is ahead from overwriting stage data another column has not read yet)."""
    from dataclasses import replace

    base = wl.scaled(wl.cfg2(), 8 * (1 << 21))  # 4 MiB chunks: 2048 columns of 8 waves
    eq = tuple([50000] * 8)
    for i, eps in enumerate([
        ((0, 0, eq), (3, 0b00100100, eq)),
        ((0, 0b1, eq), (1, 0, eq), (2, 0b10, eq), (7, 0b11110000, eq), (13, 0, eq)),
        ((0, 0, (1, 2, 3, 4, 5, 6, 7, 8)), (5, 0, (8, 7, 6, 5, 4, 3, 2, 1)), (6, 0, (1, 1, 1, 1, 1, 1, 1, 1))),
    ]):
        w = replace(base, epochs=eps, name=f"fused_drift{i}")
        _full_size(r2, oracle, w, schedule=2)


def test_sim_fused_needs_whole_vectors(r2):
    say("sim fused with 20-byte chunks is refused")
    w = wl.scaled(wl.cfg1(), 4 * 5)
    xs = wl.make_inputs(w)
    with pytest.raises(r2.R2Error) as e:
        run_gpu_sim(r2, w, xs, schedule=2)
    assert e.value.code == -1
    outs, _, _, _ = run_gpu_sim(r2, w, xs, schedule=0)  # AUTO falls back to one launch per step
    assert len(outs) == 4


def test_sim_stepwise_equals_one_call(r2, oracle):
    _full_compare_small(r2, oracle, wl.scaled(wl.cfg2(), 8 * 4096 + 8 * 8), stepwise=True)
    _full_compare_small(r2, oracle, wl.scaled(wl.cfg2(), 8 * 40000 + 8 * 8), stepwise=True, window=100000,
                        check_stage=False)


@pytest.mark.parametrize("window", [1, 8192, 70000, 1 << 20])
def test_sim_passes_leave_the_same_state(r2, oracle, window):
    """Cutting the run into passes (byte ranges of a chunk, or groups of slabs) changes the launch
    order only: buffers and log still match the oracle byte for byte.  So does the stage area,
    except where byte ranges of one slab meet a channel state that changes mid-run: then a stage
    location can be written by different transmissions in different passes, and which one is left
    over at the end depends on the pass order (what each step READS is unaffected: a pass runs its
    steps back to back)."""
    from dataclasses import replace

    w2 = wl.scaled(wl.cfg2(), 8 * 8192 * 3 + 8 * 24)
    ranges_in_use = 8 * w2.chunk_bytes > window
    _full_compare_small(r2, oracle, w2, window=window, check_stage=not ranges_in_use)            # ranges of one slab
    _full_compare_small(r2, oracle, replace(w2, epochs=w2.epochs[1:2] and ((0,) + w2.epochs[1][1:],)),
                        window=window)                                                           # same, one state
    _full_compare_small(r2, oracle, wl.scaled(wl.cfg1(), 4 * 4096 * 3 + 4 * 9), window=window)    # fp32, 36-byte tail
    _full_compare_small(r2, oracle, wl.scaled(wl.cfg4(S=32), 8 * 32 * 1100), window=window,
                        check_stage=8 * 2200 <= window)                                          # slab groups
    _full_compare_small(r2, oracle, wl.scaled(wl.cfg3(S=4), 16 * 4 * 5001), window=window,
                        check_stage=16 * 20004 <= window)                                        # element path


@pytest.mark.parametrize("phases", ["rs", "ag", "ar"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("R", [2, 3, 5])
def test_sim_phases_and_ring_sizes(r2, oracle, phases, dtype, R):
    from dataclasses import replace

    rng = np.random.default_rng(R * 10 + len(phases))
    S, C = 3, 5
    E = 777
    T = S * ((2 * R - 2) if phases == "ar" else (R - 1))
    eps = [(0, 0b00010, (3, 9, 1, 0, 4))]
    if T > 2:
        eps.append((T // 2, 0b01001, (3, 9, 1, 7, 4)))
        eps.append((T - 1, 0, (1, 1, 1, 1, 100)))
    w = replace(wl.cfg1(), name=f"ring_R{R}_{dtype}_{phases}", R=R, dtype=dtype, N=R * S * E, S=S, C=C, align=32,
                phases=phases, sigma=1.0, seed=int(rng.integers(1, 1000)), epochs=tuple(eps))
    _full_compare_small(r2, oracle, w)


def test_sim_many_channels_and_single_channel(r2, oracle):
    from dataclasses import replace

    base = wl.scaled(wl.cfg1(), 4 * 30000)
    w64 = replace(base, name="C64", C=64, align=16,
                  epochs=((0, 0xF0F0, tuple(range(1, 65))), (2, 1 << 63, tuple([7] * 64))))
    _full_compare_small(r2, oracle, w64)
    w1 = replace(base, name="C1", C=1, epochs=((0, 0, (5,)),))
    _full_compare_small(r2, oracle, w1)


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sim_maximum_ranks_and_channels(r2, oracle, dtype, schedule):
    """The limits of the interface: 64 ranks (127 fused steps, 126 transmissions per slab; in the fused
    schedule four ranks share a wave) and 64 channels, where the table rows of a fused launch no longer
    fit its LDS block and the prepared tables are read from memory instead."""
    from dataclasses import replace

    R, S, E = 64, 2, 776  # 776 elements: 3104 or 1552 bytes, whole 16-byte vectors
    T = S * (2 * R - 2)
    base = replace(wl.cfg1(), R=R, dtype=dtype, N=R * S * E, S=S, align=16, phases="ar", sigma=1.0, seed=64)
    w8 = replace(base, name=f"R64_C8_{dtype}", C=8,
                 epochs=((0, 0b1, tuple([50000] * 8)), (T // 3, 0b10100000, tuple(range(1, 9))), (T - 5, 0, tuple([1] * 8))))
    _full_compare_small(r2, oracle, w8, schedule=schedule)
    w64 = replace(base, name=f"R64_C64_{dtype}", C=64,
                  epochs=((0, 0xFF00FF00FF00FF00, tuple(range(1, 65))), (130, 1 << 63, tuple([7] * 64)),
                          (200, (1 << 64) - 2, tuple([3] * 64))))
    _full_compare_small(r2, oracle, w64, schedule=schedule)
    # one channel state for the whole run: a single fused launch whose 126 rows of 65 entries exceed the
    # LDS block, so the tables are prepared up front and the columns that straddle cuts look them up in memory
    w64b = replace(base, name=f"R64_C64_one_state_{dtype}", C=64, epochs=((0, 0x00FF00FF00FF00FE, tuple(range(1, 65))),))
    _full_compare_small(r2, oracle, w64b, schedule=schedule)


@pytest.mark.parametrize("schedule", [1, 2])
def test_sim_maximum_slabs(r2, oracle, schedule):
    """R * S just under the 65535 limit of the launch grid: 8191 slabs of 8 ranks with one 16-byte
    vector per ring chunk, the channel state changing every 1000 transmissions."""
    from dataclasses import replace

    R, S, C = 8, 8191, 4
    T = S * (2 * R - 2)
    eps = tuple((t0, (1 << ((t0 // 1000) % C)), (5, 6, 7, 8)) for t0 in range(0, T, 1000))
    w = replace(wl.cfg1(), name="S8191", R=R, dtype="f32", N=R * S * 4, S=S, C=C, align=16, phases="ar",
                sigma=1.0, seed=8191, epochs=eps)
    _full_compare_small(r2, oracle, w, schedule=schedule)


def test_sim_chunks_beyond_4GiB(r2, oracle):
    """Byte offsets that do not fit 32 bits: two ranks of 8 GiB + 8 MiB each, i.e. ring chunks of
    4 GiB + 4 MiB, moved in byte-range passes.  Too large for the oracle's step-by-step ring on the host
    as a whole, so the oracle checks windows of it element by element: the first tile, a MiB either side
    of every 2^32-byte boundary (of the chunk and of the rank buffer), of every slice cut of both channel
    states and of the chunk's end.  A window takes the same element range of every ring chunk of every
    rank, which is an all-reduce of its own with the same fold order, so `oracle.expected` gives its
    result.  Everything else is checked by what the result must be for two ranks (one fp32 addition per
    element, the same bits in either order, made with a library call), and the tables against the oracle's
    partition."""
    from gpu_util import windows_around

    R, C = 2, 3
    N = (1 << 31) + (1 << 21)
    weights = (3, 1, 2)
    epochs = [(0, 0, weights), (1, 0b010, weights)]
    desc = r2.SimDesc(R, 1, C, 256, N, r2.F32, r2.PHASE_AR, 0, r2.SCHED_STEPS)
    E = N // R
    chunk_bytes = E * 4
    assert chunk_bytes > 1 << 32 and r2.r2_sim_num_passes(desc) > 1
    say(f"sim beyond 4 GiB: R={R} N={N} chunk={chunk_bytes} B passes={r2.r2_sim_num_passes(desc)}")
    g = torch.Generator(device="cuda").manual_seed(4096)
    xs = [torch.randn(N, generator=g, dtype=torch.float32, device="cuda") for _ in range(R)]
    tables = [oracle.partition(w, mask, chunk_bytes, 256) for _, mask, w in epochs]
    points = [0, 1 << 32, (1 << 33) - chunk_bytes, chunk_bytes] + [int(x) for t in tables for x in t]
    spans = windows_around([p // 4 for p in points], E, (1 << 20) // 4)
    before = [[np.concatenate([xs[r][c * E + a:c * E + b].cpu().numpy() for c in range(R)]) for r in range(R)]
              for a, b in spans]
    want = xs[0] + xs[1]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    log = torch.full((2, C + 1), -1, dtype=torch.int64, device="cuda")
    r2.r2_ring_allreduce_sim(desc, xs, epochs, ws, log)
    torch.cuda.synchronize()
    for (a, b), mini in zip(spans, before):
        exp = oracle.expected(mini, oracle.F32, 1, oracle.PHASE_AR)
        for r in range(R):
            got = np.concatenate([xs[r][c * E + a:c * E + b].cpu().numpy() for c in range(R)])
            assert got.tobytes() == exp[r].tobytes(), f"rank {r}, elements [{a}, {b}) of every chunk vs the oracle"
    for r in range(R):
        assert torch.equal(xs[r].view(torch.int32), want.view(torch.int32)), f"rank {r}"
    got = log.cpu().numpy().view(np.uint64)
    for t in range(len(epochs)):
        assert got[t].tolist() == tables[t].tolist()
    assert int(got[0][-1]) == chunk_bytes and int(got[0][1]) > 1 << 31  # cuts beyond 2 GiB and 4 GiB
    del xs, want, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_sim_random_configurations(r2, oracle, seed):
    """Random small configurations -- ring size, slabs, channels, chunk size (ragged included), alignment,
    type, phases, schedule, pass window, channel states that change at random transmissions -- each compared
    in full (buffers, offsets log, stage area where it is comparable) with the oracle."""
    from dataclasses import replace

    rng = np.random.default_rng(9000 + seed)
    for case in range(25):
        R = int(rng.integers(2, 21))
        S = int(rng.integers(1, 6))
        C = int(rng.integers(1, 13))
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        phases = ("ar", "rs", "ag")[int(rng.integers(0, 3))]
        schedule = int(rng.integers(1, 3))
        es = 4 if dtype == "f32" else 2
        if schedule == 2 or rng.random() < 0.5:
            E = int(rng.integers(1, 400)) * (16 // es)       # whole 16-byte vectors (needed by the fused schedule)
        else:
            E = int(rng.integers(1, 3000))                    # anything, element path included
        align = (16, 32, 256)[int(rng.integers(0, 3))]
        J1 = (2 * R - 2) if phases == "ar" else (R - 1)
        T = S * J1
        eps, t0 = [], 0
        while t0 < T:
            mask = int(rng.integers(0, (1 << C) - 1)) if C > 1 else 0       # never every channel
            weights = tuple(int(x) for x in rng.integers(1, 60000, C))
            eps.append((t0, mask, weights))
            t0 += int(rng.integers(1, max(2, T)))
        window = 0 if rng.random() < 0.5 else int(rng.integers(1, 8)) * R * E * es // 2 + 256
        w = replace(wl.cfg1(), name=f"random{seed}_{case}", R=R, dtype=dtype, N=R * S * E, S=S, C=C, align=align,
                    phases=phases, sigma=1.0, seed=1000 * seed + case, epochs=tuple(eps))
        # with several passes and several states the stage area's leftovers depend on the pass order
        one_pass = window == 0
        _full_compare_small(r2, oracle, w, window=window, check_stage=one_pass or len(eps) == 1, schedule=schedule)


def _random_mid_sizes(r2, oracle, seed, n_cases, schedules):
    """Random configurations of 0.25 to 17 MiB per rank with random channel schedules, pass windows and
    schedules: the buffers against the definition, the offsets log against the oracle's partition.
    Returns how many of them ran on fused columns."""
    rng = np.random.default_rng(seed)
    n_fused = 0
    for case in range(n_cases):
        R, S, C = int(rng.integers(2, 17)), int(rng.integers(1, 9)), int(rng.integers(1, 17))
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        es = 4 if dtype == "f32" else 2
        phases = ("ar", "rs", "ag")[int(rng.integers(0, 3))]
        mib = float(rng.choice([0.25, 1, 3, 8, 17]))
        E = max(1, int(mib * (1 << 20) / es / (S * R)))
        if rng.random() < 0.7:
            E = max(8, E // 8 * 8)  # mostly whole 16-byte vectors
        n_tx = S * ((2 * R - 2) if phases == "ar" else (R - 1))
        epochs = [(0, int(rng.integers(0, (1 << C) - 1)), tuple(int(x) for x in rng.integers(1, 100000, C)))]
        for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, int(rng.integers(0, 5))))):
            epochs.append((t, int(rng.integers(0, (1 << C) - 1)), tuple(int(x) for x in rng.integers(1, 100000, C))))
        window = int(rng.choice([0, 0, 0, 1 << 20, 7 << 20]))
        schedule = int(rng.choice(schedules))
        if schedule == 2 and (E * es) % 16:
            schedule = 0
        w = wl.Workload(f"mid{case}", R, dtype, E * S * R, S, C, (16, 256)[int(rng.integers(0, 2))], phases, 1.0,
                        2000 + case, tuple(epochs))
        say(f"mid-size {seed}.{case}: R={R} S={S} C={C} {dtype} {phases} {w.N * es / 2 ** 20:.2f} MiB/rank window={window} "
            f"schedule={schedule} epochs={[(e[0], e[1]) for e in epochs]}")
        xs = wl.make_inputs(w)
        outs, log, ws, desc = run_gpu_sim(r2, w, xs, window=window, schedule=schedule)
        n_fused += r2.r2_sim_resolve_schedule(desc, list(w.epochs)) == r2.SCHED_FUSED
        dt, ph, odt, oph = codes(r2, oracle, w)
        want = oracle.expected(xs, odt, S, oph)
        for r in range(R):
            assert outs[r].tobytes() == want[r].tobytes(), f"case {case} rank {r}"
        assert log.tolist() == expected_log(oracle, w).tolist(), f"case {case}: offsets log"
        del ws, outs, xs, want
        torch.cuda.empty_cache()
    return n_fused


def test_sim_random_mid_sizes(r2, oracle):
    """The sizes where the library's own choice flips between fused columns and one launch per step."""
    n_fused = _random_mid_sizes(r2, oracle, 9100, 14, [0, 0, 1, 2])
    assert 2 <= n_fused <= 12  # both schedules were exercised


def test_sim_overlapped_passes_never_share_a_slab_across_tables(r2, oracle):
    """Byte ranges of one slab share its stage buffers; under different tables their slices overlap, so a
    pass that runs a step ahead of its neighbour on the other stream would overwrite stage bytes that
    are still to be read.  Shapes that provoke it: many byte ranges per slab (a window far below a
    chunk), a new channel state at every transmission, enough bytes for the two streams to drift apart.
    One slab (the run must take the plain schedule), two and five slabs (the streams take the even and
    the odd slabs), both types; several runs each, every one bit-exact."""
    from dataclasses import replace

    for R, S, dtype, phases in ((10, 1, "bf16", "ar"), (12, 5, "bf16", "ag"), (16, 2, "f32", "rs"), (8, 2, "bf16", "ar")):
        es = 4 if dtype == "f32" else 2
        C = 11
        E = (1 << 20) // es // 8 * 8 + 8  # chunks of just over 1 MiB
        n_tx = S * ((2 * R - 2) if phases == "ar" else (R - 1))
        rng = np.random.default_rng(R * 100 + S)
        epochs = tuple((t, int(rng.integers(0, (1 << C) - 1)), tuple(int(x) for x in rng.integers(1, 100000, C)))
                       for t in range(n_tx))
        w = replace(wl.cfg1(), name=f"overlap_hazard_R{R}_S{S}", R=R, dtype=dtype, N=E * S * R, S=S, C=C, align=16,
                    phases=phases, sigma=1.0, seed=R + S, epochs=epochs)
        xs = wl.make_inputs(w)
        _, _, odt, oph = codes(r2, oracle, w)
        want = oracle.expected(xs, odt, S, oph)
        for attempt in range(3):
            say(f"overlapped passes across tables: R={R} S={S} {dtype} {phases} chunk {E * es} B, window 1 MiB, "
                f"{len(epochs)} states, run {attempt}")
            outs, log, ws, desc = run_gpu_sim(r2, w, xs, window=1 << 20, schedule=3)
            assert r2.r2_sim_num_passes(desc) > 2 * S
            for r in range(R):
                assert outs[r].tobytes() == want[r].tobytes(), f"rank {r}"
            assert log.tolist() == expected_log(oracle, w).tolist()
            del ws, outs


def test_sim_random_mid_sizes_overlapped_passes(r2, oracle):
    """The same kind of cases under the schedule that issues pairs of passes side by side on two streams:
    odd pass counts, byte-range passes and slab groups, state changes anywhere."""
    _random_mid_sizes(r2, oracle, 9300, 12, [3])


def test_sim_result_independent_of_schedule(r2, oracle):
    """Lossless whatever the failure timing: different schedules, same bits."""
    from dataclasses import replace

    base = wl.scaled(wl.cfg2(), 8 * 10000)
    xs = wl.make_inputs(base)
    ref = None
    for i, eps in enumerate([
        ((0, 0, tuple([50000] * 8)),),
        ((0, 0b11111110, tuple([50000] * 8)),),
        ((0, 0, tuple([1, 2, 3, 4, 5, 6, 7, 8])), (1, 0b1, tuple([8, 7, 6, 5, 4, 3, 2, 1])), (9, 0b10000000, tuple([1] * 8))),
    ]):
        w = replace(base, epochs=eps, name=f"sched{i}")
        say(f"sim schedule independence {i}")
        outs, _, _, _ = run_gpu_sim(r2, w, xs)
        blob = b"".join(o.tobytes() for o in outs)
        ref = ref or blob
        assert blob == ref


def test_sim_empty_input(r2):
    say("sim N=0")
    desc = r2.SimDesc(4, 1, 4, 256, 0, r2.F32, r2.PHASE_AR)
    ws = torch.empty(max(r2.r2_sim_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    r2.r2_ring_allreduce_sim(desc, [None] * 4, [(0, 0, [1, 1, 1, 1])], ws)
    torch.cuda.synchronize()


def test_sim_all_failed_touches_nothing(r2):
    say("sim all channels failed at t=2")
    w = wl.scaled(wl.cfg1(), 4 * 1024)
    xs = wl.make_inputs(w)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.F32, r2.PHASE_AR)
    bufs = [torch.from_numpy(x).cuda() for x in xs]
    ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim(desc, bufs, [(0, 0, [1] * 4), (2, 0b1111, [1] * 4)], ws)
    assert e.value.code == -2
    torch.cuda.synchronize()
    for b, x in zip(bufs, xs):
        assert b.cpu().numpy().tobytes() == x.tobytes()
    assert bool((ws == FILL).all())


# ------------------------------------------------------------------ full benchmark sizes

def _full_size(r2, oracle, w, check_bound=False, schedule=0, window=0):
    _, _, odt, oph = codes(r2, oracle, w)
    say(f"sim full {w.name}: generating inputs")
    xs = wl.make_inputs(w)
    say(f"sim full {w.name}: GPU run, schedule={schedule}, window={window}")
    outs, log, _, _ = run_gpu_sim(r2, w, xs, schedule=schedule, window=window)
    say(f"sim full {w.name}: oracle")
    want = oracle.expected(xs, odt, w.S, oph)
    for r in range(w.R):
        assert np.array_equal(outs[r], want[r]), f"{w.name}: rank {r}"
    assert log.tolist() == expected_log(oracle, w).tolist()
    if check_bound and w.dtype == "bf16":
        # acceptance bound against the exact sum, on a sample: normwise 1e-2, and elementwise the
        # a-priori bound for R-1 roundings of unit roundoff 2^-8
        idx = np.random.default_rng(0).integers(0, w.N, size=200000)
        x64 = np.stack([wl.bf16_bits_to_f64(x[idx]) for x in xs])
        exact, absum = x64.sum(axis=0), np.abs(x64).sum(axis=0)
        y = wl.bf16_bits_to_f64(outs[0][idx])
        assert np.linalg.norm(y - exact) / np.linalg.norm(exact) <= 1e-2
        assert np.all(np.abs(y - exact) <= 1e-2 * np.abs(exact) + (w.R - 1) * 2.0 ** -8 * absum)


def test_full_cfg1(r2, oracle):
    _full_size(r2, oracle, wl.cfg1())


def test_full_cfg2(r2, oracle):
    _full_size(r2, oracle, wl.cfg2(), check_bound=True)


def test_full_cfg2_fused(r2, oracle):
    _full_size(r2, oracle, wl.cfg2(), schedule=2)


def test_full_cfg4_fused(r2, oracle):
    _full_size(r2, oracle, wl.cfg4(), schedule=2)


def test_full_cfg3(r2, oracle):
    _full_size(r2, oracle, wl.cfg3())


def test_full_cfg3_one_pass(r2, oracle):
    """The stage window opened to 256 MiB: one pass, every step stages more than the caches hold, and
    the step kernel then writes its stage around them (the variant the cold roofline figure times)."""
    _full_size(r2, oracle, wl.cfg3(), schedule=1, window=256 << 20)


def test_full_cfg2_ragged_one_pass_stage_beyond_cache(r2, oracle):
    """bf16, chunks of 16 MiB + 48 bytes in one pass: a step stages just over 128 MiB, the bf16 kernels
    write their stage around the caches, and the last tile of every chunk is ragged."""
    _full_size(r2, oracle, wl.scaled(wl.cfg2(), 8 * ((1 << 23) + 24)), schedule=1, window=1 << 30)


@pytest.mark.parametrize("make", [wl.cfg2, wl.cfg3, wl.cfg4], ids=["cfg2", "cfg3", "cfg4"])
def test_full_overlapped_passes(r2, oracle, make):
    """The opt-in schedule that issues pairs of half-window passes side by side on two streams: same
    result, same tables, at full size."""
    _full_size(r2, oracle, make(), schedule=3)


def test_sim_overlapped_passes_small(r2, oracle):
    """Small shapes under the overlapped schedule: odd numbers of passes, byte-range passes of one slab,
    slab groups, a window that leaves a single pass."""
    from dataclasses import replace

    for w, window in ((wl.scaled(wl.cfg2(), 8 * 8192 * 2 + 8 * 24), 0),          # one slab: two byte ranges
                      (wl.scaled(wl.cfg2(), 8 * 8192 * 6 + 8 * 24), 3 * 8 * 8192),   # five byte ranges (odd)
                      (wl.scaled(wl.cfg4(S=32), 8 * 32 * 1100), 0),              # 32 slabs: two groups of 16
                      (wl.scaled(wl.cfg3(S=4), 16 * 4 * 5000), 16 * 5000 * 4 * 2),   # reduce-scatter, four slabs one by one
                      (replace(wl.scaled(wl.cfg1(), 4 * 3 * 1000), S=3), 0)):     # three slabs: a pair and a single pass
        _full_compare_small(r2, oracle, w, window=window, check_stage=False, schedule=3)


def test_full_cfg4(r2, oracle):
    _full_size(r2, oracle, wl.cfg4(), check_bound=True)


@pytest.mark.parametrize("tokens", wl.CFG5_TOKENS)
def test_full_cfg5(r2, oracle, tokens):
    _full_size(r2, oracle, wl.cfg5(tokens), check_bound=True)
