"""Pins for the oracle's reduce-copy, ring schedule and bf16 rounding (CPU only).

What the paper fixes (Sec. 5.2: ring all-reduce = reduce-scatter then
all-gather; Sec. 8.2: execution stays lossless whatever the failure timing;
Sec. 4.3 Technique II: staged send buffers, chunk-granular progress; Sec. 5.1:
nothing goes to a failed NIC) is checked against things that are not the
oracle: a pure-Python ring written in another shape, exact integer sums, fp64
sums with the textbook error bound, torch's own bf16 conversion, and
metamorphic relations between schedules.
"""
import itertools

import numpy as np
import pytest
import torch

import workloads as wl

F32, BF16 = 0, 1


def _rand_inputs(rng, R, N, dtype, scale=1.0):
    xs = []
    for _ in range(R):
        x = (rng.standard_normal(N) * scale).astype(np.float32)
        if dtype == BF16:
            xs.append(torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy())
        else:
            xs.append(x)
    return xs


def _torch_round(dtype, a32: np.float32):
    """Round an fp32 value to the buffer type with the library's conversion."""
    if dtype == F32:
        return np.float32(a32)
    return torch.tensor([a32], dtype=torch.float32).to(torch.bfloat16).to(torch.float32).numpy()[0]


def _as_f32(dtype, arr):
    if dtype == F32:
        return arr.astype(np.float32)
    return (arr.astype(np.uint32) << 16).view(np.float32)


def _from_f32(dtype, arr32):
    if dtype == F32:
        return arr32.astype(np.float32)
    return (arr32.view(np.uint32) >> 16).astype(np.uint16)  # exact: values are already bf16


def _python_ring(xs, dtype, S, phases):
    """A ring of R Python 'processes' exchanging whole chunks as messages (no channels,
    no staging): the textbook reduce-scatter / all-gather, one scalar at a time."""
    R = len(xs)
    N = xs[0].size
    E = N // (S * R)
    bufs = [_as_f32(dtype, x).copy() for x in xs]
    for l in range(S):
        def chunk(r, c):
            base = (l * R + c) * E
            return bufs[r][base:base + E]
        if phases & 1:  # reduce-scatter: R-1 rounds
            for step in range(R - 1):
                msgs = [chunk(r, (r - step) % R).copy() for r in range(R)]
                for r in range(R):
                    src = (r - 1) % R
                    dst = chunk(r, (src - step) % R)
                    for i in range(E):
                        dst[i] = _torch_round(dtype, np.float32(msgs[src][i]) + np.float32(dst[i]))
        if phases & 2:  # all-gather: R-1 rounds, rank r starts from chunk r+1
            for step in range(R - 1):
                msgs = [chunk(r, (r + 1 - step) % R).copy() for r in range(R)]
                for r in range(R):
                    src = (r - 1) % R
                    chunk(r, (src + 1 - step) % R)[:] = msgs[src]
    return [_from_f32(dtype, b) for b in bufs]


def _rand_epochs(rng, C, T_total):
    n = int(rng.integers(1, 4))
    starts = sorted(set([0] + [int(x) for x in rng.integers(0, max(T_total, 1), size=n - 1)]))
    eps = []
    for t0 in starts:
        while True:
            w = [int(x) for x in rng.integers(0, 6, size=C)]
            mask = int(rng.integers(0, 1 << C))
            if sum(0 if (mask >> c) & 1 else w[c] for c in range(C)):
                break
        eps.append((t0, mask, tuple(w)))
    return eps


def test_three_ranks_by_hand(oracle):
    """R = 3, one element per ring chunk, inputs 1 2 3 | 10 20 30 | 100 200 300, worked with pencil.
    Reduce-scatter alone: chunk c starts at rank c and collects one more term per hop, so rank r holds at
    chunk c the fold of ranks c .. r (cyclically); the all-gather then spreads the full sums; an all-gather
    alone passes each rank's chunk (r + 1) round unchanged."""
    xs = [np.array(v, dtype=np.float32) for v in ([1, 2, 3], [10, 20, 30], [100, 200, 300])]
    eps = [(0, 0, (1, 1))]

    def run(phases):
        bufs = [x.copy() for x in xs]
        oracle.ring_sim(bufs, F32, 1, 2, 4, eps, phases)
        return [b.tolist() for b in bufs], [e.tolist() for e in oracle.expected(xs, F32, 1, phases)]

    want_rs = [[1, 222, 303], [11, 20, 333], [111, 220, 300]]
    want_ar = [[111, 222, 333]] * 3
    want_ag = [[100, 2, 30]] * 3  # rank r contributes chunk r+1 of its own buffer: 2, 30 and (rank 2) chunk 0 = 100
    for phases, want in ((1, want_rs), (3, want_ar), (2, want_ag)):
        got, by_definition = run(phases)
        assert got == want, phases
        assert by_definition == want, phases


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("phases", [1, 2, 3])
def test_ring_sim_vs_python_ring_and_definition(oracle, dtype, phases):
    """Step-by-step oracle == independent Python ring == plain definition, bit for bit."""
    rng = np.random.default_rng(100 + dtype * 10 + phases)
    es = 4 if dtype == F32 else 2
    for R in (2, 3, 4, 5):
        for E in (1, 2, 3, 8, 9):
            for S in (1, 2):
                N = R * S * E
                xs = _rand_inputs(rng, R, N, dtype)
                C = int(rng.integers(1, 5))
                T_total = S * oracle.num_transmissions(R, phases)
                eps = _rand_epochs(rng, C, T_total)
                align = es * int(rng.integers(1, 4))
                bufs = [x.copy() for x in xs]
                oracle.ring_sim(bufs, dtype, S, C, align, eps, phases)
                want_def = oracle.expected(xs, dtype, S, phases)
                want_py = _python_ring(xs, dtype, S, phases)
                for r in range(R):
                    assert bufs[r].tobytes() == want_py[r].tobytes(), (R, E, S, r)
                    assert bufs[r].tobytes() == want_def[r].tobytes(), (R, E, S, r)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_integer_inputs_give_exact_sum(oracle, dtype):
    """Small integers add exactly in fp32 and bf16, so the all-reduce must equal the
    integer sum whatever the order."""
    rng = np.random.default_rng(5)
    R, S, E = 8, 2, 37
    N = R * S * E
    lim = 100 if dtype == F32 else 15  # bf16 holds integers up to 256 exactly; 8*15 = 120
    ints = [rng.integers(-lim, lim + 1, size=N) for _ in range(R)]
    xs = [_from_f32(dtype, v.astype(np.float32)) if dtype == BF16 else v.astype(np.float32) for v in ints]
    total = sum(ints)
    bufs = [x.copy() for x in xs]
    oracle.ring_sim(bufs, dtype, S, 4, 16, [(0, 0b0100, (3, 1, 4, 1))], 3)
    outs = oracle.expected(xs, dtype, S, 3)
    for r in range(R):
        assert np.array_equal(_as_f32(dtype, bufs[r]).astype(np.int64), total)
        assert np.array_equal(_as_f32(dtype, outs[r]).astype(np.int64), total)


def test_fp32_error_bound_against_fp64_sum(oracle):
    """|fold - exact| <= (R-1) * 2^-24 * sum|x| * (1 + small): the textbook bound for
    R-1 roundings to nearest."""
    rng = np.random.default_rng(6)
    R, N = 8, 8 * 4096
    xs = _rand_inputs(rng, R, N, F32)
    outs = oracle.expected(xs, F32, 1, 3)
    exact = np.sum(np.stack(xs).astype(np.float64), axis=0)
    absum = np.sum(np.abs(np.stack(xs).astype(np.float64)), axis=0)
    err = np.abs(outs[0].astype(np.float64) - exact)
    assert np.all(err <= (R - 1) * 2.0 ** -24 * absum * 1.001)
    assert err.max() > 0  # not suspiciously exact


def test_bf16_error_bound_against_fp64_sum(oracle):
    """Per-hop rounding to bf16: unit roundoff 2^-8 per hop (8 significand bits)."""
    w = wl.scaled(wl.cfg2(), 8 * 8192)
    xs = wl.make_inputs(w)
    outs = oracle.expected(xs, BF16, 1, 3)
    x64 = np.stack([wl.bf16_bits_to_f64(x) for x in xs])
    exact = x64.sum(axis=0)
    absum = np.abs(x64).sum(axis=0)
    y = wl.bf16_bits_to_f64(outs[3])
    err = np.abs(y - exact)
    assert np.all(err <= (w.R - 1) * 2.0 ** -8 * absum * 1.01)
    assert np.linalg.norm(y - exact) / np.linalg.norm(exact) <= 1e-2


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_result_independent_of_channel_schedule(oracle, dtype):
    """Lossless whatever the failure timing (Sec. 8.2): any channel count, alignment and
    failure/recovery schedule leaves the same bits in the rank buffers."""
    rng = np.random.default_rng(8)
    R, S, E = 4, 3, 64
    N = R * S * E
    xs = _rand_inputs(rng, R, N, dtype)
    ref = None
    for trial in range(12):
        C = int(rng.integers(1, 9))
        eps = _rand_epochs(rng, C, S * (2 * R - 2))
        align = 16 * int(rng.integers(1, 5))
        bufs = [x.copy() for x in xs]
        oracle.ring_sim(bufs, dtype, S, C, align, eps, 3)
        blob = b"".join(b.tobytes() for b in bufs)
        if ref is None:
            ref = blob
        assert blob == ref


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_reduce_scatter_then_all_gather_is_all_reduce(oracle, dtype):
    """Sec. 5.2: all-reduce is reduce-scatter followed by all-gather."""
    rng = np.random.default_rng(9)
    R, S, E = 5, 2, 24
    xs = _rand_inputs(rng, R, R * S * E, dtype)
    eps = [(0, 0b010, (2, 5, 3))]
    a = [x.copy() for x in xs]
    oracle.ring_sim(a, dtype, S, 3, 16, eps, 3)
    b = [x.copy() for x in xs]
    oracle.ring_sim(b, dtype, S, 3, 16, eps, 1)
    oracle.ring_sim(b, dtype, S, 3, 16, eps, 2)
    for r in range(R):
        assert a[r].tobytes() == b[r].tobytes()
    # and the definition composes the same way
    d1 = oracle.expected(xs, dtype, S, 1)
    d2 = oracle.expected(d1, dtype, S, 2)
    d3 = oracle.expected(xs, dtype, S, 3)
    for r in range(R):
        assert d2[r].tobytes() == d3[r].tobytes()


def test_all_ranks_agree_after_all_reduce(oracle):
    rng = np.random.default_rng(10)
    xs = _rand_inputs(rng, 6, 6 * 50, F32)
    outs = oracle.expected(xs, F32, 1, 3)
    for r in range(1, 6):
        assert outs[r].tobytes() == outs[0].tobytes()


def test_stage_contents_and_sentinels(oracle):
    """The last two transmissions of every rank are still in the stage buffers: the slices,
    concatenated in channel order, are the chunk that was sent; nothing else in any
    stage buffer is touched, and a failed channel's buffer is never written."""
    rng = np.random.default_rng(12)
    R, S, E, C = 4, 2, 96, 4
    dtype = F32
    N = R * S * E
    chunk_bytes = E * 4
    xs = _rand_inputs(rng, R, N, dtype)
    eps = [(0, 0b0100, (5, 1, 7, 3))]  # channel 2 down throughout
    bufs = [x.copy() for x in xs]
    cap = chunk_bytes + 64
    log, stage = oracle.ring_sim(bufs, dtype, S, C, 16, eps, 3, cap=cap, stage_fill=0xA5)
    T_slab = 2 * R - 2
    assert log.shape == (S * T_slab, C + 1)
    final = oracle.expected(xs, dtype, S, 3)
    for l in range(S):
        for j in (T_slab - 2, T_slab - 1):  # last transmission of each parity
            off = [int(v) for v in log[l * T_slab + j]]
            assert off == [int(v) for v in oracle.partition(eps[0][2], eps[0][1], chunk_bytes, 16)]
            for r in range(R):
                c = (r - j) % R
                sent = final[r][(l * R + c) * E:(l * R + c + 1) * E].tobytes()  # all-gather traffic = final values
                got = b"".join(stage[j & 1, r, l, k, :off[k + 1] - off[k]].tobytes() for k in range(C))
                assert got == sent
                for k in range(C):
                    assert np.all(stage[j & 1, r, l, k, off[k + 1] - off[k]:] == 0xA5)
    assert np.all(stage[:, :, :, 2, :] == 0xA5)  # failed channel: never written


def test_single_reduce_copy_matches_numpy(oracle):
    """One fused step against numpy on reassembled arrays."""
    rng = np.random.default_rng(14)
    E, C = 1000, 3
    nbytes = E * 4
    local = rng.standard_normal(E).astype(np.float32)
    incoming = rng.standard_normal(E).astype(np.float32)
    in_off = oracle.partition([1, 2, 3], 0, nbytes, 16)
    out_off = oracle.partition([4, 1, 1], 0b010, nbytes, 16)
    cap = nbytes
    raw = incoming.view(np.uint8)
    in_stage = [np.full(cap, 0xA5, np.uint8) for _ in range(C)]
    for k in range(C):
        a, b = int(in_off[k]), int(in_off[k + 1])
        in_stage[k][:b - a] = raw[a:b]
    out_stage = [np.full(cap, 0xA5, np.uint8) for _ in range(C)]
    loc = local.copy()
    oracle.reduce_copy(loc, F32, 0, in_stage, in_off, out_stage, out_off, C, cap)
    want = incoming + local
    assert np.array_equal(loc, want)
    got = np.concatenate([out_stage[k][:int(out_off[k + 1] - out_off[k])] for k in range(C)]).view(np.float32)
    assert np.array_equal(got, want)
    # copy op
    loc = local.copy()
    oracle.reduce_copy(loc, F32, 1, in_stage, in_off, None, None, C, cap)
    assert np.array_equal(loc, incoming)
    # copy-send leaves local alone
    loc = local.copy()
    oracle.reduce_copy(loc, F32, 0, None, None, out_stage, out_off, C, cap)
    assert np.array_equal(loc, local)
    got = np.concatenate([out_stage[k][:int(out_off[k + 1] - out_off[k])] for k in range(C)]).view(np.float32)
    assert np.array_equal(got, local)


def test_reduce_copy_capacity_error(oracle):
    local = np.zeros(64, np.float32)
    off = oracle.partition([1, 1], 0, 256, 16)
    out_stage = [np.zeros(64, np.uint8) for _ in range(2)]
    with pytest.raises(oracle.OracleError):
        oracle.reduce_copy(local, F32, 0, None, None, out_stage, off, 2, 64)  # slices are 128 B


def test_all_channels_failed_aborts_before_touching_data(oracle):
    xs = [np.arange(8, dtype=np.float32) for _ in range(2)]
    bufs = [x.copy() for x in xs]
    with pytest.raises(oracle.NoHealthyChannel):
        oracle.ring_sim(bufs, F32, 1, 2, 16, [(0, 0, (1, 1)), (1, 0b11, (1, 1))], 3)
    for a, b in zip(xs, bufs):
        assert np.array_equal(a, b)


# ---------------------------------------------------------------- bf16 rounding

def test_bf16_roundtrip_all_patterns(oracle):
    """Every bf16 value widens and narrows back to itself (NaNs keep their payload's top bits)."""
    for h in range(1 << 16):
        f = oracle.bf16_to_f32(h)
        back = oracle.f32_to_bf16(f)
        is_nan = (h & 0x7FFF) > 0x7F80
        if is_nan:
            assert (back & 0x7FFF) > 0x7F80
        else:
            assert back == h


def test_bf16_rounding_matches_torch(oracle):
    """Round-to-nearest-even against the library conversion on random bit patterns and on
    every exact tie / near-tie around a spread of exponents."""
    rng = np.random.default_rng(15)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    ties = []
    for hi in rng.integers(0, 2 ** 16, size=3000, dtype=np.uint64):
        for lo in (0x7FFF, 0x8000, 0x8001, 0x0000, 0xFFFF, 0x0001):
            ties.append((int(hi) << 16) | lo)
    bits = np.concatenate([bits, np.array(ties, dtype=np.uint32)])
    f = bits.view(np.float32)
    finite = np.isfinite(f)
    f = f[finite]
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(float(x)) for x in f], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_bf16_overflow_rounds_to_inf(oracle):
    big = np.array([0x7F7FFFFF], dtype=np.uint32).view(np.float32)[0]  # FLT_MAX
    assert oracle.f32_to_bf16(float(big)) == 0x7F80
    assert oracle.f32_to_bf16(float("inf")) == 0x7F80
    assert oracle.f32_to_bf16(float("-inf")) == 0xFF80
    assert (oracle.f32_to_bf16(float("nan")) & 0x7FFF) > 0x7F80


def test_denormals_are_kept(oracle):
    """No flush-to-zero on either side of an fp32 add."""
    tiny = np.array([0x00000001, 0x00000003], dtype=np.uint32).view(np.float32)
    xs = [np.repeat(tiny[0], 4).astype(np.float32), np.repeat(tiny[1], 4).astype(np.float32)]
    outs = oracle.expected(xs, F32, 1, 3)
    assert outs[0].view(np.uint32).tolist() == [4, 4, 4, 4]
