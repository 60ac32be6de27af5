"""GPU parity: Broadcast, Reduce and All-to-All through the partitioned stage buffers
(R2_PHASE_BROADCAST / _REDUCE / _ALLTOALL) and the hop R2_OP_SUM_SEND vs the oracle, byte for byte:
buffers, offsets log, stage area."""
import numpy as np
import pytest
import torch

from gpu_util import FILL, assert_same_stage, say
from oracle import collectives as col

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def _inputs(rng, R, N, dtype):
    if dtype == "bf16":
        return [torch.from_numpy(rng.standard_normal(N).astype(np.float32)).to(torch.bfloat16)
                .view(torch.int16).numpy().view(np.uint16).copy() for _ in range(R)]
    return [rng.standard_normal(N).astype(np.float32) for _ in range(R)]


def _stage(r2, desc, ws, R, S_int, C):
    cap = r2.r2_sim_stage_capacity(desc)
    off = r2.r2_sim_stage_offset(desc)
    return ws[off:off + 2 * R * S_int * C * cap].cpu().numpy().reshape(2, R, S_int, C, cap)


def _run_chain(r2, oracle, kind, xs, dtype, root, S, C, align, epochs, window=0, check_stage=True):
    R, N = len(xs), xs[0].size
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    phase = r2.PHASE_BROADCAST if kind == "broadcast" else r2.PHASE_REDUCE
    desc = r2.SimDesc(R, S, C, align, N, gdt, phase, window, 0, root)
    assert r2.r2_sim_num_steps(desc) == R and r2.r2_sim_num_transmissions(desc) == S * (R - 1)
    ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
    log = torch.full((S * (R - 1), C + 1), -1, dtype=torch.int64, device="cuda")
    bufs = [_dev(x) for x in xs]
    r2.r2_collective_sim(desc, bufs, epochs, ws, log)
    torch.cuda.synchronize()
    o_bufs = [x.copy() for x in xs]
    if kind == "broadcast":
        o_log, o_stage = col.broadcast_sim(o_bufs, odt, root, S, C, align, epochs, FILL)
        want = col.broadcast_expected(xs, root)
    else:
        o_log, o_stage = col.reduce_sim(o_bufs, odt, root, S, C, align, epochs, FILL)
        want = col.reduce_expected(xs, odt, root)
    for r in range(R):
        got = bufs[r].cpu().numpy().view(xs[r].dtype)
        assert got.tobytes() == want[r].tobytes(), f"rank {r} vs definition"
        assert got.tobytes() == o_bufs[r].tobytes(), f"rank {r} vs step-by-step oracle"
    assert log.cpu().numpy().view(np.uint64).tolist() == o_log.tolist()
    if check_stage:
        assert_same_stage(_stage(r2, desc, ws, R, S, C), o_stage)


def _run_alltoall(r2, oracle, send, dtype, S, C, align, epochs, window=0, check_stage=True):
    R, N = len(send), send[0].size
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    desc = r2.SimDesc(R, S, C, align, N, gdt, r2.PHASE_ALLTOALL, window, 0)
    n_tx = (R - 1) * S
    assert r2.r2_sim_num_steps(desc) == 2 and r2.r2_sim_num_transmissions(desc) == n_tx
    ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
    log = torch.full((n_tx, C + 1), -1, dtype=torch.int64, device="cuda")
    sb = [_dev(x) for x in send]
    rb = [torch.zeros_like(t) for t in sb]
    r2.r2_alltoall_sim(desc, sb, rb, epochs, ws, log)
    torch.cuda.synchronize()
    o_recv = [np.zeros_like(x) for x in send]
    o_log, o_stage = col.alltoall_sim(send, o_recv, odt, S, C, align, epochs, FILL)
    want = col.alltoall_expected(send)
    for r in range(R):
        got = rb[r].cpu().numpy().view(send[r].dtype)
        assert got.tobytes() == want[r].tobytes(), f"rank {r} vs definition"
        assert got.tobytes() == o_recv[r].tobytes(), f"rank {r} vs step-by-step oracle"
        assert sb[r].cpu().numpy().view(send[r].dtype).tobytes() == send[r].tobytes(), "send buffer changed"
    assert log.cpu().numpy().view(np.uint64).tolist() == o_log.tolist()
    if check_stage:
        st = _stage(r2, desc, ws, R, n_tx, C)
        assert_same_stage(st[0], o_stage, "stage area (parity 0)")
        assert np.all(st[1] == FILL), "parity 1 is never used by a two-step exchange"


EPOCHS8 = [(0, 0, [50000] * 8), (1, 0b00100100, [50000] * 8), (4, 0b1, [1, 2, 3, 4, 5, 6, 7, 8])]


@pytest.mark.parametrize("kind", ["broadcast", "reduce"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_small(r2, oracle, kind, dtype):
    rng = np.random.default_rng(800)
    per16 = 4 if dtype == "f32" else 8
    for R, S, E, root in ((2, 1, per16 * 100, 0), (2, 2, per16 * 9, 1), (4, 5, per16 * 1031, 2), (8, 3, 7, 7),
                          (3, 2, per16 * 512 * 9 + 3, 1), (5, 1, per16 * 512 * 4, 4)):
        say(f"{kind} {dtype} R={R} S={S} E={E} root={root}")
        xs = _inputs(rng, R, S * E, dtype)
        _run_chain(r2, oracle, kind, xs, dtype, root, S, 8, 256, EPOCHS8)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_alltoall_small(r2, oracle, dtype):
    rng = np.random.default_rng(801)
    per16 = 4 if dtype == "f32" else 8
    for R, S, E in ((2, 1, per16 * 100), (4, 3, per16 * 517), (8, 2, 7), (3, 2, per16 * 512 * 3 + 3), (5, 1, 1)):
        say(f"alltoall {dtype} R={R} S={S} E={E}")
        send = _inputs(rng, R, R * S * E, dtype)
        _run_alltoall(r2, oracle, send, dtype, S, 8, 256, EPOCHS8)


@pytest.mark.parametrize("seed", [1, 2])
def test_collectives_random_configurations(r2, oracle, seed):
    rng = np.random.default_rng(810 + seed)
    for case in range(24):
        kind = ("broadcast", "reduce", "alltoall")[case % 3]
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        R, S, C = int(rng.integers(2, 10)), int(rng.integers(1, 5)), int(rng.integers(1, 10))
        E = int(rng.integers(1, 3000))
        align = (16, 64, 256)[int(rng.integers(0, 3))]
        n_tx = S * (R - 1)
        epochs = [(0, int(rng.integers(0, (1 << C) - 1)), [int(x) for x in rng.integers(1, 1000, C)])]
        for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, 3))):
            epochs.append((t, int(rng.integers(0, (1 << C) - 1)), [int(x) for x in rng.integers(1, 1000, C)]))
        window = (0, 1, 4096, 50000)[int(rng.integers(0, 4))]
        whole = window == 0  # with passes the leftover stage bytes depend on the pass order
        say(f"random {seed}.{case} {kind} {dtype} R={R} S={S} C={C} E={E} align={align} window={window} epochs={[(e[0], e[1]) for e in epochs]}")
        if kind == "alltoall":
            _run_alltoall(r2, oracle, _inputs(rng, R, R * S * E, dtype), dtype, S, C, align, epochs, window, whole)
        else:
            _run_chain(r2, oracle, kind, _inputs(rng, R, S * E, dtype), dtype, int(rng.integers(0, R)), S, C, align,
                       epochs, window, whole)


def test_collectives_large_with_passes(r2, oracle):
    """Chunks of several MiB, a stage window that forces byte-range passes, a channel that fails on the way."""
    rng = np.random.default_rng(802)
    w = [50000] * 8
    R, S = 4, 2
    N = S * (2 << 20)  # fp32: 8 MiB per chunk
    xs = _inputs(rng, R, N, "f32")
    epochs = [(0, 0, w), (2, 0b00001000, w)]
    for kind in ("broadcast", "reduce"):
        say(f"{kind} large R={R} S={S} N={N} window=3MiB, then default")
        _run_chain(r2, oracle, kind, xs, "f32", 1, S, 8, 256, epochs, window=3 << 20, check_stage=False)
        _run_chain(r2, oracle, kind, xs, "f32", 3, S, 8, 256, epochs)
    send = _inputs(rng, R, R * S * (1 << 19), "bf16")  # 1 MiB per chunk
    say("alltoall large, window 1 MiB, then default")
    _run_alltoall(r2, oracle, send, "bf16", S, 8, 256, epochs, window=1 << 20, check_stage=False)
    _run_alltoall(r2, oracle, send, "bf16", S, 8, 256, epochs)


def test_alltoall_blocks_that_are_not_16_byte_multiples(r2, oracle):
    """A rank's own block then starts off a 16-byte boundary: the 2-byte path of the own-block copy."""
    rng = np.random.default_rng(803)
    for R, S, E in ((3, 1, 5), (4, 3, 3), (2, 1, 4099)):
        say(f"alltoall odd blocks R={R} S={S} E={E}")
        _run_alltoall(r2, oracle, _inputs(rng, R, R * S * E, "bf16"), "bf16", S, 4, 16, [(0, 0b0010, [3, 1, 4, 1])])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sum_send_step(r2, oracle, dtype):
    """R2_OP_SUM_SEND: the outgoing stage gets incoming + local, local stays as it was."""
    rng = np.random.default_rng(804)
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    C, align = 4, 16
    for n in (8 * 512 * 5 + 24, 8, 8 * 1000):
        nbytes = n * (4 if dtype == "f32" else 2)
        cap = (nbytes + 255) // 256 * 256
        t_in = oracle.partition([3, 1, 4, 1], 0b0100, nbytes, align)
        t_out = oracle.partition([2, 7, 1, 8], 0b0001, nbytes, align)
        local, incoming = _inputs(rng, 2, n, dtype)
        # oracle: stage the incoming chunk, then a plain sum on a copy gives what must be sent on
        s_in = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        oracle.reduce_copy(incoming.copy(), odt, oracle.OP_SUM, None, None, s_in, t_in, C, cap)
        s_out = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        oracle.reduce_copy(local.copy(), odt, oracle.OP_SUM, s_in, t_in, s_out, t_out, C, cap)
        say(f"sum-send {dtype} n={n}")
        d_local = _dev(local)
        d_in = [torch.from_numpy(b).cuda() for b in s_in]
        d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]
        ti = torch.from_numpy(t_in.view(np.int64)).cuda()
        to = torch.from_numpy(t_out.view(np.int64)).cuda()
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        r2.r2_reduce_copy(d_local, gdt, r2.OP_SUM_SEND, d_in, ti, d_out, to, C, cap, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert d_local.cpu().numpy().view(local.dtype).tobytes() == local.tobytes(), "local changed"
        for c in range(C):
            assert d_out[c].cpu().numpy().tobytes() == s_out[c].tobytes(), f"outgoing stage, channel {c}"
    with pytest.raises(r2.R2Error):  # needs both stages
        r2.r2_reduce_copy(d_local, gdt, r2.OP_SUM_SEND, d_in, ti, None, None, C, cap, status)


def test_collectives_argument_errors(r2):
    w = [1] * 8
    sb = [torch.ones(4 * 2 * 16, dtype=torch.float32, device="cuda") for _ in range(4)]
    rb = [torch.zeros_like(t) for t in sb]
    desc = r2.SimDesc(4, 2, 8, 256, 4 * 2 * 16, r2.F32, r2.PHASE_ALLTOALL)
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    with pytest.raises(r2.R2Error):  # wrong phase
        r2.r2_alltoall_sim(r2.SimDesc(4, 2, 8, 256, 128, r2.F32, r2.PHASE_SENDRECV), sb, rb, [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error):  # in place
        r2.r2_alltoall_sim(desc, sb, [sb[1], rb[1], rb[2], rb[3]], [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error) as e:  # every channel down for the second transmission
        r2.r2_alltoall_sim(desc, sb, rb, [(0, 0, w), (1, 0xFF, w)], ws)
    assert e.value.code == -2
    for ph in (r2.PHASE_BROADCAST, r2.PHASE_REDUCE):
        d = r2.SimDesc(4, 2, 8, 256, 128, r2.F32, ph, root=2)
        space = torch.empty(r2.r2_sim_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        with pytest.raises(r2.R2Error) as e:  # a state in force for some hop has no healthy channel
            r2.r2_ring_allreduce_sim(d, sb, [(0, 0, w), (5, 0xFF, w)], space)
        assert e.value.code == -2
        with pytest.raises(r2.R2Error):  # the fused entry point does not run it
            r2.r2_sim_fused_steps(d, sb, 0, 2, space)
    torch.cuda.synchronize()
    assert all(float(t.sum()) == 128.0 for t in sb) and all(float(t.abs().sum()) == 0.0 for t in rb)


def test_collectives_maximum_ranks_and_channels(r2, oracle):
    """64 ranks and 64 channels, most of them down: every kernel argument array is used to its end."""
    rng = np.random.default_rng(805)
    C = 64
    w = [int(x) for x in rng.integers(1, 1000, C)]
    alive = (1 << 3) | (1 << 31) | (1 << 63)
    epochs = [(0, 0, w), (5, ((1 << C) - 1) & ~alive, w), (40, 1 << 63, w)]
    say("broadcast / reduce, R=64 C=64")
    xs = _inputs(rng, 64, 2 * 8 * 33, "bf16")
    _run_chain(r2, oracle, "broadcast", xs, "bf16", 63, 2, C, 16, epochs)
    _run_chain(r2, oracle, "reduce", xs, "bf16", 17, 2, C, 16, epochs)
    say("alltoall, R=64 C=64, 16 chunks per block (the most the grid allows)")
    send = _inputs(rng, 64, 64 * 16 * 4, "f32")
    _run_alltoall(r2, oracle, send, "f32", 16, C, 16, epochs)


def test_alltoall_and_reduce_in_a_graph(r2, oracle):
    """The calls only enqueue kernels (the own-block copy included), so they can be captured and
    replayed; every replay is checked, with eager work in between."""
    rng = np.random.default_rng(806)
    R, S, C, E = 4, 2, 8, 8 * 700
    epochs = [(0, 0, [50000] * C), (3, 0b00010010, [50000] * C)]
    send = _inputs(rng, R, R * S * E, "bf16")
    want_a2a = col.alltoall_expected(send)
    want_red = col.reduce_expected(send, oracle.BF16, 2)
    d_a2a = r2.SimDesc(R, S, C, 256, R * S * E, r2.BF16, r2.PHASE_ALLTOALL)
    d_red = r2.SimDesc(R, S, C, 256, R * S * E, r2.BF16, r2.PHASE_REDUCE, root=2)
    ws1 = torch.empty(r2.r2_sim_workspace_bytes(d_a2a), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(r2.r2_sim_workspace_bytes(d_red), dtype=torch.uint8, device="cuda")
    pristine = [_dev(x) for x in send]
    sb = [p.clone() for p in pristine]
    rb = [torch.zeros_like(p) for p in pristine]

    def both():
        r2.r2_alltoall_sim(d_a2a, sb, rb, epochs, ws1)
        r2.r2_ring_allreduce_sim(d_red, sb, epochs, ws2)  # reduces the send buffers in place afterwards

    say("graph capture: all-to-all, then reduce")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        both()  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        both()
    for replay in range(3):
        say(f"graph replay {replay}")
        for b, p in zip(sb, pristine):
            b.copy_(p)
        for b in rb:
            b.zero_()
        junk = torch.randn(1 << 16, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for r in range(R):
            assert rb[r].cpu().numpy().view(np.uint16).tobytes() == want_a2a[r].tobytes(), f"replay {replay}: all-to-all rank {r}"
            assert sb[r].cpu().numpy().view(np.uint16).tobytes() == want_red[r].tobytes(), f"replay {replay}: reduce rank {r}"
