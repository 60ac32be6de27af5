"""GPU parity: R2CCL-AllReduce (global + partial all-reduce + tailored broadcast) and the relay step
R2_OP_SUM_FORWARD, through the C ABI vs the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from gpu_util import FILL, say
from oracle import split

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _inputs(rng, R, N, dtype):
    xs = []
    for _ in range(R):
        x = rng.standard_normal(N).astype(np.float32)
        if dtype == "bf16":
            x = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        xs.append(x)
    return xs


def _dev(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def _run_split(r2, oracle, xs, dtype, d, n_partial, Sg, Sp, C, align, weights, mask, schedule=0):
    R, N = len(xs), xs[0].size
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    desc = r2.SplitDesc(R, d, C, align, N, n_partial, gdt, schedule, Sg, Sp)
    need = r2.r2_split_workspace_bytes(desc)
    assert need > 0
    ws = torch.full((need,), FILL, dtype=torch.uint8, device="cuda")
    bufs = [_dev(x) for x in xs]
    r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)
    torch.cuda.synchronize()
    outs = [b.cpu().numpy().view(x.dtype) for b, x in zip(bufs, xs)]
    o_bufs = [x.copy() for x in xs]
    logs = {}
    tables, stage = split.split_sim(o_bufs, odt, d, n_partial, Sg, Sp, C, align, weights, mask, ring_logs=logs)
    want = split.split_expected(xs, odt, d, n_partial, Sg, Sp)
    for r in range(R):
        assert outs[r].tobytes() == o_bufs[r].tobytes(), f"rank {r} vs step-by-step oracle"
        assert outs[r].tobytes() == want[r].tobytes(), f"rank {r} vs definition"
    # each ring's workspace begins with the table of every transmission: the global ring's is cut by the
    # degraded server's channel state, the partial ring's by the full one
    up = lambda x: (x + 255) // 256 * 256
    g_desc = r2.SimDesc(R, Sg, C, align, N - n_partial, gdt, r2.PHASE_AR, 0, schedule)
    if N - n_partial:
        got = ws[: logs["global"].size * 8].cpu().numpy().view(np.uint64).reshape(logs["global"].shape)
        assert got.tolist() == logs["global"].tolist(), "tables of the global ring"
    if n_partial:
        at = up(r2.r2_sim_workspace_bytes(g_desc))
        got = ws[at: at + logs["partial"].size * 8].cpu().numpy().view(np.uint64).reshape(logs["partial"].shape)
        assert got.tolist() == logs["partial"].tolist(), "tables of the partial ring"
    if n_partial:
        # the broadcast's tables and stage buffers sit at the end of the workspace
        es = xs[0].itemsize
        cap = (n_partial * es + 255) // 256 * 256
        tail = ws[need - 2 * C * cap:].cpu().numpy().reshape(2, C, cap)
        for par in range(2):
            for c in range(C):
                assert tail[par, c].tobytes() == stage[par][c].tobytes(), f"broadcast stage parity {par} channel {c}"
        tab_bytes = (2 * (C + 1) * 8 + 255) // 256 * 256
        tabs = ws[need - 2 * C * cap - tab_bytes: need - 2 * C * cap - tab_bytes + 2 * (C + 1) * 8].cpu().numpy().view(np.uint64)
        assert tabs.reshape(2, C + 1).tolist() == tables.tolist()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("schedule", [1, 2])
def test_split_allreduce_small(r2, oracle, dtype, schedule):
    rng = np.random.default_rng(300 + schedule)
    per16 = 4 if dtype == "f32" else 8
    for R, d in ((3, 0), (4, 2), (8, 7), (5, 1)):
        for Sg, Sp, Eg, Ep in ((1, 1, 700, 300), (2, 3, 129, 64), (1, 1, 1, 1)):
            ng, npart = Sg * R * Eg * per16, Sp * (R - 1) * Ep * per16
            say(f"split {dtype} sched={schedule} R={R} d={d} global={ng} partial={npart}")
            xs = _inputs(rng, R, ng + npart, dtype)
            _run_split(r2, oracle, xs, dtype, d, npart, Sg, Sp, 4, 32, (50000, 25000, 50000, 12500), 0b0101, schedule)


def test_split_degenerate_shares(r2, oracle):
    rng = np.random.default_rng(9)
    say("split with nothing partial / nothing global")
    xs = _inputs(rng, 4, 4 * 64 * 4, "f32")
    _run_split(r2, oracle, xs, "f32", 1, 0, 1, 1, 2, 16, (1, 1), 0b01)          # plain all-reduce
    xs = _inputs(rng, 4, 3 * 64 * 4, "f32")
    _run_split(r2, oracle, xs, "f32", 3, 3 * 64 * 4, 1, 1, 2, 16, (1, 1), 0b10)  # everything skips rank 3


def test_split_planned_size_bf16(r2, oracle):
    """8 ranks, one has lost half of its 8 NICs: the planner's share (a little over one half) of a
    16 MiB-per-rank bf16 buffer goes the partial way."""
    say("split planned, 8 ranks x 8 Mi bf16")
    R, d, N = 8, 3, 1 << 23
    use, y, thr = r2.r2_split_plan(R, 1, 0.5)
    assert use and 0.5 < y < 0.52
    granule = 8 * 7 * 8  # global chunks of 8 ranks, partial chunks of 7, whole 16-byte vectors
    npart = int(round(y * N / granule)) * granule
    assert (N - npart) % (8 * 8) == 0 and npart % (7 * 8) == 0
    rng = np.random.default_rng(10)
    xs = [torch.randn(N, generator=torch.Generator().manual_seed(50 + r)).mul_(0.02).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
          for r in range(R)]
    _run_split(r2, oracle, xs, "bf16", d, npart, 1, 1, 8, 256, tuple([50000] * 8), 0b11110000)


def test_split_argument_checks(r2):
    say("split argument checks")
    ok = dict(n_ranks=4, degraded_rank=1, n_channels=2, align=16, n_elems=4 * 64 + 3 * 64, n_partial=3 * 64, dtype=0)
    assert r2.r2_split_workspace_bytes(r2.SplitDesc(**ok)) > 0
    for bad in (dict(n_ranks=2), dict(degraded_rank=4), dict(n_partial=10 ** 9), dict(n_partial=3 * 64 + 3),
                dict(align=8), dict(n_channels=0), dict(dtype=5), dict(n_slabs_global=0),
                dict(schedule=3)):  # the two rings already run side by side: no overlapped passes inside them
        assert r2.r2_split_workspace_bytes(r2.SplitDesc(**{**ok, **bad})) == 0, bad
    desc = r2.SplitDesc(**ok)
    ws = torch.empty(r2.r2_split_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    bufs = [torch.zeros(ok["n_elems"], dtype=torch.float32, device="cuda") for _ in range(4)]
    with pytest.raises(r2.R2Error) as e:
        r2.r2_split_allreduce_sim(desc, bufs, (1, 1), 0b11, ws)  # the degraded server has no NIC left
    assert e.value.code == -2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_relay_step(r2, oracle, dtype):
    """R2_OP_SUM_FORWARD alone: local gets the sum, the outgoing stage the incoming data."""
    rng = np.random.default_rng(11)
    es = 4 if dtype == "f32" else 2
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    C = 3
    for n_el in (4, 1000, 40000, 300001):
        say(f"relay step {dtype} n_el={n_el}")
        nbytes = n_el * es
        local, incoming = _inputs(rng, 2, n_el, dtype)
        in_off = oracle.partition([3, 1, 2], 0, nbytes, 16)
        out_off = oracle.partition([1, 1, 1], 0b010, nbytes, 16)
        cap = (nbytes + 15) // 16 * 16 + 32
        o_in = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        raw = incoming.view(np.uint8)
        for k in range(C):
            a, b = int(in_off[k]), int(in_off[k + 1])
            o_in[k][:b - a] = raw[a:b]
        o_out = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        o_local = local.copy()
        oracle.reduce_copy(o_local, odt, oracle.OP_SUM_FORWARD, o_in, in_off, o_out, out_off, C, cap)
        d_local = _dev(local.copy())
        d_in = [_dev(a.copy()) for a in o_in]
        d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]
        r2.r2_reduce_copy(d_local, gdt, r2.OP_SUM_FORWARD, d_in, _dev(in_off), d_out, _dev(out_off), C, cap, nbytes=nbytes)
        torch.cuda.synchronize()
        assert d_local.cpu().numpy().tobytes() == o_local.tobytes()
        for k in range(C):
            assert d_out[k].cpu().numpy().tobytes() == o_out[k].tobytes()
    with pytest.raises(r2.R2Error):
        r2.r2_reduce_copy(d_local, gdt, r2.OP_SUM_FORWARD, d_in, _dev(in_off), None, None, C, cap, nbytes=nbytes)
