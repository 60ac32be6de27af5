"""GPU parity: a ring whose ranks lost different rails (R2_PHASE_LINKS, r2_ring_rails_sim; Sec. 6) vs the
oracle, byte for byte: rank buffers, the per-link tables, the stage area; and the bridge re-ranking
feeding the ring order."""
import numpy as np
import pytest
import torch

from gpu_util import FILL, assert_same_stage, say
from oracle import rails

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


def _run(r2, oracle, xs, dtype, phases, S, C, align, weights, masks, window=0, check_stage=True, schedules=None):
    """``schedules``: per-rank epoch lists; by default the static state (weights, masks[r]) of every rank.
    Runs the case under R2_SCHED_AUTO, under the step schedule and, where the library accepts it, under
    fused columns; returns the schedules that ran (AUTO as what it resolved to)."""
    R, N = len(xs), xs[0].size
    if schedules is None:
        schedules = rails.static_epochs(weights, masks)
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    gph = {"rs": r2.PHASE_RS, "ag": r2.PHASE_AG, "ar": r2.PHASE_AR}[phases] | r2.PHASE_LINKS
    oph = {"rs": oracle.PHASE_RS, "ag": oracle.PHASE_AG, "ar": oracle.PHASE_AR}[phases]
    n_tx = S * ((2 * R - 2) if phases == "ar" else (R - 1))
    o_bufs = [x.copy() for x in xs]
    tables, stage = rails.ring_rails_sim(o_bufs, odt, S, C, align, schedules, oph, FILL)
    want = oracle.expected(xs, odt, S, oph)
    ran = []
    for sched in (r2.SCHED_AUTO, r2.SCHED_STEPS, r2.SCHED_FUSED):
        desc = r2.SimDesc(R, S, C, align, N, gdt, gph, window, sched)
        assert r2.r2_sim_num_transmissions(desc) == R * n_tx  # a block of tables per link
        with pytest.raises(r2.R2Error):  # one epoch list says nothing about per-link tables
            r2.r2_sim_resolve_schedule(desc, [(0, 0, [1] * C)])
        try:
            resolved = r2.r2_rails_resolve_schedule(desc, schedules)
        except r2.R2Error as e:  # fused columns do not fit this case (ragged vectors, or too many rows for LDS)
            assert sched == r2.SCHED_FUSED and e.code == -1
            continue
        assert resolved == sched or sched == r2.SCHED_AUTO
        if resolved in ran:
            continue  # AUTO already ran this schedule
        say(f"  schedule {sched} -> {resolved}")
        ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
        log = torch.full((R, n_tx, C + 1), -1, dtype=torch.int64, device="cuda")
        bufs = [_dev(x) for x in xs]
        r2.r2_ring_rails_sim(desc, bufs, schedules, ws, log)
        torch.cuda.synchronize()
        for r in range(R):
            got = bufs[r].cpu().numpy().view(xs[r].dtype)
            assert got.tobytes() == want[r].tobytes(), f"rank {r} vs definition"
            assert got.tobytes() == o_bufs[r].tobytes(), f"rank {r} vs step-by-step oracle"
        assert log.cpu().numpy().view(np.uint64).tolist() == tables.tolist()
        assert ws[:R * n_tx * (C + 1) * 8].cpu().numpy().view(np.uint64).reshape(R, n_tx, C + 1).tolist() == tables.tolist()
        if check_stage or resolved == r2.SCHED_FUSED:  # fused columns run no passes
            cap = r2.r2_sim_stage_capacity(desc)
            off = r2.r2_sim_stage_offset(desc)
            st = ws[off:off + 2 * R * S * C * cap].cpu().numpy()
            assert_same_stage(st, stage)
        ran.append(resolved)
    return ran


@pytest.mark.parametrize("phases", ["rs", "ag", "ar"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rails_small(r2, oracle, dtype, phases):
    rng = np.random.default_rng(900)
    per16 = 4 if dtype == "f32" else 8
    w = [50000, 25000, 50000, 12500, 50000, 50000, 1, 50000]
    for R, S, E in ((2, 1, per16 * 100), (4, 3, per16 * 1031), (8, 2, 7), (3, 2, per16 * 512 * 5 + 3), (5, 1, per16 * 512 * 2)):
        masks = [int(rng.integers(0, 256)) & ~0b00010000 for _ in range(R)]  # rail 4 survives everywhere
        say(f"rails {phases} {dtype} R={R} S={S} E={E} masks={masks}")
        ran = _run(r2, oracle, _inputs(rng, R, S * R * E, dtype), dtype, phases, S, 8, 256, w, masks)
        assert (r2.SCHED_FUSED in ran) == (E % per16 == 0)  # whole 16-byte vectors: fused columns ran too


@pytest.mark.parametrize("seed", [1, 2])
def test_rails_random_configurations(r2, oracle, seed):
    rng = np.random.default_rng(910 + seed)
    for case in range(20):
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        phases = ("rs", "ag", "ar")[int(rng.integers(0, 3))]
        R, S, C = int(rng.integers(2, 12)), int(rng.integers(1, 4)), int(rng.integers(1, 12))
        E = int(rng.integers(1, 2500))
        align = (16, 64, 256)[int(rng.integers(0, 3))]
        w = [int(x) for x in rng.integers(1, 1000, C)]
        up = int(rng.integers(0, C))
        masks = [int(rng.integers(0, 1 << C)) & ~(1 << up) if rng.random() < 0.7 else 0 for _ in range(R)]
        window = (0, 1, 4096, 50000)[int(rng.integers(0, 4))]
        schedules = None
        if case % 2:  # every rank's state also changes on the way: failures, recoveries, other speeds
            n_tx = S * ((2 * R - 2) if phases == "ar" else (R - 1))
            schedules = []
            for r in range(R):
                eps = [(0, masks[r], w)]
                for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, int(rng.integers(0, 3))))):
                    eps.append((t, int(rng.integers(0, 1 << C)) & ~(1 << up), [int(x) for x in rng.integers(1, 1000, C)]))
                schedules.append(eps)
        say(f"rails random {seed}.{case} {phases} {dtype} R={R} S={S} C={C} E={E} align={align} window={window} masks={masks} "
            f"changes={[len(e) - 1 for e in schedules] if schedules else 0}")
        # with passes and tables that change on the way the stage area's leftovers depend on the pass order
        _run(r2, oracle, _inputs(rng, R, S * R * E, dtype), dtype, phases, S, C, align, w, masks, window,
             schedules is None or window == 0, schedules)


@pytest.mark.parametrize("seed", [1, 2])
def test_rails_fused_columns_random(r2, oracle, seed):
    """Ring chunks of whole 16-byte vectors, so that fused columns run: narrow and wide columns, a ragged
    last column, more ranks than a workgroup has waves, tables that change on the way (launch cuts)."""
    rng = np.random.default_rng(930 + seed)
    fused_runs = 0
    for case in range(16):
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        per16 = 4 if dtype == "f32" else 8
        phases = ("rs", "ag", "ar")[int(rng.integers(0, 3))]
        R = int(rng.integers(17, 23)) if case % 4 == 0 or case % 8 == 1 else int(rng.integers(2, 10))
        S, C = int(rng.integers(1, 4)), int(rng.integers(1, 12))
        E = per16 * int(rng.integers(1, 700))
        if case % 5 == 0:
            R, S, E = int(rng.integers(2, 5)), 2, per16 * int(rng.integers(16400, 17000))  # > 256 KiB chunks: wide columns
        align = (16, 64, 256)[int(rng.integers(0, 3))]
        w = [int(x) for x in rng.integers(1, 1000, C)]
        up = int(rng.integers(0, C))
        masks = [int(rng.integers(0, 1 << C)) & ~(1 << up) if rng.random() < 0.7 else 0 for _ in range(R)]
        n_tx = S * ((2 * R - 2) if phases == "ar" else (R - 1))
        schedules = []
        for r in range(R):
            eps = [(0, masks[r], w)]
            if case % 2:
                for t in sorted(set(int(x) for x in rng.integers(1, n_tx + 1, int(rng.integers(0, 3))))):
                    eps.append((t, int(rng.integers(0, 1 << C)) & ~(1 << up), [int(x) for x in rng.integers(1, 1000, C)]))
            schedules.append(eps)
        say(f"rails fused {seed}.{case} {phases} {dtype} R={R} S={S} C={C} E={E} align={align} "
            f"changes={[len(e) - 1 for e in schedules]}")
        ran = _run(r2, oracle, _inputs(rng, R, S * R * E, dtype), dtype, phases, S, C, align, w, masks, 0, True, schedules)
        steps = (2 * R - 1) if phases == "ar" else R
        if R * steps * ((C + 1) * 8 + 24) <= 56 * 1024:  # the rows of even one launch over all steps fit LDS
            assert r2.SCHED_FUSED in ran
        fused_runs += r2.SCHED_FUSED in ran
    assert fused_runs >= 10


def test_rails_maximum_ranks_and_channels_and_large_chunks(r2, oracle):
    rng = np.random.default_rng(920)
    C = 64
    w = [int(x) for x in rng.integers(1, 1000, C)]
    masks = [int(rng.integers(0, 1 << 63)) & ~(1 << 40) for _ in range(64)]
    masks[63] |= 1 << 63
    say("rails R=64 C=64")
    _run(r2, oracle, _inputs(rng, 64, 64 * 8 * 5, "bf16"), "bf16", "ar", 1, C, 16, w, masks)
    say("rails R=32, one rank's state changes at every transmission: fused launches of one or two steps")
    w8 = [50000] * 8
    flapping = [[(t, t & 1, w8) for t in range(62)]] + rails.static_epochs(w8, [0] * 31)
    ran = _run(r2, oracle, _inputs(rng, 32, 32 * 64, "bf16"), "bf16", "ar", 1, 8, 16, w8, None, 0, True, flapping)
    assert ran == [r2.SCHED_STEPS, r2.SCHED_FUSED]
    say("rails R=22 C=11 reduce-scatter: 55,440 bytes of link rows, just under the fused kernel's LDS limit")
    w11 = [int(x) for x in rng.integers(1, 1000, 11)]
    masks22 = [int(rng.integers(0, 1 << 11)) & ~(1 << 6) for _ in range(22)]
    ran = _run(r2, oracle, _inputs(rng, 22, 22 * 4 * 300, "f32"), "f32", "rs", 1, 11, 64, w11, masks22)
    assert r2.SCHED_FUSED in ran
    say("rails 2 MiB chunks, a window that forces byte-range passes")
    xs = _inputs(rng, 4, 4 * (1 << 19), "f32")
    _run(r2, oracle, xs, "f32", "ar", 1, 8, 256, [50000] * 8, [0b1, 0b10, 0, 0b1100], window=3 << 20)


def test_rails_failure_and_recovery_at_one_server(r2, oracle):
    """Server 2 of 4 loses a NIC at transmission 3 and gets a faster one back at 6, with multi-tile chunks."""
    rng = np.random.default_rng(922)
    w = [50000] * 4
    sched = [[(0, 0, w)] for _ in range(4)]
    sched[2] = [(0, 0, w), (3, 0b0010, w), (6, 0, [50000, 100000, 50000, 50000])]
    sched[3] = [(0, 0, w), (6, 0b1000, [50000, 100000, 50000, 50000])]
    say("rails: failure and recovery at one server")
    _run(r2, oracle, _inputs(rng, 4, 2 * 4 * 8 * 1500, "bf16"), "bf16", "ar", 2, 4, 256, w, None, 0, True, sched)


def test_rails_changes_at_both_ends_at_slab_starts_and_beyond_the_run(r2, oracle):
    """Neighbours change state at the same transmission (one link epoch, not two), a state begins exactly
    where a slab begins (no launch cut needed: the slab's stage buffers are its own), and an epoch that
    starts after the last transmission is never in force."""
    rng = np.random.default_rng(924)
    R, S, C = 4, 3, 4
    T = 2 * R - 2  # transmissions per slab
    w, fast = [50000] * C, [50000, 100000, 25000, 50000]
    sched = [[(0, 0, w)] for _ in range(R)]
    sched[0] = [(0, 0, w), (T, 0b0001, w), (2 * T, 0, fast)]              # changes only where slabs begin
    sched[1] = [(0, 0, w), (2, 0b0100, w), (T + 3, 0, w), (S * T + 5, 0b1111, w)]  # the last one never applies
    sched[2] = [(0, 0, w), (2, 0b1000, fast), (T + 3, 0b0010, w)]         # same transmissions as rank 1
    for dtype in ("f32", "bf16"):
        say(f"rails: simultaneous changes, slab-start changes, {dtype}")
        ran = _run(r2, oracle, _inputs(rng, R, S * R * 8 * 350, dtype), dtype, "ar", S, C, 64, w, None, 0, True, sched)
        assert r2.SCHED_FUSED in ran and r2.SCHED_STEPS in ran


def test_rails_call_marshalled_once(r2, oracle):
    """RailsCall issues the same call from arguments marshalled once: two runs on fresh inputs, same bits."""
    rng = np.random.default_rng(923)
    R, C, N = 4, 4, 4 * 8 * 900
    xs = _inputs(rng, R, N, "bf16")
    sched = r2.static_rails([3, 1, 4, 1], [0b0001, 0, 0b0100, 0])
    desc = r2.SimDesc(R, 1, C, 64, N, r2.BF16, r2.PHASE_AR | r2.PHASE_LINKS)
    ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
    bufs = [_dev(x) for x in xs]
    call = r2.RailsCall(desc, bufs, sched, ws)
    want = oracle.expected(xs, oracle.BF16, 1, oracle.PHASE_AR)
    say("rails: RailsCall, two runs")
    for _ in range(2):
        for b, x in zip(bufs, xs):
            b.copy_(_dev(x))
        call.run()
        torch.cuda.synchronize()
        for r in range(R):
            assert bufs[r].cpu().numpy().view(np.uint16).tobytes() == want[r].tobytes()
    with pytest.raises(ValueError):
        r2.RailsCall(desc, bufs, sched[:3], ws)


def test_rerank_then_ring(r2, oracle):
    """Neighbours that lost different rails share nothing; the library's bridge re-ranking moves a healthy
    node between them and the ring over the new order runs."""
    rng = np.random.default_rng(921)
    w = [50000, 50000]
    masks = [0b01, 0b10, 0, 0]
    N = 4 * 8 * 300
    xs = _inputs(rng, 4, N, "bf16")
    desc = r2.SimDesc(4, 1, 2, 256, N, r2.BF16, r2.PHASE_AR | r2.PHASE_LINKS)
    ws = torch.full((r2.r2_sim_workspace_bytes(desc),), FILL, dtype=torch.uint8, device="cuda")
    bufs = [_dev(x) for x in xs]
    say("rails: a link without a channel is refused before any launch")
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_rails_sim(desc, bufs, r2.static_rails(w, masks), ws)
    assert e.value.code == -2
    torch.cuda.synchronize()
    assert all(b.cpu().numpy().view(np.uint16).tobytes() == x.tobytes() for b, x in zip(bufs, xs))
    order, moved = r2.r2_bridge_rerank([0, 1, 2, 3], [~m & 0b11 for m in masks])
    assert moved == 1 and sorted(order) == [0, 1, 2, 3]
    say(f"rails: re-ranked order {order}")
    _run(r2, oracle, [xs[n] for n in order], "bf16", "ar", 1, 2, 256, w, [masks[n] for n in order])


def test_rails_argument_errors(r2):
    w = [1] * 4
    bufs = [torch.ones(4 * 16, dtype=torch.float32, device="cuda") for _ in range(4)]
    desc = r2.SimDesc(4, 1, 4, 16, 64, r2.F32, r2.PHASE_AR | r2.PHASE_LINKS)
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    plain = r2.SimDesc(4, 1, 4, 16, 64, r2.F32, r2.PHASE_AR)
    with pytest.raises(r2.R2Error):  # the flag is missing
        r2.r2_ring_rails_sim(plain, bufs, r2.static_rails(w, [0] * 4), ws)
    with pytest.raises(r2.R2Error):  # per-link tables do not come from epochs
        r2.r2_ring_allreduce_sim(desc, bufs, [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error):
        r2.r2_sim_prepare(desc, [(0, 0, w)], ws)
    with pytest.raises(r2.R2Error):  # too small a workspace
        r2.r2_ring_rails_sim(desc, bufs, r2.static_rails(w, [0] * 4), ws[:256])
    with pytest.raises(r2.R2Error):  # a rank's list does not start at transmission 0
        r2.r2_ring_rails_sim(desc, bufs, [[(1, 0, w)]] + r2.static_rails(w, [0] * 3), ws)
    with pytest.raises(r2.R2Error):  # ... or does not increase
        r2.r2_ring_rails_sim(desc, bufs, [[(0, 0, w), (2, 1, w), (2, 0, w)]] + r2.static_rails(w, [0] * 3), ws)
    with pytest.raises(r2.R2Error) as e:  # rank 1 loses, at transmission 4, the only channel rank 2 has left
        r2.r2_ring_rails_sim(desc, bufs, [[(0, 0, w)], [(0, 0, w), (4, 0b0001, w)], [(0, 0b1110, w)], [(0, 0, w)]], ws)
    assert e.value.code == -2
    for bad in (r2.PHASE_LINKS, r2.PHASE_LINKS | r2.PHASE_SENDRECV, r2.PHASE_LINKS | r2.PHASE_BROADCAST):
        assert r2.r2_sim_num_steps(r2.SimDesc(4, 1, 4, 16, 64, r2.F32, bad)) == 0
    assert r2.r2_sim_num_steps(r2.SimDesc(4, 1, 4, 16, 64, r2.F32, r2.PHASE_AR | r2.PHASE_LINKS, 0, r2.SCHED_FUSED)) == 7
    ragged = r2.SimDesc(4, 1, 4, 16, 4 * 5, r2.F32, r2.PHASE_AR | r2.PHASE_LINKS, 0, r2.SCHED_FUSED)  # 20-byte ring chunks
    with pytest.raises(r2.R2Error):
        r2.r2_rails_resolve_schedule(ragged, r2.static_rails(w, [0] * 4))
    with pytest.raises(r2.R2Error):
        r2.r2_ring_rails_sim(ragged, bufs, r2.static_rails(w, [0] * 4), ws)
    with pytest.raises(r2.R2Error):
        r2.r2_sim_fused_steps(desc, bufs, 0, 2, ws)
    torch.cuda.synchronize()
    assert all(float(b.sum()) == 64.0 for b in bufs)
