"""The entry points only enqueue kernels on the caller's stream (no allocation, no copy, no wait), so a
whole ring run can be captured in a HIP graph and replayed.  Every replay is checked against the
oracle, with ordinary eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import codes, say, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


@pytest.mark.parametrize("schedule", [1, 2])
def test_ring_run_in_a_graph(r2, oracle, schedule):
    w = wl.scaled(wl.cfg2(), 8 * 8192 * 4)
    dt, ph, odt, oph = codes(r2, oracle, w)
    xs = wl.make_inputs(w)
    want = oracle.expected(xs, odt, w.S, oph)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, dt, ph, 0, schedule)
    pristine = [to_device(x) for x in xs]
    bufs = [p.clone() for p in pristine]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    log = torch.zeros((r2.r2_sim_num_transmissions(desc), w.C + 1), dtype=torch.int64, device="cuda")

    say(f"graph capture, schedule={schedule}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r2.r2_ring_allreduce_sim(desc, bufs, w.epochs, ws, log)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r2.r2_ring_allreduce_sim(desc, bufs, w.epochs, ws, log)
    for replay in range(4):
        say(f"graph replay {replay}")
        for b, p in zip(bufs, pristine):
            b.copy_(p)                                   # eager work between replays
        log.zero_()
        junk = torch.randn(1 << 16, device="cuda").sum()  # library kernels in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for r in range(w.R):
            got = bufs[r].cpu().numpy().view(xs[r].dtype)
            assert np.array_equal(got, want[r]), f"replay {replay}, rank {r}"
        assert log.cpu().numpy().any()


def _replayed_run(r2, oracle, w, run, what):
    """Captures `run(bufs)` in a graph after one eager call, replays it four times from pristine inputs
    with eager work in between, and checks every replay against the oracle's result."""
    dt, ph, odt, oph = codes(r2, oracle, w)
    xs = wl.make_inputs(w)
    want = oracle.expected(xs, odt, w.S, oph)
    pristine = [to_device(x) for x in xs]
    bufs = [p.clone() for p in pristine]
    say(f"graph capture: {what}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(bufs)  # once outside the capture: streams, events and symbol addresses are looked up here
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(bufs)
    for replay in range(4):
        say(f"graph replay {replay}: {what}")
        for b, p in zip(bufs, pristine):
            b.copy_(p)
        junk = torch.randn(1 << 16, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for r in range(w.R):
            assert np.array_equal(bufs[r].cpu().numpy().view(xs[r].dtype), want[r]), f"{what}: replay {replay}, rank {r}"


def test_overlapped_passes_in_a_graph(r2, oracle):
    """The overlapped step schedule forks the caller's stream behind its partition launch and joins it
    again: captured, a fork and a join inside the graph.  32 slabs in two groups, a flapping channel."""
    w = wl.scaled(wl.cfg4(S=32), 8 * 32 * 4096)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR, 0, r2.SCHED_STEPS_OVERLAP)
    assert r2.r2_sim_num_passes(desc) == 2
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    _replayed_run(r2, oracle, w, lambda bufs: r2.r2_ring_allreduce_sim(desc, bufs, w.epochs, ws), "overlapped passes")


@pytest.mark.parametrize("schedule", [1, 2])
def test_inflight_run_in_a_graph(r2, oracle, schedule):
    """The run with a failure in flight: its plan launch and the run in one graph; the plan of every
    replay is the oracle's."""
    w = wl.scaled(wl.cfg2(), 8 * 8192 * 4)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR, 0, schedule)
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    plans = torch.zeros((2, w.C, w.C + 1), dtype=torch.int64, device="cuda")

    def run(bufs):
        plans.fill_(-1)  # a fill kernel, captured with the rest: every replay must write the plans anew
        r2.r2_ring_allreduce_sim_inflight(desc, bufs, w.epochs, [False, True], ws, None, plans)

    _replayed_run(r2, oracle, w, run, f"failure in flight, schedule {schedule}")
    old = oracle.partition(w.epochs[0][2], w.epochs[0][1], w.chunk_bytes, w.align)
    want = oracle.rollback_plan(old, w.epochs[1][2], w.epochs[0][1], w.epochs[1][1], w.align)
    got = plans.cpu().numpy().view(np.uint64)
    assert got[0].tolist() == np.zeros_like(want).tolist() and got[1].tolist() == want.tolist()


def test_split_run_in_a_graph(r2, oracle):
    """The split all-reduce forks the caller's stream into a library-owned one and joins it again with
    events; captured, that becomes a fork and a join inside the graph."""
    from oracle import split

    rng = np.random.default_rng(77)
    R, d, C = 5, 2, 8
    ng, npart = R * 8 * 700, (R - 1) * 8 * 300
    xs = []
    for _ in range(R):
        x = torch.from_numpy(rng.standard_normal(ng + npart).astype(np.float32) * 0.02)
        xs.append(x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy())
    weights, mask = [50000] * C, 0b00110000
    want = split.split_expected(xs, oracle.BF16, d, npart, 1, 1)
    desc = r2.SplitDesc(R, d, C, 256, ng + npart, npart, r2.BF16, 0, 1, 1)
    pristine = [to_device(x) for x in xs]
    bufs = [p.clone() for p in pristine]
    ws = torch.empty(r2.r2_split_workspace_bytes(desc), dtype=torch.uint8, device="cuda")

    say("graph capture of the split all-reduce")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)
    for replay in range(3):
        say(f"split graph replay {replay}")
        for b, p in zip(bufs, pristine):
            b.copy_(p)
        junk = torch.randn(1 << 16, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for r in range(R):
            got = bufs[r].cpu().numpy().view(np.uint16)
            assert np.array_equal(got, want[r]), f"replay {replay}, rank {r}"


@pytest.mark.parametrize("schedule", [1, 2])
def test_rails_run_in_a_graph(r2, oracle, schedule):
    """The ring with per-link tables merges the ranks' epoch lists on the host and then only launches:
    captured and replayed under either schedule, with a table change on the way (a launch cut)."""
    from oracle import rails

    rng = np.random.default_rng(78)
    R, C, N = 6, 8, 6 * 8 * 1100
    xs = []
    for _ in range(R):
        x = torch.from_numpy(rng.standard_normal(N).astype(np.float32) * 0.02)
        xs.append(x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy())
    w = [50000] * C
    sched = rails.static_epochs(w, [0b1, 0b10, 0, 0b100, 0, 0b1000])
    sched[2] = [(0, 0, w), (4, 0b00010000, w)]  # rank 2 loses a rail at transmission 4
    want = oracle.expected(xs, oracle.BF16, 1, oracle.PHASE_AR)
    o_bufs = [x.copy() for x in xs]
    tables, _ = rails.ring_rails_sim(o_bufs, oracle.BF16, 1, C, 256, sched, oracle.PHASE_AR)
    desc = r2.SimDesc(R, 1, C, 256, N, r2.BF16, r2.PHASE_AR | r2.PHASE_LINKS, 0, schedule)
    assert r2.r2_rails_resolve_schedule(desc, sched) == schedule
    pristine = [to_device(x) for x in xs]
    bufs = [p.clone() for p in pristine]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    log = torch.zeros((R, 2 * R - 2, C + 1), dtype=torch.int64, device="cuda")

    say(f"graph capture of the per-link ring, schedule={schedule}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r2.r2_ring_rails_sim(desc, bufs, sched, ws, log)  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r2.r2_ring_rails_sim(desc, bufs, sched, ws, log)
    for replay in range(3):
        say(f"rails graph replay {replay}")
        for b, p in zip(bufs, pristine):
            b.copy_(p)
        log.zero_()
        junk = torch.randn(1 << 16, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for r in range(R):
            got = bufs[r].cpu().numpy().view(np.uint16)
            assert np.array_equal(got, want[r]), f"replay {replay}, rank {r}"
        assert log.cpu().numpy().view(np.uint64).tolist() == tables.tolist()
