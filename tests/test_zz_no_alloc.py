"""GPU: the entry point whose workspace is the library's static device array (for callers that cannot
allocate) against r2_ring_allreduce_sim with a caller-allocated workspace, and against the oracle.

Two calls in a row share the one array; the second is smaller than the first, so it runs over what
the first left behind.  Buffers and offsets logs must agree bit for bit.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import codes, expected_log, run_gpu_sim, say, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _run_static(r2, w, xs, schedule):
    dt = r2.F32 if w.dtype == "f32" else r2.BF16
    ph = {"ar": r2.PHASE_AR, "rs": r2.PHASE_RS, "ag": r2.PHASE_AG}[w.phases]
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, dt, ph, 0, schedule)
    assert 0 < r2.r2_sim_workspace_bytes(desc) <= r2.STATIC_WORKSPACE_BYTES
    bufs = [to_device(x) for x in xs]
    T = r2.r2_sim_num_transmissions(desc)
    log = torch.full((max(T, 1), w.C + 1), -1, dtype=torch.int64, device="cuda")
    r2.r2_ring_allreduce_sim_static(desc, bufs, w.epochs, log)
    torch.cuda.synchronize()
    return [to_host(b, x) for b, x in zip(bufs, xs)], log.cpu().numpy().view(np.uint64)[:T]


# (first call, second and smaller call): state changes mid-run, ragged tails, both element types
PAIRS = [
    (lambda: wl.scaled(wl.cfg2(), 8 * (1 << 16) + 8 * 24), lambda: wl.scaled(wl.cfg2(), 8 * 8192 * 2 + 8 * 8)),
    (lambda: wl.cfg5(256), lambda: wl.cfg5(16)),
    (lambda: wl.scaled(wl.cfg4(S=32), 8 * 32 * 1104), lambda: wl.scaled(wl.cfg1(), 4 * 4096 * 3 + 4 * 8)),
]


@pytest.mark.parametrize("schedule", [1, 2], ids=["steps", "fused"])
@pytest.mark.parametrize("pair", PAIRS, ids=["cfg2_mid_failure", "cfg5_tok256_then_tok16", "cfg4_flapping_then_cfg1_f32"])
def test_static_workspace_matches_caller_workspace(r2, oracle, pair, schedule):
    for which, make in zip(("first", "second, smaller"), pair):
        w = make()
        _, _, odt, oph = codes(r2, oracle, w)
        xs = wl.make_inputs(w)
        say(f"static workspace, {which} call: {w.name} N={w.N} S={w.S} {w.dtype} schedule={schedule}")
        got, got_log = _run_static(r2, w, xs, schedule)
        say(f"caller workspace, same case: {w.name}")
        ref, ref_log, _, _ = run_gpu_sim(r2, w, xs, schedule=schedule)
        want = oracle.expected(xs, odt, w.S, oph)
        for r in range(w.R):
            assert got[r].tobytes() == ref[r].tobytes(), f"{w.name} ({which}): rank {r} differs from the caller-workspace run"
            assert got[r].tobytes() == want[r].tobytes(), f"{w.name} ({which}): rank {r} differs from the oracle"
        assert got_log.tolist() == ref_log.tolist()
        assert got_log.tolist() == expected_log(oracle, w).tolist()


@pytest.mark.parametrize("schedule", [1, 2], ids=["steps", "fused"])
def test_static_workspace_run_in_a_graph(r2, oracle, schedule):
    """What the entry point is for: a caller under graph capture, where nothing may be allocated.  One
    eager call first (the array's address is looked up then), then the call is captured and replayed
    four times from pristine inputs, every replay against the oracle."""
    w = wl.cfg5(64)
    _, _, odt, oph = codes(r2, oracle, w)
    xs = wl.make_inputs(w)
    want = oracle.expected(xs, odt, w.S, oph)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR, 0, schedule)
    pristine = [to_device(x) for x in xs]
    bufs = [p.clone() for p in pristine]
    say(f"static workspace under graph capture, schedule={schedule}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        r2.r2_ring_allreduce_sim_static(desc, bufs, w.epochs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r2.r2_ring_allreduce_sim_static(desc, bufs, w.epochs)
    for replay in range(4):
        for b, p in zip(bufs, pristine):
            b.copy_(p)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for r in range(w.R):
            assert np.array_equal(to_host(bufs[r], xs[r]), want[r]), f"replay {replay}, rank {r}"


def test_static_workspace_refuses_what_does_not_fit(r2):
    """A run that needs more than the array holds is refused before anything is launched; the same
    arguments that r2_ring_allreduce_sim refuses are refused here too."""
    w = wl.scaled(wl.cfg2(), 8 * (1 << 20))  # 2 MiB chunks: 2 x 8 x 8 x 2 MiB = 256 MiB of stage
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR)
    assert r2.r2_sim_workspace_bytes(desc) > r2.STATIC_WORKSPACE_BYTES
    bufs = [torch.zeros(w.N, dtype=torch.int16, device="cuda") for _ in range(w.R)]
    say("static workspace: oversize run must be refused")
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim_static(desc, bufs, w.epochs)
    assert e.value.code == -4
    torch.cuda.synchronize()
    assert all(int(b.abs().max()) == 0 for b in bufs)
    small = r2.SimDesc(8, 1, 8, 256, 8 * 64, r2.BF16, r2.PHASE_AR)
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim_static(small, [b[:512] for b in bufs], [(0, 0xFF, [1] * 8)])
    assert e.value.code == -2  # no healthy channel
    overlapped = r2.SimDesc(8, 1, 8, 256, 8 * 64, r2.BF16, r2.PHASE_AR, 0, r2.SCHED_STEPS_OVERLAP)
    with pytest.raises(r2.R2Error) as e:  # would create a side stream and events at first use
        r2.r2_ring_allreduce_sim_static(overlapped, [b[:512] for b in bufs], [(0, 0, [1] * 8)])
    assert e.value.code == -1
