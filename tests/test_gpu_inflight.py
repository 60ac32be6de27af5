"""GPU parity: the ring run with failures in flight (Sec. 4.3 Technique II) through the C ABI against
the oracle -- rank buffers, offsets log, the whole stage area and every epoch's failover plan, bit for
bit, under both schedules; the second benchmark configuration at reduced and at full size."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import FILL, codes, say, to_device, to_host
from inflight_util import random_case
from oracle import inflight

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _run_gpu(r2, w, xs, flags, schedule, fill=True):
    dt = r2.F32 if w.dtype == "f32" else r2.BF16
    ph = {"ar": r2.PHASE_AR, "rs": r2.PHASE_RS, "ag": r2.PHASE_AG}[w.phases]
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, dt, ph, 0, schedule)
    bufs = [to_device(x) for x in xs]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    if fill:
        ws.fill_(FILL)
    T = r2.r2_sim_num_transmissions(desc)
    log = torch.full((max(T, 1), w.C + 1), -1, dtype=torch.int64, device="cuda")
    plans = torch.full((len(w.epochs), w.C, w.C + 1), -1, dtype=torch.int64, device="cuda")
    r2.r2_ring_allreduce_sim_inflight(desc, bufs, w.epochs, flags, ws, log, plans)
    torch.cuda.synchronize()
    outs = [to_host(b, x) for b, x in zip(bufs, xs)]
    return outs, log.cpu().numpy().view(np.uint64)[:T], plans.cpu().numpy().view(np.uint64), ws, desc


def _compare(r2, oracle, w, flags, schedule, check_stage=True, full=False):
    _, _, odt, oph = codes(r2, oracle, w)
    xs = wl.make_inputs(w)
    say(f"in flight: {w.name} R={w.R} N={w.N} S={w.S} C={w.C} {w.dtype} {w.phases} schedule={schedule} "
        f"epochs={[(e[0], hex(e[1])) for e in w.epochs]} flags={flags}")
    outs, log, plans, ws, desc = _run_gpu(r2, w, xs, flags, schedule, fill=check_stage)
    if full:  # too large for the oracle's step-by-step ring in a test: the result by its plain definition,
        # the tables and plans from the oracle's partition and failover plan, state by state
        want = oracle.expected(xs, odt, w.S, oph)
        rows = []
        for t in range(log.shape[0]):
            state = [e for e, fl in zip(w.epochs, flags) if e[0] < t or (e[0] == t and not fl)][-1]
            rows.append(oracle.partition(state[2], state[1], w.chunk_bytes, w.align))
        o_log = np.array(rows, dtype=np.uint64)
        o_plans = {i: oracle.rollback_plan(o_log[w.epochs[i][0]], w.epochs[i][2], w.epochs[i - 1][1], w.epochs[i][1], w.align)
                   for i, fl in enumerate(flags) if fl and w.epochs[i][0] < log.shape[0]}
    else:
        cap = r2.r2_sim_stage_capacity(desc)
        want = [x.copy() for x in xs]
        o_log, o_stage, o_plans = inflight.ring_sim_inflight(want, odt, w.S, w.C, w.align, list(w.epochs), flags, oph,
                                                             cap=cap, stage_fill=FILL)
        if check_stage:
            off = r2.r2_sim_stage_offset(desc)
            stage = ws[off:off + o_stage.size].cpu().numpy()
            assert stage.tobytes() == o_stage.tobytes(), "stage area"
    for r in range(w.R):
        assert outs[r].tobytes() == want[r].tobytes(), f"rank {r}"
    assert log.tolist() == o_log.tolist(), "offsets log"
    zero = np.zeros((w.C, w.C + 1), dtype=np.uint64)
    for i in range(len(w.epochs)):
        assert plans[i].tolist() == o_plans.get(i, zero).tolist(), f"plan of epoch {i}"
    return o_plans


@pytest.mark.parametrize("schedule", [1, 2], ids=["steps", "fused"])
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_inflight_random(r2, oracle, seed, schedule):
    rng = np.random.default_rng(seed)
    n_plans = 0
    for _ in range(25):
        w, flags, _ = random_case(rng, vectors_only=schedule == 2)
        n_plans += len(_compare(r2, oracle, w, flags, schedule))
    assert n_plans > 5


@pytest.mark.parametrize("schedule", [1, 2], ids=["steps", "fused"])
def test_inflight_cfg2_scaled(r2, oracle, schedule):
    """cfg2's shape at 1/512 of its size, its two failures striking during transmission 3: several tiles,
    a ragged tail, and the plan next to the run."""
    w = wl.scaled(wl.cfg2(), 8 * (1 << 14) + 8 * 24)
    plans = _compare(r2, oracle, w, [False, True], schedule)
    assert sorted(plans) == [1]


@pytest.mark.parametrize("schedule", [1, 2], ids=["steps", "fused"])
def test_inflight_cfg2_full(r2, oracle, schedule):
    """cfg2 at full size (hand-worked case B of the failover plan): row 3 keeps the even split, the two
    failed 2 MiB slices are shared out over the six survivors, every element of every rank matches."""
    w = wl.cfg2()
    plans = _compare(r2, oracle, w, [False, True], schedule, check_stage=False, full=True)
    assert plans[1][2].tolist() == [0, 349440, 698880, 698880, 1048576, 1398016, 1398016, 1747456, 2097152]
    assert plans[1][5].tolist() == plans[1][2].tolist()


def test_inflight_many_epochs_and_channels(r2, oracle):
    """More epochs than one kernel-argument batch holds (64 channels: ten epochs per batch), every
    second one in flight, a new channel failing each time."""
    R, S, C = 4, 8, 64
    T = S * (2 * R - 2)
    weights = tuple(int(x) for x in np.random.default_rng(3).integers(1, 1000, size=C))
    epochs, flags, mask = [(0, 0, weights)], [False], 0
    for i, t0 in enumerate(range(1, T, 2)):
        mask |= 1 << i
        epochs.append((t0, mask, weights))
        flags.append(i % 2 == 0)
    w = replace(wl.cfg1(), name="inflight_many", R=R, dtype="bf16", N=R * S * 4096, S=S, C=C, align=16, phases="ar",
                sigma=0.5, seed=77, epochs=tuple(epochs))
    assert len(epochs) > 20
    for schedule in (1, 2):
        _compare(r2, oracle, w, flags, schedule, check_stage=schedule == 1)


def test_inflight_without_flags_is_the_plain_run(r2, oracle):
    w = wl.scaled(wl.cfg2(), 8 * 4096)
    _compare(r2, oracle, w, [False, False], 1)
    xs = wl.make_inputs(w)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR)
    bufs = [to_device(x) for x in xs]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    say("in flight: no flags array, no plans array")
    r2.r2_ring_allreduce_sim_inflight(desc, bufs, w.epochs, None, ws)
    torch.cuda.synchronize()
    want = oracle.expected(xs, oracle.BF16, w.S, oracle.PHASE_AR)
    assert all(to_host(b, x).tobytes() == e.tobytes() for b, x, e in zip(bufs, xs, want))


def test_inflight_empty_buffers_still_get_their_plans_written(r2):
    """Nothing to move: the run is a no-op, and every row of the plans is written all the same (zero: an
    empty chunk has empty slices)."""
    eq = tuple([1] * 4)
    desc = r2.SimDesc(4, 2, 4, 16, 0, r2.F32, r2.PHASE_AR)
    bufs = [torch.zeros(4, dtype=torch.float32, device="cuda") for _ in range(4)]
    ws = torch.empty(max(r2.r2_sim_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    plans = torch.full((2, 4, 5), -1, dtype=torch.int64, device="cuda")
    say("in flight: empty buffers")
    r2.r2_ring_allreduce_sim_inflight(desc, bufs, [(0, 0, eq), (3, 0b10, eq)], [False, True], ws, None, plans)
    torch.cuda.synchronize()
    assert int(plans.abs().max()) == 0


def test_inflight_argument_errors(r2):
    w = wl.scaled(wl.cfg2(), 8 * 4096)
    desc = r2.SimDesc(w.R, w.S, w.C, w.align, w.N, r2.BF16, r2.PHASE_AR)
    bufs = [torch.zeros(w.N, dtype=torch.int16, device="cuda") for _ in range(w.R)]
    ws = torch.empty(r2.r2_sim_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    plans = torch.zeros((2, w.C, w.C + 1), dtype=torch.int64, device="cuda")
    eq = tuple([1] * w.C)
    say("in flight: argument errors")
    for epochs, flags, pl, code in [
        ([(0, 0, eq), (3, 0b100, eq)], [True, False], plans, -1),        # the first epoch cannot strike in flight
        ([(0, 0b1, eq), (3, 0b100, eq)], [False, True], plans, -1),      # channel 0 recovers in flight
        ([(0, 0, eq), (3, 0b100, eq)], [False, True], None, -1),         # nowhere to put the plan
        ([(0, 0, eq), (3, 0xFF, eq)], [False, True], plans, -2),         # nobody left to re-carry anything
    ]:
        with pytest.raises(r2.R2Error) as e:
            r2.r2_ring_allreduce_sim_inflight(desc, bufs, epochs, flags, ws, None, pl)
        assert e.value.code == code
    torch.cuda.synchronize()
    assert all(int(b.abs().max()) == 0 for b in bufs)
