"""GPU parity: the recursive R2CCL-AllReduce schedule (Sec. 6) through the C ABI vs the oracle, bit for
bit: against the oracle's step-by-step schedule and against the definition of the result."""
import numpy as np
import pytest
import torch

from gpu_util import FILL, say
from oracle import recursive as rec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _inputs(rng, R, N, dtype, sigma=1.0):
    xs = []
    for _ in range(R):
        x = (rng.standard_normal(N) * sigma).astype(np.float32)
        if dtype == "bf16":
            x = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        xs.append(x)
    return xs


def _dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def _levels(r2, plan):
    return [r2.Level(sum(1 << r for r in l.members), l.fail_mask, l.bandwidth, l.increment, float(l.share))
            for l in plan]


def _run(r2, oracle, xs, dtype, plan, elems, S, C, align, weights, masks, schedule=0, step_by_step=True):
    R, N = len(xs), xs[0].size
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    levels = _levels(r2, plan)
    desc = r2.RecursiveDesc(R, C, align, N, gdt, len(levels), S, schedule)
    need = r2.r2_recursive_workspace_bytes(desc, levels, elems)
    assert need > 0
    ws = torch.full((need,), FILL, dtype=torch.uint8, device="cuda")
    bufs = [_dev(x) for x in xs]
    r2.r2_recursive_allreduce_sim(desc, bufs, weights, masks, levels, elems, ws)
    torch.cuda.synchronize()
    outs = [b.cpu().numpy().view(x.dtype) for b, x in zip(bufs, xs)]
    want = rec.recursive_expected(xs, odt, plan, elems, S)
    for r in range(R):
        assert outs[r].tobytes() == want[r].tobytes(), f"rank {r} vs definition"
    if step_by_step:
        o_bufs = [x.copy() for x in xs]
        trace = rec.recursive_sim(o_bufs, odt, plan, elems, S, C, align, weights, masks)
        for r in range(R):
            assert outs[r].tobytes() == o_bufs[r].tobytes(), f"rank {r} vs step-by-step oracle"
        # Every level has its own part of the workspace: the ring's workspace (its per-link tables come
        # first), the chain's hop tables (room for a relay on every hop), the chain's stage, and the
        # place relayed data lands in.
        es = xs[0].itemsize
        up = lambda x: (x + 255) // 256 * 256
        at = 0
        for lv, n, tr in zip(plan, elems, trace):
            if n == 0:
                continue
            p = len(lv.members)
            assert r2.r2_recursive_ring_order(C, masks, sum(1 << r for r in lv.members)) == lv.order
            ring = r2.SimDesc(p, S, C, align, n, gdt, r2.PHASE_AR | r2.PHASE_LINKS, 0, schedule)
            ring_tables, visits, tables, stage = tr
            got_ring = ws[at: at + ring_tables.size * 8].cpu().numpy().view(np.uint64).reshape(ring_tables.shape)
            assert got_ring.tolist() == ring_tables.tolist(), f"per-link tables of the ring {lv.order}"
            at += up(r2.r2_sim_workspace_bytes(ring))
            if visits is None:
                continue
            cap = up(n * es)
            got_tab = ws[at: at + tables.size * 8].cpu().numpy().view(np.uint64).reshape(tables.shape)
            assert got_tab.tolist() == tables.tolist(), f"hop tables of the chain of the ring {lv.order}"
            hops = p + 2 * (R - p) - 1
            assert len(visits) - 1 <= 2 * hops
            at += up(2 * hops * (C + 1) * 8)
            got_stage = ws[at: at + 2 * C * cap].cpu().numpy().reshape(2, C, cap)
            for par in range(2):
                for c in range(C):
                    assert got_stage[par, c].tobytes() == stage[par][c].tobytes(), \
                        f"chain stage of the ring {lv.order}: parity {par} channel {c}"
            at += 2 * C * cap + cap
        assert at == need
    return outs


CASES = [
    # weights, per-rank failed-channel masks
    ([3, 5, 7, 11], [0b0001, 0b0011, 0, 0b0001, 0]),
    ([50000] * 8, [0b1111, 0b0011, 0, 0]),
    ([50000] * 8, [0, 0, 0b00111100, 0, 0, 0, 0, 0]),               # one degraded rank: Sec. 5.2
    ([5] * 6, [0b000110, 0b000010, 0b000100, 0, 0, 0]),            # two equally slow ranks leave together
    ([50000] * 8, [0] * 6),                                           # no failure: one ring
    ([9, 9, 9], [0b001, 0b011, 0, 0b001, 0, 0, 0b011, 0, 0]),
    ([1] * 8, [0b00001111, 0b11110000, 0, 0, 0, 0]),                  # two servers lost complementary halves: no rail is
                                                                      # up everywhere; re-ranked ring, relayed broadcast hops
    ([1, 1, 1, 1], [0b0011, 0b0100, 0, 0]),                           # the global ring is re-ranked (0 2 1 3)
    ([2, 3, 5, 7, 11, 13], [0b000111, 0b111000, 0b010101, 0, 0b000001, 0, 0]),  # three levels, relays, unequal rails
    ([1] * 8, [0b11111100, 0b00000011, 0, 0]),                        # a relay on the way in only, ahead of the relay's
                                                                      # own turn as a member: its result must survive
    ([1] * 8, [0b11111100, 0b11110011, 0b11111001, 0b00001100, 0]),   # the first member is linked to one end only, a rank
                                                                      # left out to both: the second member relays
    ([50000] * 8, [0b01111111] + [0b00111111] * 5 + [0, 0]),          # shares 48 : 49 : 504, all rings finish together
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("schedule", [1, 2])
def test_recursive_small(r2, oracle, dtype, schedule):
    rng = np.random.default_rng(500 + schedule)
    per16 = 4 if dtype == "f32" else 8
    for weights, masks in CASES:
        plan = rec.plan(weights, masks)
        R, C = len(masks), len(weights)
        for S, unit in ((1, 37), (2, 5), (1, 1)):
            elems = [S * len(l.members) * per16 * unit * (1 + (k + 1) % 3) for k, l in enumerate(plan)]
            say(f"recursive {dtype} sched={schedule} R={R} C={C} levels={len(plan)} S={S} elems={elems}")
            xs = _inputs(rng, R, sum(elems), dtype)
            _run(r2, oracle, xs, dtype, plan, elems, S, C, 16, weights, masks, schedule)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_recursive_random_failure_patterns(r2, oracle, seed):
    """Random failure patterns: ranks lose random channels -- no channel is kept up everywhere, so that
    rings get re-ranked and broadcast hops relayed; where the oracle finds no way the product must refuse
    too --, random weights, types, schedules and segment sizes."""
    rng = np.random.default_rng(600 + seed)
    n_multi = n_relay = n_refused = n_reranked = 0
    for case in range(25):
        R, C = int(rng.integers(2, 10)), int(rng.integers(2, 9))
        weights = [int(x) for x in rng.integers(1, 1000, C)]
        masks = []
        for _ in range(R):
            m = 0
            if rng.random() < 0.6:
                m = int(rng.integers(0, 1 << C))
                if m == (1 << C) - 1:
                    m &= ~(1 << int(rng.integers(0, C)))
            masks.append(m)
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        per16 = 4 if dtype == "f32" else 8
        S = int(rng.integers(1, 3))
        schedule = int(rng.integers(0, 2))
        try:
            plan = rec.plan(weights, masks)
        except oracle.NoHealthyChannel:  # a link of the global ring has no channel, re-ranked or not
            n_refused += 1
            with pytest.raises(r2.R2Error) as e:
                r2.r2_recursive_plan(weights, masks)
            assert e.value.code == -2
            continue
        try:
            for lv in plan:
                rec.chain_visits(R, C, masks, lv)
        except oracle.NoHealthyChannel:  # a broadcast hop with no way round: the run itself refuses
            n_refused += 1
            lv = _levels(r2, plan)
            elems = [S * len(l.members) * per16 for l in plan]
            desc = r2.RecursiveDesc(R, C, 16, sum(elems), r2.F32 if dtype == "f32" else r2.BF16, len(lv), S, schedule)
            ws = torch.empty(r2.r2_recursive_workspace_bytes(desc, lv, elems), dtype=torch.uint8, device="cuda")
            bufs = [torch.zeros(sum(elems), dtype=torch.float32 if dtype == "f32" else torch.int16, device="cuda")
                    for _ in range(R)]
            with pytest.raises(r2.R2Error) as e:
                r2.r2_recursive_allreduce_sim(desc, bufs, weights, masks, lv, elems, ws)
            assert e.value.code == -2
            continue
        n_multi += len(plan) > 2
        n_relay += any(role == "relay" for lv in plan for _, role in rec.chain_visits(R, C, masks, lv))
        n_reranked += any(lv.order != sorted(lv.order) and lv.order != rec.ring_order(R, C, [0] * R, lv.members) for lv in plan)
        elems = [S * len(l.members) * per16 * int(rng.integers(0, 40)) for l in plan]
        if sum(elems) == 0:
            elems[0] = S * R * per16
        say(f"recursive random {seed}.{case} {dtype} sched={schedule} R={R} C={C} masks={masks} levels={len(plan)} elems={elems}")
        xs = _inputs(rng, R, sum(elems), dtype)
        _run(r2, oracle, xs, dtype, plan, elems, S, C, (16, 256)[int(rng.integers(0, 2))], weights, masks, schedule)
    say(f"recursive random {seed}: multi-level {n_multi}, with relays {n_relay}, re-ranked {n_reranked}, refused {n_refused}")
    assert n_multi >= 3


def test_recursive_empty_levels_and_truncated_plans(r2, oracle):
    rng = np.random.default_rng(51)
    weights, masks = [50000] * 8, [0b1111, 0b0011, 0, 0, 0b0001]
    full = rec.plan(weights, masks)
    assert len(full) == 4
    for depth in (1, 2, 3, 4):
        plan = rec.plan(weights, masks, 1, depth)
        for empty in range(len(plan)):
            elems = [0 if k == empty else len(l.members) * 4 * 11 for k, l in enumerate(plan)]
            if sum(elems) == 0:
                continue
            say(f"recursive truncated depth={depth} empty level {empty} elems={elems}")
            xs = _inputs(rng, 5, sum(elems), "f32")
            _run(r2, oracle, xs, "f32", plan, elems, 1, 8, 256, weights, masks)


def test_recursive_equals_split_for_one_degraded_rank(r2, oracle):
    """Two levels with one rank left out is R2CCL-AllReduce: same bits as the split entry point."""
    rng = np.random.default_rng(52)
    R, d, C = 6, 4, 8
    weights = [50000] * C
    masks = [0] * R
    masks[d] = 0b00100100
    plan = rec.plan(weights, masks)
    ng, npart = R * 8 * 300, (R - 1) * 8 * 123
    xs = _inputs(rng, R, ng + npart, "bf16", 0.02)
    say(f"recursive vs split R={R} d={d} global={ng} partial={npart}")
    outs = _run(r2, oracle, xs, "bf16", plan, [ng, npart], 1, C, 256, weights, masks)
    desc = r2.SplitDesc(R, d, C, 256, ng + npart, npart, r2.BF16, 0, 1, 1)
    ws = torch.empty(r2.r2_split_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    bufs = [_dev(x) for x in xs]
    r2.r2_split_allreduce_sim(desc, bufs, weights, masks[d], ws)
    torch.cuda.synchronize()
    for r in range(R):
        assert bufs[r].cpu().numpy().view(np.uint16).tobytes() == outs[r].tobytes()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recursive_large(r2, oracle, dtype):
    """Segments of several MiB (many tiles, the step schedule's launch shapes), shares from the plan."""
    rng = np.random.default_rng(53)
    R, C = 8, 8
    weights = [50000] * C
    masks = [0b00001111, 0, 0b00000011, 0, 0, 0b00000001, 0, 0]
    plan = rec.plan(weights, masks)
    assert len(plan) == 4
    total = 8 * 7 * 6 * 5 * 8 * 300
    gdt = r2.F32 if dtype == "f32" else r2.BF16
    elems = r2.r2_recursive_segments(r2.RecursiveDesc(R, C, 256, total, gdt, len(plan), 1, 1), _levels(r2, plan))
    assert elems == rec.segments(plan, R, total, 1, 4 if dtype == "f32" else 2) and all(elems)
    say(f"recursive large {dtype} elems={elems}")
    xs = _inputs(rng, R, total, dtype, 0.02 if dtype == "bf16" else 1.0)
    _run(r2, oracle, xs, dtype, plan, elems, 1, C, 256, weights, masks, schedule=1, step_by_step=False)


def test_recursive_argument_errors(r2):
    weights, masks = [50000] * 4, [0b0011, 0, 0, 0]
    plan = rec.plan(weights, masks)
    levels = _levels(r2, plan)
    elems = [4 * 4 * 3, 3 * 4 * 3]
    N = sum(elems)
    desc = r2.RecursiveDesc(4, 4, 16, N, r2.F32, 2)
    need = r2.r2_recursive_workspace_bytes(desc, levels, elems)
    assert need > 0
    bufs = [torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(4)]
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def fails(code, d=desc, lv=levels, el=elems, w=weights, m=masks, space=ws):
        with pytest.raises(r2.R2Error) as e:
            r2.r2_recursive_allreduce_sim(d, bufs, w, m, lv, el, space)
        assert e.value.code == code

    fails(-4, space=ws[:need - 256])                                          # workspace too small
    fails(-1, el=[elems[0], elems[1] - 12])                             # sizes do not add up
    fails(-1, el=[elems[0] + 4, elems[1] - 4])                          # a segment does not divide into its ring
    fails(-1, lv=[levels[0], r2.Level(0b10011, 0)])                     # members not among the ranks
    fails(-1, lv=[levels[0], r2.Level(0b1111, 0)])                      # not shrinking
    fails(-1, lv=[levels[0], r2.Level(0b1000, 0)])                      # a ring of one
    fails(-1, lv=[r2.Level(0b0111, 0), levels[1]])                      # level 0 must hold everybody
    fails(-2, m=[0b0011, 0b1100, 0b1111, 0])                            # rank 2 has no channel left: no ring through it
    fails(-2, m=[0b0011, 0b1100, 0b0110, 0b1001], d=r2.RecursiveDesc(4, 4, 16, N, r2.F32, 1), lv=[levels[0]],
          el=[N])                                                       # four ranks, every second pair shares nothing
    assert r2.r2_recursive_workspace_bytes(r2.RecursiveDesc(4, 4, 16, N, r2.F32, 0), levels, elems) == 0
    torch.cuda.synchronize()
    assert all(float(b.abs().sum()) == 0.0 for b in bufs)               # nothing ran
