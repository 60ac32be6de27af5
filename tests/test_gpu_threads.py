"""GPU: calls that fork onto the library's side streams (the split and the recursive all-reduce) are
issued from two host threads at once, each on a stream and buffers of its own; every result must be
the oracle's, bit for bit.  The library serialises the *issuing* of such calls per device; the work
itself is ordered by events only."""
import threading

import numpy as np
import pytest
import torch

from gpu_util import say
from oracle import recursive as rec
from oracle import split

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _split_case(r2, oracle, rng, R, d):
    C, weights, mask = 4, (50000, 25000, 50000, 12500), 0b0101
    ng, npart = R * 4 * 300, (R - 1) * 4 * 170
    xs = [rng.standard_normal(ng + npart).astype(np.float32) for _ in range(R)]
    desc = r2.SplitDesc(R, d, C, 32, ng + npart, npart, r2.F32, 0, 1, 1)
    want = split.split_expected(xs, oracle.F32, d, npart, 1, 1)
    need = r2.r2_split_workspace_bytes(desc)

    def call(bufs, ws):
        r2.r2_split_allreduce_sim(desc, bufs, weights, mask, ws)

    return xs, want, need, call


def _recursive_case(r2, oracle, rng):
    weights, masks = [50000] * 8, [0b1111, 0b0011, 0, 0, 0b0001]
    plan = rec.plan(weights, masks)
    R, C = len(masks), len(weights)
    elems = [len(l.members) * 4 * 60 * (k + 1) for k, l in enumerate(plan)]
    xs = [rng.standard_normal(sum(elems)).astype(np.float32) for _ in range(R)]
    levels = [r2.Level(sum(1 << r for r in l.members), l.fail_mask, l.bandwidth, l.increment, float(l.share))
              for l in plan]
    desc = r2.RecursiveDesc(R, C, 16, sum(elems), r2.F32, len(levels), 1, 0)
    want = rec.recursive_expected(xs, oracle.F32, plan, elems, 1)
    need = r2.r2_recursive_workspace_bytes(desc, levels, elems)

    def call(bufs, ws):
        r2.r2_recursive_allreduce_sim(desc, bufs, weights, masks, levels, elems, ws)

    return xs, want, need, call


def test_forking_calls_from_two_threads(r2, oracle):
    rng = np.random.default_rng(77)
    cases = [_split_case(r2, oracle, rng, 4, 2), _recursive_case(r2, oracle, rng),
             _split_case(r2, oracle, rng, 6, 0), _recursive_case(r2, oracle, rng)]
    rounds = 6
    errors = []

    def worker(tid):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for i in range(rounds):
                    xs, want, need, call = cases[(2 * i + tid) % len(cases)]
                    bufs = [torch.from_numpy(x).cuda() for x in xs]
                    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
                    stream.synchronize()  # the uploads ran on this stream; keep the case self-contained
                    call(bufs, ws)
                    stream.synchronize()
                    for r, b in enumerate(bufs):
                        if b.cpu().numpy().tobytes() != want[r].tobytes():
                            errors.append(f"thread {tid} round {i} rank {r}")
        except Exception as e:  # noqa: BLE001 - reported below, on the main thread
            errors.append(f"thread {tid}: {e!r}")

    say(f"two host threads x {rounds} forking calls")
    threads = [threading.Thread(target=worker, args=(t,), daemon=True) for t in range(2)]  # daemon: a stuck call must not keep the process alive
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a thread did not finish"
    torch.cuda.synchronize()
    assert not errors, errors
