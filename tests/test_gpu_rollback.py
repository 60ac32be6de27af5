"""GPU parity: in-flight failover plan through the C ABI vs the oracle, bit for bit."""
import os

import numpy as np
import pytest
import torch

from gpu_util import say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _dev64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.uint64).view(np.int64)).cuda()


def _run(r2, offs, W, mb, ma, align):
    T, C = W.shape
    plan = torch.full((T, C, C + 1), -1, dtype=torch.int64, device="cuda")
    st = torch.zeros(T, dtype=torch.int32, device="cuda")
    r2.r2_rollback_plan_device(_dev64(offs), torch.from_numpy(W.astype(np.uint32).view(np.int32)).cuda(),
                               _dev64(mb), _dev64(ma), align, plan, st)
    torch.cuda.synchronize()
    return plan.cpu().numpy().view(np.uint64), st.cpu().numpy()


@pytest.mark.parametrize("C", [1, 2, 4, 8, 33, 64])
def test_rollback_plan_random(r2, oracle, C):
    rng = np.random.default_rng(900 + C)
    T = 257
    for align in (16, 256):
        say(f"rollback_plan C={C} align={align} T={T}")
        W = rng.integers(0, 100000, size=(T, C))
        W[rng.integers(0, 4, size=T) == 0] = 50000
        full = (1 << C) - 1
        mb = np.array([int(rng.integers(0, 2 ** 62)) & full for _ in range(T)], dtype=np.uint64)
        mb[rng.integers(0, 2, size=T) == 0] = 0
        ma = np.array([int(b) | (int(rng.integers(0, 2 ** 62)) & int(rng.integers(0, 2 ** 62)) & full) for b in mb], dtype=np.uint64)
        nbytes = rng.integers(0, 1 << 30, size=T)
        offs = np.zeros((T, C + 1), dtype=np.uint64)
        valid = np.ones(T, dtype=bool)
        for p in range(T):
            try:
                offs[p] = oracle.partition(W[p], int(mb[p]), int(nbytes[p]), align)
            except oracle.NoHealthyChannel:
                valid[p] = False  # leave a zero table: nothing to fail over
        plan, st = _run(r2, offs, W, mb, ma, align)
        for p in range(T):
            try:
                want = oracle.rollback_plan(offs[p], W[p], int(mb[p]), int(ma[p]), align)
                assert st[p] == 0, p
            except oracle.NoHealthyChannel:
                assert st[p] == -2, p
                # rows that could be served are still filled in by both sides; the others are zero
                want = None
            if want is not None:
                assert plan[p].tolist() == want.tolist(), (p, hex(int(mb[p])), hex(int(ma[p])))
            else:
                alive = [0 if (int(ma[p]) >> c) & 1 else int(W[p, c]) for c in range(C)]
                assert sum(alive) == 0 and not plan[p].any()


def test_rollback_plan_worked_examples(r2):
    golden = os.path.join(os.path.dirname(__file__), "golden", "rollback_cases.txt")
    for line in open(golden):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, w, mb, ma, align, off, rows, status = [s.strip() for s in line.split("|")]
        say(f"rollback_plan golden {name}")
        w = np.array([[int(x) for x in w.split()]])
        C = w.shape[1]
        plan, st = _run(r2, np.array([[int(x) for x in off.split()]], dtype=np.uint64), w,
                        np.array([int(mb, 16)], dtype=np.uint64), np.array([int(ma, 16)], dtype=np.uint64), int(align))
        assert st[0] == int(status)
        want = np.zeros((C, C + 1), dtype=np.uint64)
        for part in rows.split(";"):
            if part.strip():
                f, vals = part.split(":")
                want[int(f)] = [int(x) for x in vals.split()]
        assert plan[0].tolist() == want.tolist()
