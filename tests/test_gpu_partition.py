"""GPU parity: channel partition through the C ABI vs the oracle, bit for bit."""
import os

import numpy as np
import pytest
import torch

from gpu_util import say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()  # raises if the HIP library is not built: there is no fallback
    assert torch.cuda.is_available()
    return pkg


def _u64_to_i64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.uint64).view(np.int64))


def _run_device(r2, W, masks, nbytes, align):
    T, C = W.shape
    w_d = torch.from_numpy(W.astype(np.uint32).view(np.int32)).cuda()
    m_d = _u64_to_i64(masks).cuda()
    b_d = _u64_to_i64(nbytes).cuda()
    off = torch.full((T, C + 1), -1, dtype=torch.int64, device="cuda")
    st = torch.full((T,), 77, dtype=torch.int32, device="cuda")
    r2.r2_partition_device(w_d, m_d, b_d, align, off, st)
    torch.cuda.synchronize()
    return off.cpu().numpy().view(np.uint64), st.cpu().numpy()


def _alive_sum(w, mask):
    return sum(0 if (mask >> c) & 1 else int(w[c]) for c in range(len(w)))


@pytest.mark.parametrize("C", [1, 2, 3, 4, 8, 17, 63, 64])
def test_partition_device_random(r2, oracle, C):
    rng = np.random.default_rng(1000 + C)
    T = 1031  # not a multiple of the four problems a workgroup takes
    for align in (1, 16, 256, 4096):
        say(f"partition_device C={C} align={align} T={T}")
        kind = rng.integers(0, 3, size=T)
        W = np.where(kind[:, None] == 0, rng.integers(0, 4, size=(T, C)),
                     np.where(kind[:, None] == 1, rng.integers(1, 400001, size=(T, C)),
                              rng.integers(0, 2 ** 32, size=(T, C), dtype=np.uint64).astype(np.int64)))
        masks = rng.integers(0, 2 ** 63, size=T, dtype=np.uint64) & np.uint64((1 << C) - 1 if C < 64 else 2 ** 64 - 1)
        masks[rng.integers(0, 3, size=T) == 0] = 0
        sizes = np.array([0, 1, 100, 4095, 1 << 20, (1 << 24) + 48, 2 ** 64 - 1, 2 ** 63 + 12345], dtype=np.uint64)
        nbytes = np.where(rng.integers(0, 2, size=T) == 0, sizes[rng.integers(0, len(sizes), size=T)],
                          rng.integers(0, 2 ** 40, size=T, dtype=np.uint64))
        off, st = _run_device(r2, W, masks, nbytes, align)
        for p in range(T):
            w = [int(x) for x in W[p]]
            if _alive_sum(w, int(masks[p])) == 0:
                assert st[p] == -2
                assert not off[p].any()
                continue
            assert st[p] == 0
            want = oracle.partition(w, int(masks[p]), int(nbytes[p]), align)
            assert off[p].tolist() == want.tolist(), (p, w, hex(int(masks[p])), int(nbytes[p]), align)


def test_partition_extreme_weights(r2, oracle):
    """All 64 channels at the largest weight, byte counts near 2^64: the 128-bit path."""
    say("partition_device extreme")
    C, T = 64, 8
    W = np.full((T, C), 2 ** 32 - 1, dtype=np.int64)
    W[1::2, ::3] = 1
    masks = np.array([0, 1, 2 ** 63, 0xFFFF, 0, 0xF0F0F0F0F0F0F0F0, 5, 2 ** 64 - 2], dtype=np.uint64)
    nbytes = np.array([2 ** 64 - 1, 2 ** 64 - 256, 2 ** 63, 2 ** 62 + 1, 12345678901234567, 2 ** 64 - 1, 2 ** 50, 2 ** 64 - 1],
                      dtype=np.uint64)
    for align in (1, 16, 256):
        off, st = _run_device(r2, W, masks, nbytes, align)
        for p in range(T):
            want = oracle.partition([int(x) for x in W[p]], int(masks[p]), int(nbytes[p]), align)
            assert st[p] == 0 and off[p].tolist() == want.tolist(), (p, align)


def test_partition_host_call_and_worked_examples(r2, oracle):
    golden = os.path.join(os.path.dirname(__file__), "golden", "partition_cases.txt")
    for line in open(golden):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, w, mask, nbytes, align, off = [s.strip() for s in line.split("|")]
        say(f"r2_partition golden {name}")
        got = r2.r2_partition([int(x) for x in w.split()], int(mask, 16), int(nbytes), int(align))
        assert got == [int(x) for x in off.split()]
    rng = np.random.default_rng(3)
    for _ in range(50):
        C = int(rng.integers(1, 65))
        w = [int(x) for x in rng.integers(0, 100000, size=C)]
        mask = int(rng.integers(0, 2 ** 63)) & ((1 << C) - 1)
        nbytes = int(rng.integers(0, 2 ** 34))
        if _alive_sum(w, mask) == 0:
            with pytest.raises(r2.R2Error) as e:
                r2.r2_partition(w, mask, nbytes, 256)
            assert e.value.code == -2
            continue
        assert r2.r2_partition(w, mask, nbytes, 256) == oracle.partition(w, mask, nbytes, 256).tolist()


def test_partition_device_zero_problems(r2):
    say("partition_device T=0")
    r2.load_library().r2_partition_device(None, None, None, 4, 16, 0, None, None, None)
