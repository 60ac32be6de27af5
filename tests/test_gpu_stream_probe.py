"""The bare kernels of `bench.py --stream-mix` do what their timing is quoted for: every byte of every
stream is moved, nothing beyond it."""
import ctypes
import os

import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def probe():
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2512_25059_amd", "libr2probe.so"))
    lib.r2probe_cold_mix.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int,
                                     ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    lib.r2probe_ring_pattern.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int, ctypes.c_uint64,
                                         ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
    return lib


def _buffers(n, nbytes, guard=4096):
    """Random bytes with a guard band behind each buffer."""
    g = torch.Generator(device="cuda").manual_seed(5)
    full = [torch.randint(0, 256, (nbytes + guard,), dtype=torch.uint8, device="cuda", generator=g) for _ in range(n)]
    return full, [f.clone() for f in full]


def test_cold_copy_moves_every_byte_and_no_other(probe):
    nbytes = 3 * 8192
    bufs, before = _buffers(4, nbytes)
    addrs = (ctypes.c_uint64 * 4)(*[b.data_ptr() for b in bufs])
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    print(f"stream probe: 1R2W, {nbytes} bytes", flush=True)
    assert probe.r2probe_cold_mix(1, 2, addrs, 4, nbytes, 1, stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(bufs[0], before[0]) and torch.equal(bufs[1], before[1])
    for w in (2, 3):
        assert torch.equal(bufs[w][:nbytes], before[0][:nbytes])
        assert torch.equal(bufs[w][nbytes:], before[w][nbytes:])  # guard band untouched


def test_ring_pattern_hands_the_stage_from_launch_to_launch(probe):
    nbytes = 5 * 8192
    bufs, before = _buffers(5, nbytes)
    locs = (ctypes.c_uint64 * 3)(*[b.data_ptr() for b in bufs[:3]])
    sa, sb = bufs[3], bufs[4]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    print(f"stream probe: staged copy, 3 launches of {nbytes} bytes", flush=True)
    # staged copy: launch 0 reads stage b, writes local 0 and stage a; launch 1 reads a, writes local 1 and b; ...
    assert probe.r2probe_ring_pattern(1, locs, 3, sa.data_ptr(), sb.data_ptr(), nbytes, 3, stream) == 0
    torch.cuda.synchronize()
    want = before[4][:nbytes]
    for b in bufs:
        assert torch.equal(b[:nbytes], want)
    for b, old in zip(bufs, before):
        assert torch.equal(b[nbytes:], old[nbytes:])
