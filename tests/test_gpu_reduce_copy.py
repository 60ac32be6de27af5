"""GPU parity: one fused reduce-copy through the C ABI vs the oracle, bit for bit, including the
stage buffers byte by byte (sentinels outside the written slices must survive)."""
import zlib

import numpy as np
import pytest
import torch

from gpu_util import FILL, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg

    pkg.load_library()
    assert torch.cuda.is_available()
    return pkg


def _rand_chunk(rng, n_el, dtype, scale=1.0):
    x = (rng.standard_normal(n_el) * scale).astype(np.float32)
    if dtype == "bf16":
        return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    return x


def _dev(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def _case(r2, oracle, rng, dtype, op, n_el, C, has_in, has_out, align=16, local_shift_el=0, slack=64):
    es = 4 if dtype == "f32" else 2
    nbytes = n_el * es
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    gdt = r2.F32 if dtype == "f32" else r2.BF16

    def table():
        while True:
            w = [int(x) for x in rng.integers(0, 5, size=C)]
            mask = int(rng.integers(0, 1 << C)) if C < 63 else 0
            if sum(0 if (mask >> c) & 1 else w[c] for c in range(C)):
                return oracle.partition(w, mask, nbytes, align)

    in_off = table() if has_in else None
    out_off = table() if has_out else None
    cap = (nbytes + 15) // 16 * 16 + slack
    local = _rand_chunk(rng, n_el, dtype)
    incoming = _rand_chunk(rng, n_el, dtype)

    # oracle side
    o_local = local.copy()
    o_in = None
    if has_in:
        o_in = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        raw = incoming.view(np.uint8)
        for k in range(C):
            a, b = int(in_off[k]), int(in_off[k + 1])
            o_in[k][:b - a] = raw[a:b]
    o_out = [np.full(cap, FILL, np.uint8) for _ in range(C)] if has_out else None
    oracle.reduce_copy(o_local, odt, op, o_in, in_off, o_out, out_off, C, cap)

    # HIP side: local sits inside a padded allocation so that overruns show up, optionally at an
    # address that is only element-aligned
    pad = 64  # elements
    host = np.full(n_el + 2 * pad + 8, 0, dtype=local.dtype)
    guard = _rand_chunk(rng, host.size, dtype)
    host[:] = guard
    start = pad + local_shift_el
    host[start:start + n_el] = local
    d_all = _dev(host)
    d_local = d_all[start:start + n_el]
    d_in = [_dev(a.copy()) for a in o_in] if has_in else None
    d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)] if has_out else None
    d_in_off = _dev(in_off) if has_in else None
    d_out_off = _dev(out_off) if has_out else None
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    r2.r2_reduce_copy(d_local, gdt, op, d_in, d_in_off, d_out, d_out_off, C, cap, status, nbytes=nbytes)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    got_all = d_all.cpu().numpy().view(local.dtype)
    assert got_all[start:start + n_el].tobytes() == o_local.tobytes()
    assert got_all[:start].tobytes() == guard[:start].tobytes()
    assert got_all[start + n_el:].tobytes() == guard[start + n_el:].tobytes()
    if has_out:
        for k in range(C):
            assert d_out[k].cpu().numpy().tobytes() == o_out[k].tobytes(), f"out stage {k}"
    if has_in:
        for k in range(C):
            assert d_in[k].cpu().numpy().tobytes() == o_in[k].tobytes(), f"in stage {k} was modified"


SIZES_F32 = [1, 3, 4, 5, 1000, 4096, 4 * 1024 * 4 + 4, 300001]  # elements; 16 KiB tile = 4096 fp32
SIZES_BF16 = [1, 7, 8, 9, 2001, 8192, 8 * 1024 * 3 + 10, 600007]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("variant", ["send", "sum", "sum_last", "copy", "copy_last"])
def test_reduce_copy_parity(r2, oracle, dtype, variant):
    rng = np.random.default_rng(zlib.crc32(f"{dtype}/{variant}".encode()))
    op = oracle.OP_COPY if variant.startswith("copy") else oracle.OP_SUM
    has_in = variant != "send"
    has_out = not variant.endswith("last")
    for n_el in (SIZES_F32 if dtype == "f32" else SIZES_BF16):
        for C in (1, 3, 8):
            for align in (16, 256):
                say(f"reduce_copy {dtype} {variant} n_el={n_el} C={C} align={align}")
                _case(r2, oracle, rng, dtype, op, n_el, C, has_in, has_out, align=align)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reduce_copy_element_aligned_local(r2, oracle, dtype):
    """A local chunk whose address is not a multiple of 16 takes the element-wise route."""
    rng = np.random.default_rng(77)
    for shift in (1, 2, 3):
        for n_el in (5, 1000, 70001):
            say(f"reduce_copy unaligned {dtype} shift={shift} n_el={n_el}")
            _case(r2, oracle, rng, dtype, oracle.OP_SUM, n_el, 4, True, True, local_shift_el=shift)
            _case(r2, oracle, rng, dtype, oracle.OP_COPY, n_el, 4, True, True, local_shift_el=shift)
            _case(r2, oracle, rng, dtype, oracle.OP_SUM, n_el, 4, False, True, local_shift_el=shift)


def test_reduce_copy_64_channels(r2, oracle):
    rng = np.random.default_rng(78)
    say("reduce_copy C=64")
    _case(r2, oracle, rng, "f32", oracle.OP_SUM, 100003, 64, True, True)
    _case(r2, oracle, rng, "bf16", oracle.OP_SUM, 100003, 64, True, True)


def test_reduce_copy_special_values(r2, oracle):
    """Denormals are kept, infinities and rounding ties behave as in the oracle."""
    say("reduce_copy special values")
    C, cap = 2, 4096
    for dtype, odt, gdt in (("f32", oracle.F32, r2.F32), ("bf16", oracle.BF16, r2.BF16)):
        if dtype == "f32":
            bits_a = np.array([1, 3, 0x007FFFFF, 0x7F7FFFFF, 0x7F800000, 0x80000001, 0x3F800000, 0x00800000] * 4, dtype=np.uint32)
            bits_b = np.array([1, 5, 1, 0x7F7FFFFF, 0xFF7FFFFF, 0x00000001, 0x33800000, 0x80800001] * 4, dtype=np.uint32)
            a, b = bits_a.view(np.float32), bits_b.view(np.float32)
        else:
            a = np.array([0x0001, 0x0003, 0x007F, 0x7F7F, 0x7F80, 0x8001, 0x3F80, 0x3F80, 0x3F81, 0x4000, 0x0080, 0x3F80] * 4, dtype=np.uint16)
            b = np.array([0x0001, 0x0005, 0x0001, 0x7F7F, 0xFF7F, 0x0001, 0x3B80, 0x3C00, 0x3B80, 0x3C00, 0x8081, 0x3C80] * 4, dtype=np.uint16)
        nbytes = a.nbytes
        off = oracle.partition([1, 1], 0, nbytes, 16)
        o_in = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        raw = a.view(np.uint8)
        for k in range(C):
            lo, hi = int(off[k]), int(off[k + 1])
            o_in[k][:hi - lo] = raw[lo:hi]
        o_out = [np.full(cap, FILL, np.uint8) for _ in range(C)]
        o_local = b.copy()
        oracle.reduce_copy(o_local, odt, oracle.OP_SUM, o_in, off, o_out, off, C, cap)
        d_local = _dev(b.copy())
        d_in = [_dev(x) for x in o_in]
        d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]
        d_off = _dev(off)
        r2.r2_reduce_copy(d_local, gdt, r2.OP_SUM, d_in, d_off, d_out, d_off, C, cap)
        torch.cuda.synchronize()
        assert d_local.cpu().numpy().tobytes() == o_local.tobytes(), dtype
        for k in range(C):
            assert d_out[k].cpu().numpy().tobytes() == o_out[k].tobytes()


def test_reduce_copy_bad_tables_move_nothing(r2, oracle):
    """A table that does not describe the chunk is refused by the kernel: status set, no byte moved."""
    n_el, C, cap = 4096, 4, 8192
    nbytes = n_el * 4
    good = oracle.partition([1, 1, 1, 1], 0, nbytes, 16)
    bad_tables = {
        "does not start at 0": (good + np.uint64(16)).astype(np.uint64),
        "does not end at bytes": np.array([0, 4096, 8192, 12288, nbytes - 16], dtype=np.uint64),
        "decreasing": np.array([0, 8192, 4096, 12288, nbytes], dtype=np.uint64),
        "cut not on 16 bytes": np.array([0, 4100, 8192, 12288, nbytes], dtype=np.uint64),
        "all zero (failed partition)": np.zeros(5, dtype=np.uint64),
    }
    too_long = np.array([0, 0, 0, 0, nbytes], dtype=np.uint64)  # one slice of 16 KiB > cap 8 KiB
    rng = np.random.default_rng(5)
    for name, tab in list(bad_tables.items()) + [("slice exceeds capacity", too_long)]:
        say(f"reduce_copy bad table: {name}")
        local = rng.standard_normal(n_el).astype(np.float32)
        d_local = _dev(local.copy())
        d_in = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]
        d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        r2.r2_reduce_copy(d_local, r2.F32, r2.OP_SUM, d_in, _dev(tab), d_out, _dev(good if name != "slice exceeds capacity" else tab),
                          C, cap, status)
        torch.cuda.synchronize()
        want = -4 if name == "slice exceeds capacity" else -1
        assert int(status.item()) == want, name
        assert d_local.cpu().numpy().tobytes() == local.tobytes()
        for k in range(C):
            assert bool((d_out[k] == FILL).all())


def test_reduce_copy_zero_bytes(r2):
    say("reduce_copy bytes=0")
    r2.r2_reduce_copy(None, r2.F32, r2.OP_SUM, [256], 256, None, None, 1, 16, nbytes=0)


def test_reduce_copy_chunk_beyond_4GiB(r2, oracle):
    """A chunk of 4 GiB + 1 MiB + 6 bytes of bf16 (2^31 + 2^19 + 3 elements): slice offsets, stage
    addresses and the ragged tail all lie beyond 32 bits.  Too large for the host oracle as a whole, so
    `oracle.reduce_copy` checks windows of it byte for byte -- the first tile, a MiB either side of the
    2^32-byte boundary, of every cut of the incoming and of the outgoing table, and the ragged end: the
    window's incoming bytes are taken out of the stage buffers by the oracle's incoming table, the
    oracle adds them to the window's local bytes, and the local chunk and the outgoing stage (read back
    through the oracle's outgoing table) must hold exactly that.  The rest of the chunk is compared with
    values built on the GPU with library operations from the definition."""
    from gpu_util import windows_around

    n_el = (1 << 31) + (1 << 19) + 3
    nbytes = n_el * 2
    C = 3
    in_off = oracle.partition([2, 1, 3], 0b000, nbytes, 256)
    out_off = oracle.partition([2, 1, 3], 0b010, nbytes, 256)
    cap = int(max(np.diff(in_off.astype(np.int64)).max(), np.diff(out_off.astype(np.int64)).max()))
    cap = (cap + 255) // 256 * 256
    say(f"reduce_copy beyond 4 GiB: bytes={nbytes} in_off={in_off.tolist()} out_off={out_off.tolist()} cap={cap}")
    g = torch.Generator(device="cuda").manual_seed(99)
    local = torch.randn(n_el, generator=g, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    incoming = torch.randn(n_el, generator=g, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    want = torch.empty_like(local)
    step = 1 << 28  # in pieces: the fp32 temporaries of the whole chunk would be 16 GiB
    for a in range(0, n_el, step):
        b = min(a + step, n_el)
        want[a:b] = (incoming[a:b].float() + local[a:b].float()).to(torch.bfloat16)
    raw_in = incoming.view(torch.uint8)
    d_in = []
    for k in range(C):
        buf = torch.full((cap,), FILL, dtype=torch.uint8, device="cuda")
        a, b = int(in_off[k]), int(in_off[k + 1])
        buf[:b - a] = raw_in[a:b]
        d_in.append(buf)
    d_out = [torch.full((cap,), FILL, dtype=torch.uint8, device="cuda") for _ in range(C)]

    def through_table(bufs, off, a, b):
        """Bytes [a, b) of the chunk as the stage buffers hold them under table `off` (host copy)."""
        parts = []
        for k in range(C):
            lo, hi = max(a, int(off[k])), min(b, int(off[k + 1]))
            if lo < hi:
                parts.append(bufs[k][lo - int(off[k]):hi - int(off[k])].cpu().numpy())
        return np.concatenate(parts)

    points = [0, 1 << 32, nbytes] + [int(x) for x in in_off] + [int(x) for x in out_off]
    spans = windows_around(points, nbytes, 1 << 20, unit=2)
    local_before = [local.view(torch.uint8)[a:b].cpu().numpy().copy() for a, b in spans]
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    r2.r2_reduce_copy(local.view(torch.int16), r2.BF16, r2.OP_SUM, d_in, _dev(in_off), d_out, _dev(out_off), C, cap,
                      status, nbytes=nbytes)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    for (a, b), loc in zip(spans, local_before):
        n = b - a
        one = np.array([0, n], dtype=np.uint64)  # the window as a chunk of its own, one channel each way
        o_local = loc.view(np.uint16).copy()
        o_in = [through_table(d_in, in_off, a, b)]
        o_out = [np.full(n, FILL, np.uint8)]
        oracle.reduce_copy(o_local, oracle.BF16, oracle.OP_SUM, o_in, one, o_out, one, 1, n)
        assert local.view(torch.uint8)[a:b].cpu().numpy().tobytes() == o_local.tobytes(), f"local bytes [{a}, {b})"
        assert through_table(d_out, out_off, a, b).tobytes() == o_out[0].tobytes(), f"outgoing stage, bytes [{a}, {b})"
    assert torch.equal(local.view(torch.int16), want.view(torch.int16))
    raw_want = want.view(torch.uint8)
    for k in range(C):
        a, b = int(out_off[k]), int(out_off[k + 1])
        assert torch.equal(d_out[k][:b - a], raw_want[a:b]), f"out stage {k}"
        assert bool((d_out[k][b - a:] == FILL).all()), f"out stage {k}: bytes beyond the slice"
    del local, incoming, want, d_in, d_out
    torch.cuda.empty_cache()
