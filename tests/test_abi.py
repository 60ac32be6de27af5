"""The C ABI without a GPU: the library loads, exports what the header declares, and rejects bad
arguments before any device work."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")
HEADERS = [os.path.join(INCLUDE, "r2ccl.h"), os.path.join(INCLUDE, "r2ccl_ext.h")]


def _header_text():
    return "\n".join(open(h).read() for h in HEADERS)


@pytest.fixture(scope="module")
def r2():
    import paper_2512_25059_amd as pkg
    from paper_2512_25059_amd import build as hip_build

    if hip_build.is_stale():
        hip_build.build()
    pkg.load_library()
    return pkg


def _declared_functions():
    text = _header_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(r2_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(r2):
    names = _declared_functions()
    assert {"r2_partition", "r2_partition_device", "r2_reduce_copy", "r2_ring_allreduce_sim",
            "r2_sim_prepare", "r2_sim_step", "r2_sim_workspace_bytes", "r2_strerror"} <= set(names)
    lib = C.CDLL(r2.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/*.h but not exported"


def test_binding_constants_and_structs_follow_the_header(r2):
    """The Python names carry the header's values, every exported function has a binding of the same name,
    and the descriptor structs are laid out as the C compiler lays them out."""
    text = re.sub(r"/\*.*?\*/", "", _header_text(), flags=re.S)
    enums = dict((k, int(v)) for k, v in re.findall(r"\b(R2_[A-Z0-9_]+)\s*=\s*(-?\d+)", text))
    defines = dict((k, int(v)) for k, v in re.findall(r"#define\s+(R2_[A-Z0-9_]+)\s+(\d+)", text))
    assert len(enums) >= 20
    for name, value in enums.items():
        short = name[3:]
        if short.startswith("ERR_") or short == "OK":
            continue  # error codes travel as R2Error.code
        assert getattr(r2, short) == value, name
    assert r2.MAX_LEVELS == defines["R2_MAX_LEVELS"]
    for fn in _declared_functions():
        assert hasattr(r2, fn) or hasattr(r2.binding, fn), f"no binding for {fn}"
    # struct sizes as gcc computes them from the header
    import subprocess
    import tempfile
    names = ["r2_sim_desc", "r2_split_desc", "r2_recursive_desc", "r2_level", "r2_epoch"]
    src = '#include <stdio.h>\n#include "r2ccl_ext.h"\nint main(void){' + "".join(
        f'printf("%zu\\n", sizeof({n}));' for n in names) + "return 0;}"
    with tempfile.TemporaryDirectory() as d:
        c, exe = os.path.join(d, "s.c"), os.path.join(d, "s")
        open(c, "w").write(src)
        subprocess.run(["gcc", "-I", INCLUDE, c, "-o", exe], check=True)
        sizes = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    b = r2.binding
    assert sizes == [C.sizeof(b._SimDesc), C.sizeof(b._SplitDesc), C.sizeof(b._RecursiveDesc), C.sizeof(b._Level),
                     C.sizeof(b._Epoch)]


def test_strerror(r2):
    assert r2.r2_strerror(0) == "success"
    for code in (-1, -2, -3, -4, -5):
        assert r2.r2_strerror(code) not in ("success", "unknown r2ccl error code")
    assert r2.r2_strerror(-99) == "unknown r2ccl error code"


def test_sim_shape_arithmetic(r2):
    d = r2.SimDesc(n_ranks=8, n_slabs=1, n_channels=8, align=256, n_elems=1 << 26, dtype=r2.BF16,
                   phases=r2.PHASE_AR)
    assert r2.r2_sim_num_steps(d) == 15
    assert r2.r2_sim_num_transmissions(d) == 14
    cap = r2.r2_sim_stage_capacity(d)
    pad = (128 << 10) + 256  # channel buffers of chunks of 1 MiB and more are kept off power-of-two distances
    assert cap == (16 << 20) + pad
    off = r2.r2_sim_stage_offset(d)
    assert off % 256 == 0 and off >= 14 * 9 * 8
    assert r2.r2_sim_workspace_bytes(d) == off + 2 * 8 * 1 * 8 * cap
    rs = r2.SimDesc(16, 4, 8, 256, 1 << 26, r2.F32, r2.PHASE_RS)
    assert r2.r2_sim_num_steps(rs) == 16 and r2.r2_sim_num_transmissions(rs) == 60
    assert r2.r2_sim_stage_capacity(rs) == (4 << 20) + pad
    assert r2.r2_sim_stage_capacity(r2.SimDesc(4, 1, 4, 256, 1 << 20, r2.F32, r2.PHASE_AR)) == (1 << 20) + pad
    assert r2.r2_sim_stage_capacity(r2.SimDesc(8, 1, 8, 256, 1 << 21, r2.BF16, r2.PHASE_AR)) == 512 << 10  # below 1 MiB: none


def test_pass_planning(r2):
    """Passes bound the stage bytes one step writes (over all ranks) by the window."""
    mib = 1 << 20
    # 8 ranks x 16 MiB chunks = 128 MiB per step: exactly the default window, one pass
    d = r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, r2.PHASE_AR)
    assert r2.r2_sim_num_passes(d) == 1
    # 16 ranks x 4 MiB = 64 MiB per slab: two slabs per pass
    assert r2.r2_sim_num_passes(r2.SimDesc(16, 4, 8, 256, 1 << 26, r2.F32, r2.PHASE_RS)) == 2
    # a 32 MiB window cuts the 16 MiB chunks into four byte ranges
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, r2.PHASE_AR, 32 * mib)) == 4
    # 32 slabs of 8 x 256 KiB = 2 MiB each: all in one pass by default, one per pass at 2 MiB
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 32, 8, 256, 1 << 25, r2.BF16, r2.PHASE_AR)) == 1
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 32, 8, 256, 1 << 25, r2.BF16, r2.PHASE_AR, 2 * mib)) == 32
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 32, 8, 256, 1 << 25, r2.BF16, r2.PHASE_AR, 5 * mib)) == 16
    # five slabs of 2 MiB under a 4 MiB window: two per pass, the last pass holds one
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 5, 8, 256, 5 * (1 << 20), r2.BF16, r2.PHASE_AR, 4 * mib)) == 3
    # 128 MiB per step under a 48 MiB window: three byte ranges (two would stage 64 MiB each)
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, r2.PHASE_AR, 48 * mib)) == 3
    # two slabs of 128 MiB per step under a 64 MiB window: two byte ranges of each slab
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 2, 8, 256, 1 << 27, r2.BF16, r2.PHASE_AR, 64 * mib)) == 4
    # the two-step exchanges use one stage parity, so their default window is twice as wide: 8 ranks x 32 MiB
    # messages are one pass, 8 x 64 MiB two
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 1, 8, 256, 1 << 24, r2.BF16, r2.PHASE_SENDRECV)) == 1
    assert r2.r2_sim_num_passes(r2.SimDesc(8, 1, 8, 256, 1 << 25, r2.BF16, r2.PHASE_SENDRECV)) == 2
    # empty input: one empty pass
    assert r2.r2_sim_num_passes(r2.SimDesc(4, 1, 4, 256, 0, r2.F32, r2.PHASE_AR)) == 1
    # per-link tables: a block of rows per ring link, 4 links x 6 transmissions x 5 entries of 8 bytes
    assert r2.r2_sim_stage_offset(r2.SimDesc(4, 1, 4, 256, 4 * 64, r2.F32, r2.PHASE_AR)) == 256
    assert r2.r2_sim_stage_offset(r2.SimDesc(4, 1, 4, 256, 4 * 64, r2.F32, r2.PHASE_AR | r2.PHASE_LINKS)) == 1024


@pytest.mark.parametrize("bad", [
    dict(n_ranks=1), dict(n_ranks=65), dict(n_channels=0), dict(n_channels=65), dict(n_slabs=0),
    dict(align=0), dict(align=8), dict(align=24), dict(n_elems=(1 << 20) + 1), dict(dtype=7),
    dict(phases=0), dict(phases=5), dict(phases=7), dict(phases=9), dict(phases=24), dict(phases=48), dict(phases=64),
    dict(n_slabs=8192, n_elems=8192 * 8 * 4), dict(schedule=4), dict(phases=3 | 64, schedule=3), dict(root=1),
    dict(phases=8, root=8), dict(phases=8, root=-1), dict(phases=16, root=8), dict(phases=32, root=1),
    dict(phases=8, schedule=2), dict(phases=16, schedule=2), dict(phases=32, schedule=2),
    dict(phases=32, n_slabs=1171, n_elems=1171 * 8 * 16),  # all-to-all: R*(R-1)*S > 65535
])
def test_invalid_descriptors(r2, bad):
    base = dict(n_ranks=8, n_slabs=1, n_channels=8, align=256, n_elems=1 << 20, dtype=r2.BF16,
                phases=r2.PHASE_AR)
    base.update(bad)
    d = r2.SimDesc(**base)
    assert r2.r2_sim_num_steps(d) == 0
    assert r2.r2_sim_workspace_bytes(d) == 0
    with pytest.raises(r2.R2Error) as e:
        lists = 2 if base["phases"] in (r2.PHASE_SENDRECV, r2.PHASE_ALLTOALL) else 1
        r2.r2_ring_allreduce_sim(d, [256] * (lists * base["n_ranks"]), [(0, 0, [1] * max(base["n_channels"], 1))],
                                 4096, workspace_bytes=1 << 40)
    assert e.value.code == -1


def test_sendrecv_descriptor_arithmetic(r2):
    """Point-to-point: two steps, one transmission per message chunk, chunks of n_elems / n_slabs."""
    d = r2.SimDesc(8, 6, 8, 256, 6 * 1000, r2.BF16, r2.PHASE_SENDRECV)
    assert r2.r2_sim_num_steps(d) == 2
    assert r2.r2_sim_num_transmissions(d) == 6
    assert r2.r2_sim_stage_capacity(d) == 2048  # 2000 bytes per chunk, rounded up to 256
    assert r2.r2_sim_resolve_schedule(d, [(0, 0, [1] * 8)]) == r2.SCHED_STEPS
    assert r2.r2_sim_num_steps(r2.SimDesc(8, 6, 8, 256, 6 * 1000 + 1, r2.BF16, r2.PHASE_SENDRECV)) == 0
    assert r2.r2_sim_num_steps(r2.SimDesc(8, 6, 8, 256, 6000, r2.BF16, r2.PHASE_SENDRECV, 0, r2.SCHED_FUSED)) == 0


def test_chain_and_alltoall_descriptor_arithmetic(r2):
    """Broadcast and Reduce: R steps, R-1 transmissions per message chunk, one rank at work per step (so
    the stage window counts one rank's chunk).  All-to-all: two steps, (R-1)*S internal slabs."""
    for ph in (r2.PHASE_BROADCAST, r2.PHASE_REDUCE):
        d = r2.SimDesc(8, 6, 8, 256, 6 * 1000, r2.BF16, ph, root=7)
        assert r2.r2_sim_num_steps(d) == 8
        assert r2.r2_sim_num_transmissions(d) == 6 * 7
        assert r2.r2_sim_stage_capacity(d) == 2048
        assert r2.r2_sim_resolve_schedule(d, [(0, 0, [1] * 8)]) == r2.SCHED_STEPS
        assert r2.r2_sim_num_steps(r2.SimDesc(8, 6, 8, 256, 6 * 1000 + 1, r2.BF16, ph)) == 0
        # 4 chunks of 64 MiB each, one rank per step: two chunks fit the 128 MiB window
        assert r2.r2_sim_num_passes(r2.SimDesc(8, 4, 8, 256, 1 << 27, r2.BF16, ph)) == 2
    d = r2.SimDesc(4, 5, 8, 256, 4 * 5 * 100, r2.F32, r2.PHASE_ALLTOALL)
    assert r2.r2_sim_num_steps(d) == 2
    assert r2.r2_sim_num_transmissions(d) == 3 * 5
    assert r2.r2_sim_stage_capacity(d) == 512  # 400 bytes per chunk
    assert r2.r2_sim_workspace_bytes(d) == r2.r2_sim_stage_offset(d) + 2 * 4 * 15 * 8 * 512
    assert r2.r2_sim_num_steps(r2.SimDesc(4, 5, 8, 256, 4 * 5 * 100 + 4, r2.F32, r2.PHASE_ALLTOALL)) == 0


def test_overlapped_schedule_cuts_at_least_two_passes(r2):
    """R2_SCHED_STEPS_OVERLAP halves the stage window and always leaves a pair of passes to overlap."""
    mk = lambda N, S, sched, window=0: r2.SimDesc(8, S, 8, 256, N, r2.BF16, r2.PHASE_AR, window, sched)
    assert r2.r2_sim_num_passes(mk(1 << 26, 1, r2.SCHED_STEPS)) == 1          # cfg2: 128 MiB staged per step
    assert r2.r2_sim_num_passes(mk(1 << 26, 1, r2.SCHED_STEPS_OVERLAP)) == 2  # two byte ranges of 64 MiB
    assert r2.r2_sim_num_passes(mk(1 << 25, 32, r2.SCHED_STEPS)) == 1         # cfg4: 64 MiB staged per step
    assert r2.r2_sim_num_passes(mk(1 << 25, 32, r2.SCHED_STEPS_OVERLAP)) == 2  # two groups of 16 slabs
    assert r2.r2_sim_num_passes(mk(1 << 28, 1, r2.SCHED_STEPS)) == 4
    assert r2.r2_sim_num_passes(mk(1 << 28, 1, r2.SCHED_STEPS_OVERLAP)) == 8
    assert r2.r2_sim_num_passes(mk(8 * 3 * 64, 3, r2.SCHED_STEPS_OVERLAP)) == 3  # three small slabs: one by one
    assert r2.r2_sim_resolve_schedule(mk(1 << 26, 1, r2.SCHED_STEPS_OVERLAP), [(0, 0, [1] * 8)]) == r2.SCHED_STEPS_OVERLAP
    assert r2.r2_sim_resolve_schedule(mk(1 << 26, 1, r2.SCHED_AUTO), [(0, 0, [1] * 8)]) == r2.SCHED_STEPS  # never by itself
    # one slab whose channel state changes on the way: its byte ranges share stage buffers under different
    # tables and may not run side by side -> the plain step schedule; with several slabs the streams split by slab
    changing = [(0, 0, [1] * 8), (3, 0b100100, [1] * 8)]
    assert r2.r2_sim_resolve_schedule(mk(1 << 26, 1, r2.SCHED_STEPS_OVERLAP), changing) == r2.SCHED_STEPS
    assert r2.r2_sim_resolve_schedule(mk(1 << 26, 2, r2.SCHED_STEPS_OVERLAP), changing) == r2.SCHED_STEPS_OVERLAP
    assert r2.r2_sim_resolve_schedule(mk(1 << 26, 1, r2.SCHED_STEPS_OVERLAP), [(0, 0, [1] * 8), (14, 1, [1] * 8)]) == r2.SCHED_STEPS_OVERLAP  # beyond the run


def test_forking_schedules_do_not_nest(r2):
    """The split and the recursive all-reduce fork the caller's stream themselves; the overlapped step
    schedule, which forks too, is refused inside them (host check, no GPU needed)."""
    assert r2.r2_split_workspace_bytes(r2.SplitDesc(4, 1, 2, 16, 7 * 64, 3 * 64, r2.F32, r2.SCHED_STEPS)) > 0
    assert r2.r2_split_workspace_bytes(r2.SplitDesc(4, 1, 2, 16, 7 * 64, 3 * 64, r2.F32, r2.SCHED_STEPS_OVERLAP)) == 0
    lv = [r2.Level(0b1111, 0, 8, 8, 1.0)]
    assert r2.r2_recursive_workspace_bytes(r2.RecursiveDesc(4, 4, 16, 64, r2.F32, 1, 1, r2.SCHED_STEPS), lv, [64]) > 0
    assert r2.r2_recursive_workspace_bytes(r2.RecursiveDesc(4, 4, 16, 64, r2.F32, 1, 1, r2.SCHED_STEPS_OVERLAP), lv, [64]) == 0


def test_static_workspace_call_refuses_the_forking_schedule(r2):
    """The call for callers that may not allocate cannot create the overlapped schedule's side stream and
    events either: refused on the host, before any HIP call; an oversize descriptor likewise."""
    import ctypes

    lib = r2.load_library()
    d = r2.SimDesc(8, 1, 8, 256, 8 * 64, r2.BF16, r2.PHASE_AR, 0, r2.SCHED_STEPS_OVERLAP)
    assert lib.r2_ring_allreduce_sim_static(ctypes.byref(d.c()), None, None, 0, None, None) == -1
    big = r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, r2.PHASE_AR)
    assert r2.r2_sim_workspace_bytes(big) > r2.STATIC_WORKSPACE_BYTES
    assert lib.r2_ring_allreduce_sim_static(ctypes.byref(big.c()), None, None, 0, None, None) == -4


def test_rails_schedule_is_host_arithmetic(r2):
    """r2_rails_resolve_schedule: fused columns for launch-bound sizes whose ring chunks are whole
    16-byte vectors and whose links' rows fit LDS, else one launch per step; the errors r2_ring_rails_sim
    would return before launching."""
    links = r2.PHASE_AR | r2.PHASE_LINKS
    w = [50000] * 8
    rails = r2.static_rails(w, [1, 2, 0, 0, 4, 0, 0, 8])
    small = r2.SimDesc(8, 1, 8, 256, 8192, r2.BF16, links)
    assert r2.r2_rails_resolve_schedule(small, rails) == r2.SCHED_FUSED
    big = r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, links)  # 128 MiB per rank
    assert r2.r2_rails_resolve_schedule(big, rails) == r2.SCHED_STEPS
    assert r2.r2_rails_resolve_schedule(r2.SimDesc(8, 1, 8, 256, 1 << 26, r2.BF16, links, 0, r2.SCHED_FUSED), rails) == r2.SCHED_FUSED
    assert r2.r2_rails_resolve_schedule(r2.SimDesc(8, 1, 8, 256, 8192, r2.BF16, links, 0, r2.SCHED_STEPS), rails) == r2.SCHED_STEPS
    ragged = r2.SimDesc(8, 1, 8, 256, 8 * 7, r2.BF16, links)  # 14-byte ring chunks
    assert r2.r2_rails_resolve_schedule(ragged, rails) == r2.SCHED_STEPS
    with pytest.raises(r2.R2Error) as e:
        r2.r2_rails_resolve_schedule(r2.SimDesc(8, 1, 8, 256, 8 * 7, r2.BF16, links, 0, r2.SCHED_FUSED), rails)
    assert e.value.code == -1
    # 32 ranks x 62 transmissions x (9 * 8 + 24) bytes = 190 KiB of rows: more than a workgroup's LDS
    many = r2.static_rails(w, [0] * 32)
    assert r2.r2_rails_resolve_schedule(r2.SimDesc(32, 1, 8, 256, 32 * 64, r2.BF16, links), many) == r2.SCHED_STEPS
    with pytest.raises(r2.R2Error):
        r2.r2_rails_resolve_schedule(r2.SimDesc(32, 1, 8, 256, 32 * 64, r2.BF16, links, 0, r2.SCHED_FUSED), many)
    # ... unless the links' tables change so often that every launch is short: cuts before steps 1..61
    flapping = [[(t, t & 1, w) for t in range(62)]] + r2.static_rails(w, [0] * 31)
    assert r2.r2_rails_resolve_schedule(r2.SimDesc(32, 1, 8, 256, 32 * 64, r2.BF16, links, 0, r2.SCHED_FUSED),
                                        flapping) == r2.SCHED_FUSED
    assert r2.r2_rails_resolve_schedule(r2.SimDesc(32, 1, 8, 256, 32 * 64, r2.BF16, links), flapping) == r2.SCHED_STEPS  # saves no launch
    # neighbours that share no rail
    with pytest.raises(r2.R2Error) as e:
        r2.r2_rails_resolve_schedule(small, r2.static_rails(w, [0x0f, 0xf0, 0, 0, 0, 0, 0, 0]))
    assert e.value.code == -2
    with pytest.raises(r2.R2Error):  # the flag is missing
        r2.r2_rails_resolve_schedule(r2.SimDesc(8, 1, 8, 256, 8192, r2.BF16, r2.PHASE_AR), rails)
    with pytest.raises(r2.R2Error):  # one epoch list says nothing about per-link tables
        r2.r2_sim_resolve_schedule(small, [(0, 0, w)])


def test_binding_checks_list_lengths(r2):
    """The C side reads as many pointers and weights as the descriptor says: the binding refuses shorter lists."""
    d = r2.SimDesc(4, 1, 4, 256, 4096, r2.F32, r2.PHASE_ALLTOALL)
    with pytest.raises(ValueError):
        r2.r2_collective_sim(d, [256] * 4, [(0, 0, [1] * 4)], 4096, workspace_bytes=1 << 40)  # needs 2R pointers
    with pytest.raises(ValueError):
        r2.r2_ring_allreduce_sim(r2.SimDesc(4, 1, 4, 256, 4096, r2.F32, r2.PHASE_AR), [256] * 4, [(0, 0, [1] * 3)],
                                 4096, workspace_bytes=1 << 40)  # three weights for four channels


def test_sim_rejects_bad_epochs_and_buffers_before_any_device_work(r2):
    d = r2.SimDesc(4, 1, 4, 256, 4096, r2.F32, r2.PHASE_AR)
    need = r2.r2_sim_workspace_bytes(d)
    bufs = [4096 * (i + 1) for i in range(4)]  # fake but aligned addresses: never dereferenced
    ok_ep = [(0, 0, [1, 1, 1, 1])]
    cases = [
        ([], -1),                                               # no epoch
        ([(1, 0, [1, 1, 1, 1])], -1),                           # first epoch must start at 0
        ([(0, 0, [1] * 4), (5, 0, [1] * 4), (5, 0, [1] * 4)], -1),  # not strictly increasing
        ([(0, 0b1111, [1, 1, 1, 1])], -2),                      # all failed
        ([(0, 0, [0, 0, 0, 0])], -2),                           # all zero bandwidth
        ([(0, 0, [1] * 4), (3, 0b1111, [1] * 4)], -2),          # fails later, still before any launch
    ]
    for eps, code in cases:
        with pytest.raises(r2.R2Error) as e:
            r2.r2_ring_allreduce_sim(d, bufs, eps, 4096, workspace_bytes=need)
        assert e.value.code == code, eps
    # an epoch that starts after the last transmission is never in force
    # (checked through the workspace error that comes next)
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim(d, bufs, [(0, 0, [1] * 4), (6, 0b1111, [1] * 4)], 4096, workspace_bytes=need - 1)
    assert e.value.code == -4
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim(d, bufs, ok_ep, 4096 + 16, workspace_bytes=need)  # workspace not 256-aligned
    assert e.value.code == -1
    with pytest.raises(r2.R2Error) as e:
        r2.r2_ring_allreduce_sim(d, [4096, 8192, 12288 + 4, 16384], ok_ep, 4096, workspace_bytes=need)
    assert e.value.code == -1
    with pytest.raises(r2.R2Error) as e:
        r2.r2_sim_step(d, bufs, 0, 7, 4096, workspace_bytes=need)  # J = 7: steps are 0..6
    assert e.value.code == -1
    with pytest.raises(r2.R2Error) as e:
        r2.r2_sim_step(d, bufs, 1, 0, 4096, workspace_bytes=need)  # a single pass
    assert e.value.code == -1


def test_reduce_copy_and_partition_argument_checks(r2):
    with pytest.raises(r2.R2Error) as e:
        r2.r2_reduce_copy(4096, r2.F32, r2.OP_SUM, None, None, None, None, 4, 1024, nbytes=64)
    assert e.value.code == -1  # neither incoming nor outgoing
    with pytest.raises(r2.R2Error) as e:
        r2.r2_reduce_copy(4096, r2.F32, r2.OP_SUM, [256] * 4, 512, None, None, 4, 1024, nbytes=66)
    assert e.value.code == -1  # not a whole number of fp32 elements
    with pytest.raises(r2.R2Error) as e:
        r2.r2_reduce_copy(4096, r2.F32, r2.OP_SUM, [256, 256, 264, 256], 512, None, None, 4, 1024, nbytes=64)
    assert e.value.code == -1  # stage buffer not 16-byte aligned
    with pytest.raises(r2.R2Error) as e:
        r2.r2_reduce_copy(4096, r2.F32, 5, [256] * 4, 512, None, None, 4, 1024, nbytes=64)
    assert e.value.code == -1
    with pytest.raises(r2.R2Error) as e:
        r2.r2_partition([1, 2, 3], 0b111, 4096, 256)
    assert e.value.code == -2  # decided on the host, offsets zeroed
    with pytest.raises(r2.R2Error) as e:
        r2.r2_partition([1, 2, 3], 0, 4096, 0)
    assert e.value.code == -1


def test_product_package_does_not_import_the_oracle():
    """The product path must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2512_25059_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".hpp", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in ("r2_oracle.c", "r2_oracle.py", "__init__.py"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2512_25059_amd" not in text and "r2ccl" not in text, f
