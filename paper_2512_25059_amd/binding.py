"""ctypes binding of ``libr2ccl.so`` (see ``include/r2ccl.h`` and ``include/r2ccl_ext.h`` for the contract).

Argument marshalling only.  torch is used for device memory and streams; a
torch tensor stands for "device pointer + size".  Each wrapper has the name of
the C entry point it calls and raises :class:`R2Error` on a non-zero code.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch  # imported before the library so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libr2ccl.so")

F32, BF16 = 0, 1
OP_SUM, OP_COPY, OP_SUM_FORWARD, OP_SUM_SEND = 0, 1, 2, 3
PHASE_RS, PHASE_AG = 1, 2
PHASE_AR = PHASE_RS | PHASE_AG
PHASE_SENDRECV, PHASE_BROADCAST, PHASE_REDUCE, PHASE_ALLTOALL, PHASE_LINKS = 4, 8, 16, 32, 64
SCHED_AUTO, SCHED_STEPS, SCHED_FUSED, SCHED_STEPS_OVERLAP = 0, 1, 2, 3

R2_OK = 0
R2_ERR_INVALID = -1
R2_ERR_NO_HEALTHY_CHANNEL = -2
R2_ERR_OVERFLOW = -3
R2_ERR_CAPACITY = -4
R2_ERR_DEVICE = -5


class R2Error(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {r2_strerror(code)} ({code})")
        self.code = code


class _Epoch(C.Structure):
    _fields_ = [("t_start", C.c_uint64), ("fail_mask", C.c_uint64), ("weights", C.POINTER(C.c_uint32))]


class _SplitDesc(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("degraded_rank", C.c_uint32), ("n_channels", C.c_uint32),
                ("align", C.c_uint32), ("n_elems", C.c_uint64), ("n_partial", C.c_uint64),
                ("dtype", C.c_int32), ("schedule", C.c_int32), ("n_slabs_global", C.c_uint32),
                ("n_slabs_partial", C.c_uint32)]


class _Level(C.Structure):
    _fields_ = [("members", C.c_uint64), ("fail_mask", C.c_uint64), ("bandwidth", C.c_uint64),
                ("increment", C.c_uint64), ("share", C.c_double)]


class _RecursiveDesc(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("n_channels", C.c_uint32), ("align", C.c_uint32),
                ("dtype", C.c_int32), ("schedule", C.c_int32), ("n_slabs", C.c_uint32),
                ("n_levels", C.c_uint32), ("reserved", C.c_uint32), ("n_elems", C.c_uint64)]


class _SimDesc(C.Structure):
    _fields_ = [("n_ranks", C.c_uint32), ("n_slabs", C.c_uint32), ("n_channels", C.c_uint32),
                ("align", C.c_uint32), ("n_elems", C.c_uint64), ("dtype", C.c_int32),
                ("phases", C.c_int32), ("stage_window_bytes", C.c_uint64), ("schedule", C.c_int32),
                ("root", C.c_int32)]


@dataclass(frozen=True)
class SimDesc:
    n_ranks: int
    n_slabs: int
    n_channels: int
    align: int
    n_elems: int
    dtype: int
    phases: int
    stage_window_bytes: int = 0  # 0 = library default
    schedule: int = 0            # SCHED_AUTO
    root: int = 0                # PHASE_BROADCAST / PHASE_REDUCE

    def c(self) -> _SimDesc:
        return _SimDesc(self.n_ranks, self.n_slabs, self.n_channels, self.align, self.n_elems,
                        self.dtype, self.phases, self.stage_window_bytes, self.schedule, self.root)


@dataclass(frozen=True)
class SplitDesc:
    n_ranks: int
    degraded_rank: int
    n_channels: int
    align: int
    n_elems: int
    n_partial: int
    dtype: int
    schedule: int = 0
    n_slabs_global: int = 1
    n_slabs_partial: int = 1

    def c(self) -> _SplitDesc:
        return _SplitDesc(self.n_ranks, self.degraded_rank, self.n_channels, self.align, self.n_elems,
                          self.n_partial, self.dtype, self.schedule, self.n_slabs_global,
                          self.n_slabs_partial)


MAX_LEVELS = 16


@dataclass(frozen=True)
class Level:
    """One ring of the recursive decomposition (mirror of r2_level)."""
    members: int
    fail_mask: int
    bandwidth: int = 0
    increment: int = 0
    share: float = 0.0

    def ranks(self) -> List[int]:
        return [r for r in range(64) if (self.members >> r) & 1]


@dataclass(frozen=True)
class RecursiveDesc:
    n_ranks: int
    n_channels: int
    align: int
    n_elems: int
    dtype: int
    n_levels: int
    n_slabs: int = 1
    schedule: int = 0

    def c(self) -> _RecursiveDesc:
        return _RecursiveDesc(self.n_ranks, self.n_channels, self.align, self.dtype, self.schedule,
                              self.n_slabs, self.n_levels, 0, self.n_elems)


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library.  It is never built here: run ``__graft_entry__.build()`` (or
    ``python -m paper_2512_25059_amd.build``) first."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2512_25059_amd.build`; "
                           "there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
    lib.r2_strerror.restype = C.c_char_p
    lib.r2_strerror.argtypes = [i32]
    lib.r2_partition.restype = i32
    lib.r2_partition.argtypes = [vp, u64, u32, u64, u32, vp]
    lib.r2_partition_device.restype = i32
    lib.r2_partition_device.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp, vp]
    lib.r2_rollback_plan_device.restype = i32
    lib.r2_rollback_plan_device.argtypes = [vp, vp, vp, vp, u32, u32, u32, vp, vp, vp]
    lib.r2_split_plan.restype = i32
    lib.r2_split_plan.argtypes = [u32, u32, C.c_double, vp, vp, vp]
    lib.r2_split_time.restype = C.c_double
    lib.r2_split_partial_elems.restype = u64
    lib.r2_split_partial_elems.argtypes = [u32, u32, u32, i32, u64, C.c_double]
    lib.r2_split_time.argtypes = [u32, u32, C.c_double, C.c_double]
    lib.r2_split_workspace_bytes.restype = u64
    lib.r2_split_workspace_bytes.argtypes = [C.POINTER(_SplitDesc)]
    lib.r2_split_allreduce_sim.restype = i32
    lib.r2_split_allreduce_sim.argtypes = [C.POINTER(_SplitDesc), vp, vp, u64, vp, u64, vp]
    lib.r2_recursive_plan.restype = i32
    lib.r2_recursive_plan.argtypes = [u32, u32, u32, vp, vp, u32, vp, vp]
    lib.r2_recursive_ring_order.restype = i32
    lib.r2_recursive_ring_order.argtypes = [u32, u32, vp, u64, vp]
    lib.r2_recursive_time.restype = C.c_double
    lib.r2_recursive_time.argtypes = [u32, u32, vp, u32, C.c_double, C.c_double, C.c_double]
    lib.r2_select_strategy.restype = i32
    lib.r2_select_strategy.argtypes = [u32, u32, u32, vp, vp, C.c_double, C.c_double, C.c_double, vp, vp, vp]
    lib.r2_recursive_segments.restype = i32
    lib.r2_recursive_segments.argtypes = [C.POINTER(_RecursiveDesc), vp, vp]
    lib.r2_recursive_workspace_bytes.restype = u64
    lib.r2_recursive_workspace_bytes.argtypes = [C.POINTER(_RecursiveDesc), vp, vp]
    lib.r2_recursive_allreduce_sim.restype = i32
    lib.r2_recursive_allreduce_sim.argtypes = [C.POINTER(_RecursiveDesc), vp, vp, vp, vp, vp, vp, u64, vp]
    lib.r2_bridge_rerank.restype = i32
    lib.r2_bridge_rerank.argtypes = [vp, vp, u32, vp, vp]
    lib.r2_reduce_copy.restype = i32
    lib.r2_reduce_copy.argtypes = [vp, u64, i32, i32, vp, vp, vp, vp, u32, u64, vp, vp]
    pd = C.POINTER(_SimDesc)
    lib.r2_sim_num_steps.restype = u32
    lib.r2_sim_num_steps.argtypes = [pd]
    for name in ("r2_sim_num_transmissions", "r2_sim_workspace_bytes", "r2_sim_stage_offset",
                 "r2_sim_stage_capacity", "r2_sim_num_passes"):
        getattr(lib, name).restype = u64
        getattr(lib, name).argtypes = [pd]
    lib.r2_sim_prepare.restype = i32
    lib.r2_sim_prepare.argtypes = [pd, vp, u32, vp, u64, vp, vp]
    lib.r2_sim_step.restype = i32
    lib.r2_sim_step.argtypes = [pd, vp, u64, u32, vp, u64, vp]
    lib.r2_sim_resolve_schedule.restype = i32
    lib.r2_sim_resolve_schedule.argtypes = [pd, vp, u32]
    lib.r2_sim_fused_steps.restype = i32
    lib.r2_sim_fused_steps.argtypes = [pd, vp, u32, u32, vp, u64, vp]
    lib.r2_ring_allreduce_sim.restype = i32
    lib.r2_ring_allreduce_sim.argtypes = [pd, vp, vp, u32, vp, u64, vp, vp]
    lib.r2_ring_allreduce_sim_static.restype = i32
    lib.r2_ring_allreduce_sim_static.argtypes = [pd, vp, vp, u32, vp, vp]
    lib.r2_ring_allreduce_sim_inflight.restype = i32
    lib.r2_ring_allreduce_sim_inflight.argtypes = [pd, vp, vp, vp, u32, vp, u64, vp, vp, vp]
    lib.r2_sendrecv_sim.restype = i32
    lib.r2_sendrecv_sim.argtypes = [pd, vp, vp, vp, u32, vp, u64, vp, vp]
    lib.r2_collective_sim.restype = i32
    lib.r2_collective_sim.argtypes = [pd, vp, vp, u32, vp, u64, vp, vp]
    lib.r2_ring_rails_sim.restype = i32
    lib.r2_ring_rails_sim.argtypes = [pd, vp, vp, vp, vp, u64, vp, vp]
    lib.r2_rails_resolve_schedule.restype = i32
    lib.r2_rails_resolve_schedule.argtypes = [pd, vp, vp]
    lib.r2_alltoall_sim.restype = i32
    lib.r2_alltoall_sim.argtypes = [pd, vp, vp, vp, u32, vp, u64, vp, vp]
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != R2_OK:
        raise R2Error(rc, what)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if isinstance(t, torch.Tensor) else int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr_array(ts: Optional[Sequence]) -> Tuple[Optional[C.Array], Optional[int]]:
    if ts is None:
        return None, None
    arr = (C.c_void_p * len(ts))(*[_ptr(t) for t in ts])
    return arr, C.cast(arr, C.c_void_p).value


def _check_lists(desc: "SimDesc", rank_bufs: Sequence, epochs) -> None:
    """The C side reads n_ranks pointers (2 * n_ranks for the two-list phases) and n_channels weights per
    epoch: make sure they are there."""
    if not (2 <= desc.n_ranks <= 64 and 1 <= desc.n_channels <= 64):
        return  # the library rejects the descriptor before it reads any list
    want = desc.n_ranks * (2 if desc.phases in (PHASE_SENDRECV, PHASE_ALLTOALL) else 1)
    if len(rank_bufs) != want:
        raise ValueError(f"expected {want} rank buffers, got {len(rank_bufs)}")
    if any(len(w) != desc.n_channels for _, _, w in epochs):
        raise ValueError("every epoch needs one weight per channel")


def _epoch_array(epochs: Sequence[Tuple[int, int, Sequence[int]]]):
    keep = []
    arr = (_Epoch * max(len(epochs), 1))()
    for i, (t0, mask, w) in enumerate(epochs):
        wa = (C.c_uint32 * len(w))(*[int(x) for x in w])
        keep.append(wa)
        arr[i].t_start = int(t0)
        arr[i].fail_mask = int(mask)
        arr[i].weights = C.cast(wa, C.POINTER(C.c_uint32))
    return arr, keep


def r2_strerror(code: int) -> str:
    return load_library().r2_strerror(int(code)).decode()


def r2_partition(weights: Sequence[int], fail_mask: int, nbytes: int, align: int) -> List[int]:
    """Host-pointer convenience call: returns the C+1 offsets."""
    n = len(weights)
    w = (C.c_uint32 * max(n, 1))(*[int(x) for x in weights])
    off = (C.c_uint64 * (n + 1))()
    rc = load_library().r2_partition(C.cast(w, C.c_void_p), int(fail_mask), n, int(nbytes), int(align),
                                     C.cast(off, C.c_void_p))
    _check(rc, "r2_partition")
    return list(off)


def r2_partition_device(weights: torch.Tensor, fail_mask: torch.Tensor, nbytes: torch.Tensor,
                        align: int, offsets: torch.Tensor, status: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    """weights [T, C] (4-byte ints), fail_mask [T], nbytes [T], offsets [T, C+1] (8-byte ints),
    status [T] int32 or None; all on the device."""
    T, n_channels = weights.shape
    assert weights.element_size() == 4 and weights.is_contiguous()
    assert fail_mask.element_size() == 8 and nbytes.element_size() == 8 and offsets.element_size() == 8
    assert fail_mask.numel() == T and nbytes.numel() == T and offsets.numel() == T * (n_channels + 1)
    assert status is None or (status.element_size() == 4 and status.numel() == T)
    rc = load_library().r2_partition_device(_ptr(weights), _ptr(fail_mask), _ptr(nbytes), n_channels,
                                            int(align), T, _ptr(offsets), _ptr(status), _stream(stream))
    _check(rc, "r2_partition_device")


def r2_split_plan(n_servers: int, gpus_per_server: int, lost_fraction: float) -> Tuple[bool, float, float]:
    """Returns (use the split schedule?, Y*, threshold on the lost fraction)."""
    use, y, thr = C.c_int32(0), C.c_double(0.0), C.c_double(0.0)
    rc = load_library().r2_split_plan(int(n_servers), int(gpus_per_server), float(lost_fraction),
                                      C.cast(C.pointer(use), C.c_void_p), C.cast(C.pointer(y), C.c_void_p),
                                      C.cast(C.pointer(thr), C.c_void_p))
    _check(rc, "r2_split_plan")
    return bool(use.value), float(y.value), float(thr.value)


def r2_split_time(n_servers: int, gpus_per_server: int, lost_fraction: float, y: float) -> float:
    return float(load_library().r2_split_time(int(n_servers), int(gpus_per_server), float(lost_fraction), float(y)))


def r2_split_partial_elems(n_ranks: int, n_slabs_global: int, n_slabs_partial: int, dtype: int, n_elems: int,
                           y: float) -> int:
    """Host call: the size of the tail for share y, rounded to what both rings divide into."""
    return int(load_library().r2_split_partial_elems(int(n_ranks), int(n_slabs_global), int(n_slabs_partial),
                                                     int(dtype), int(n_elems), float(y)))


def r2_split_workspace_bytes(desc: SplitDesc) -> int:
    return int(load_library().r2_split_workspace_bytes(C.byref(desc.c())))


def r2_split_allreduce_sim(desc: SplitDesc, rank_bufs: Sequence, weights: Sequence[int], degraded_fail_mask: int,
                           workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    if 2 <= desc.n_ranks <= 64 and 1 <= desc.n_channels <= 64:  # else the library rejects it before reading
        if len(rank_bufs) != desc.n_ranks or len(weights) != desc.n_channels:
            raise ValueError("r2_split_allreduce_sim: one buffer per rank, one weight per channel")
    arr, p = _ptr_array(rank_bufs)
    w = (C.c_uint32 * max(len(weights), 1))(*[int(x) for x in weights])
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_split_allreduce_sim(C.byref(desc.c()), p, C.cast(w, C.c_void_p),
                                               int(degraded_fail_mask), wp, wb, _stream(stream))
    del arr
    _check(rc, "r2_split_allreduce_sim")


def _u32s(xs: Sequence[int]):
    return (C.c_uint32 * max(len(xs), 1))(*[int(x) for x in xs])


def _u64s(xs: Sequence[int]):
    return (C.c_uint64 * max(len(xs), 1))(*[int(x) for x in xs])


def _levels(levels: Sequence[Level]):
    arr = (_Level * max(len(levels), 1))()
    for i, lv in enumerate(levels):
        arr[i] = _Level(int(lv.members), int(lv.fail_mask), int(lv.bandwidth), int(lv.increment), float(lv.share))
    return arr


def r2_recursive_plan(weights: Sequence[int], fail_masks: Sequence[int], gpus_per_rank: int = 1,
                      max_levels: int = MAX_LEVELS) -> List[Level]:
    """Host call: the peel plan for per-rank failed-channel masks."""
    w, m = _u32s(weights), _u64s(fail_masks)
    out = (_Level * MAX_LEVELS)()
    n = C.c_uint32(0)
    rc = load_library().r2_recursive_plan(len(fail_masks), int(gpus_per_rank), len(weights), C.cast(w, C.c_void_p),
                                          C.cast(m, C.c_void_p), int(max_levels), C.cast(out, C.c_void_p),
                                          C.cast(C.pointer(n), C.c_void_p))
    _check(rc, "r2_recursive_plan")
    return [Level(int(l.members), int(l.fail_mask), int(l.bandwidth), int(l.increment), float(l.share))
            for l in out[:n.value]]


def r2_recursive_ring_order(n_channels: int, fail_masks: Sequence[int], members: int) -> List[int]:
    """Host call: the order in which the ring over `members` (a bit mask of ranks) visits them."""
    m = _u64s(fail_masks)
    n = bin(int(members)).count("1")
    out = (C.c_uint32 * max(n, 1))()
    rc = load_library().r2_recursive_ring_order(len(fail_masks), int(n_channels), C.cast(m, C.c_void_p), int(members),
                                                C.cast(out, C.c_void_p))
    _check(rc, "r2_recursive_ring_order")
    return list(out)[:n]


def r2_recursive_time(n_ranks: int, gpus_per_rank: int, levels: Sequence[Level], nbytes: float, alpha: float,
                      beta: float) -> float:
    arr = _levels(levels)
    return float(load_library().r2_recursive_time(int(n_ranks), int(gpus_per_rank), C.cast(arr, C.c_void_p),
                                                  len(levels), float(nbytes), float(alpha), float(beta)))


def r2_select_strategy(weights: Sequence[int], fail_masks: Sequence[int], gpus_per_rank: int, nbytes: float,
                       alpha: float, beta: float) -> Tuple[int, List[float]]:
    """Host call: returns (chosen depth, modelled time of every depth)."""
    w, m = _u32s(weights), _u64s(fail_masks)
    depth, nd = C.c_uint32(0), C.c_uint32(0)
    times = (C.c_double * MAX_LEVELS)()
    rc = load_library().r2_select_strategy(len(fail_masks), int(gpus_per_rank), len(weights), C.cast(w, C.c_void_p),
                                           C.cast(m, C.c_void_p), float(nbytes), float(alpha), float(beta),
                                           C.cast(C.pointer(depth), C.c_void_p), C.cast(times, C.c_void_p),
                                           C.cast(C.pointer(nd), C.c_void_p))
    _check(rc, "r2_select_strategy")
    return int(depth.value), [float(t) for t in times[:nd.value]]


def r2_recursive_segments(desc: RecursiveDesc, levels: Sequence[Level]) -> List[int]:
    """Host call: segment sizes (elements per level) that follow the plan's shares."""
    if len(levels) != desc.n_levels:
        raise ValueError("r2_recursive_segments: one level per desc.n_levels")
    arr = _levels(levels)
    out = (C.c_uint64 * max(len(levels), 1))()
    rc = load_library().r2_recursive_segments(C.byref(desc.c()), C.cast(arr, C.c_void_p), C.cast(out, C.c_void_p))
    _check(rc, "r2_recursive_segments")
    return [int(x) for x in out[:len(levels)]]


def r2_recursive_workspace_bytes(desc: RecursiveDesc, levels: Sequence[Level], level_elems: Sequence[int]) -> int:
    arr, e = _levels(levels), _u64s(level_elems)
    return int(load_library().r2_recursive_workspace_bytes(C.byref(desc.c()), C.cast(arr, C.c_void_p),
                                                           C.cast(e, C.c_void_p)))


def r2_recursive_allreduce_sim(desc: RecursiveDesc, rank_bufs: Sequence, weights: Sequence[int],
                               fail_masks: Sequence[int], levels: Sequence[Level], level_elems: Sequence[int],
                               workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    if 2 <= desc.n_ranks <= 64 and 1 <= desc.n_channels <= 64 and 1 <= desc.n_levels <= MAX_LEVELS:
        if (len(rank_bufs) != desc.n_ranks or len(fail_masks) != desc.n_ranks or len(weights) != desc.n_channels
                or len(levels) != desc.n_levels or len(level_elems) != desc.n_levels):
            raise ValueError("r2_recursive_allreduce_sim: list lengths do not match the descriptor")
    keep, p = _ptr_array(rank_bufs)
    w, m, arr, e = _u32s(weights), _u64s(fail_masks), _levels(levels), _u64s(level_elems)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_recursive_allreduce_sim(C.byref(desc.c()), p, C.cast(w, C.c_void_p), C.cast(m, C.c_void_p),
                                                   C.cast(arr, C.c_void_p), C.cast(e, C.c_void_p), wp, wb,
                                                   _stream(stream))
    del keep
    _check(rc, "r2_recursive_allreduce_sim")


def r2_bridge_rerank(ring: Sequence[int], rails: Sequence[int]) -> Tuple[List[int], int]:
    """Host call: ring is a permutation of 0..n-1, rails[node] a bit mask.  Returns (new ring, relocations)."""
    n = len(ring)
    r = (C.c_uint32 * max(n, 1))(*[int(x) for x in ring])
    m = (C.c_uint64 * max(n, 1))(*[int(x) for x in rails])
    out = (C.c_uint32 * max(n, 1))()
    moved = C.c_uint32(0)
    rc = load_library().r2_bridge_rerank(C.cast(r, C.c_void_p), C.cast(m, C.c_void_p), n,
                                         C.cast(out, C.c_void_p), C.cast(C.pointer(moved), C.c_void_p))
    _check(rc, "r2_bridge_rerank")
    return list(out)[:n], int(moved.value)


def r2_rollback_plan_device(offsets: torch.Tensor, weights: torch.Tensor, mask_before: torch.Tensor,
                            mask_after: torch.Tensor, align: int, plan: torch.Tensor,
                            status: Optional[torch.Tensor] = None, stream=None) -> None:
    """offsets [T, C+1], weights [T, C], masks [T], plan [T, C, C+1] (8-byte ints except the 4-byte
    weights), status [T] int32 or None; all on the device."""
    T, n_channels = weights.shape
    assert weights.element_size() == 4 and weights.is_contiguous()
    assert offsets.numel() == T * (n_channels + 1) and plan.numel() == T * n_channels * (n_channels + 1)
    assert mask_before.numel() == T and mask_after.numel() == T
    rc = load_library().r2_rollback_plan_device(_ptr(offsets), _ptr(weights), _ptr(mask_before),
                                                _ptr(mask_after), n_channels, int(align), T, _ptr(plan),
                                                _ptr(status), _stream(stream))
    _check(rc, "r2_rollback_plan_device")


def r2_reduce_copy(local: torch.Tensor, dtype: int, op: int,
                   in_stage: Optional[Sequence[torch.Tensor]], in_offsets: Optional[torch.Tensor],
                   out_stage: Optional[Sequence[torch.Tensor]], out_offsets: Optional[torch.Tensor],
                   n_channels: int, stage_capacity: int, status: Optional[torch.Tensor] = None,
                   stream=None, nbytes: Optional[int] = None) -> None:
    if nbytes is None:
        nbytes = local.numel() * local.element_size()
    if 1 <= n_channels <= 64:  # else the library rejects the call before it reads the lists
        for what, stage, table in (("in", in_stage, in_offsets), ("out", out_stage, out_offsets)):
            if stage is not None and len(stage) != n_channels:
                raise ValueError(f"r2_reduce_copy: {what}_stage needs one buffer per channel")
            if hasattr(table, "numel") and table.numel() < n_channels + 1:
                raise ValueError(f"r2_reduce_copy: {what}_offsets needs n_channels + 1 entries")
    in_arr, in_p = _ptr_array(in_stage)
    out_arr, out_p = _ptr_array(out_stage)
    rc = load_library().r2_reduce_copy(_ptr(local), int(nbytes), int(dtype), int(op), in_p,
                                       _ptr(in_offsets), out_p, _ptr(out_offsets), int(n_channels),
                                       int(stage_capacity), _ptr(status), _stream(stream))
    del in_arr, out_arr
    _check(rc, "r2_reduce_copy")


def r2_sim_num_steps(desc: SimDesc) -> int:
    return int(load_library().r2_sim_num_steps(C.byref(desc.c())))


def r2_sim_num_transmissions(desc: SimDesc) -> int:
    return int(load_library().r2_sim_num_transmissions(C.byref(desc.c())))


def r2_sim_num_passes(desc: SimDesc) -> int:
    return int(load_library().r2_sim_num_passes(C.byref(desc.c())))


def r2_sim_workspace_bytes(desc: SimDesc) -> int:
    return int(load_library().r2_sim_workspace_bytes(C.byref(desc.c())))


def r2_sim_stage_offset(desc: SimDesc) -> int:
    return int(load_library().r2_sim_stage_offset(C.byref(desc.c())))


def r2_sim_stage_capacity(desc: SimDesc) -> int:
    return int(load_library().r2_sim_stage_capacity(C.byref(desc.c())))


def _ws(workspace, workspace_bytes):
    if isinstance(workspace, torch.Tensor):
        return workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return (int(workspace) if workspace is not None else None), int(workspace_bytes or 0)


def r2_sim_prepare(desc: SimDesc, epochs, workspace, offsets_log: Optional[torch.Tensor] = None,
                   stream=None, workspace_bytes: Optional[int] = None) -> None:
    ep, keep = _epoch_array(epochs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_sim_prepare(C.byref(desc.c()), C.cast(ep, C.c_void_p), len(epochs), wp, wb,
                                       _ptr(offsets_log), _stream(stream))
    del keep
    _check(rc, "r2_sim_prepare")


def r2_sim_step(desc: SimDesc, rank_bufs: Sequence, pass_index: int, step: int, workspace, stream=None,
                workspace_bytes: Optional[int] = None) -> None:
    arr, p = _ptr_array(rank_bufs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_sim_step(C.byref(desc.c()), p, int(pass_index), int(step), wp, wb, _stream(stream))
    del arr
    _check(rc, "r2_sim_step")


def r2_sim_resolve_schedule(desc: SimDesc, epochs) -> int:
    ep, keep = _epoch_array(epochs)
    rc = load_library().r2_sim_resolve_schedule(C.byref(desc.c()), C.cast(ep, C.c_void_p), len(epochs))
    del keep
    if rc < 0:
        raise R2Error(rc, "r2_sim_resolve_schedule")
    return rc


class ReduceCopyCall:
    """The arguments of r2_reduce_copy marshalled once; ``run()`` is a single foreign call."""

    def __init__(self, local: torch.Tensor, dtype: int, op: int, in_stage, in_offsets, out_stage, out_offsets,
                 n_channels: int, stage_capacity: int, status: Optional[torch.Tensor] = None, stream=None,
                 nbytes: Optional[int] = None):
        self._fn = load_library().r2_reduce_copy
        if nbytes is None:
            nbytes = local.numel() * local.element_size()
        self._in, in_p = _ptr_array(in_stage)
        self._out, out_p = _ptr_array(out_stage)
        self._refs = (local, in_stage, in_offsets, out_stage, out_offsets, status)
        self._args = (_ptr(local), int(nbytes), int(dtype), int(op), in_p, _ptr(in_offsets), out_p,
                      _ptr(out_offsets), int(n_channels), int(stage_capacity), _ptr(status), _stream(stream))

    def run(self) -> None:
        rc = self._fn(*self._args)
        if rc != R2_OK:
            raise R2Error(rc, "r2_reduce_copy")


class SimCall:
    """The arguments of r2_ring_allreduce_sim marshalled once, for callers that issue the same
    collective many times (a serving loop): ``run()`` is then a single foreign call."""

    def __init__(self, desc: SimDesc, rank_bufs: Sequence, epochs, workspace,
                 offsets_log: Optional[torch.Tensor] = None, stream=None,
                 workspace_bytes: Optional[int] = None):
        _check_lists(desc, rank_bufs, epochs)
        self._fn = load_library().r2_ring_allreduce_sim
        self._desc = desc.c()
        self._bufs, bufs_p = _ptr_array(rank_bufs)
        self._epochs, self._keep = _epoch_array(epochs)
        wp, wb = _ws(workspace, workspace_bytes)
        self._refs = (rank_bufs, workspace, offsets_log)  # keep the device memory alive
        self._args = (C.byref(self._desc), bufs_p, C.cast(self._epochs, C.c_void_p), len(epochs), wp, wb,
                      _ptr(offsets_log), _stream(stream))

    def run(self) -> None:
        rc = self._fn(*self._args)
        if rc != R2_OK:
            raise R2Error(rc, "r2_ring_allreduce_sim")


def r2_sim_fused_steps(desc: SimDesc, rank_bufs: Sequence, step_begin: int, step_end: int, workspace,
                       stream=None, workspace_bytes: Optional[int] = None) -> None:
    arr, p = _ptr_array(rank_bufs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_sim_fused_steps(C.byref(desc.c()), p, int(step_begin), int(step_end), wp, wb,
                                           _stream(stream))
    del arr
    _check(rc, "r2_sim_fused_steps")


def r2_ring_allreduce_sim(desc: SimDesc, rank_bufs: Sequence, epochs, workspace,
                          offsets_log: Optional[torch.Tensor] = None, stream=None,
                          workspace_bytes: Optional[int] = None) -> None:
    _check_lists(desc, rank_bufs, epochs)
    arr, p = _ptr_array(rank_bufs)
    ep, keep = _epoch_array(epochs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_ring_allreduce_sim(C.byref(desc.c()), p, C.cast(ep, C.c_void_p), len(epochs),
                                              wp, wb, _ptr(offsets_log), _stream(stream))
    del arr, keep
    _check(rc, "r2_ring_allreduce_sim")


def r2_ring_allreduce_sim_inflight(desc: SimDesc, rank_bufs: Sequence, epochs, in_flight: Optional[Sequence[bool]],
                                   workspace, offsets_log: Optional[torch.Tensor] = None,
                                   plans: Optional[torch.Tensor] = None, stream=None,
                                   workspace_bytes: Optional[int] = None) -> None:
    """in_flight[i]: epoch i's failures strike during transmission epochs[i][0]; plans: device tensor of
    n_epochs * C * (C+1) 8-byte integers."""
    _check_lists(desc, rank_bufs, epochs)
    if in_flight is not None and len(in_flight) != len(epochs):
        raise ValueError("r2_ring_allreduce_sim_inflight: one flag per epoch")
    if plans is not None:
        assert plans.element_size() == 8 and plans.numel() >= len(epochs) * desc.n_channels * (desc.n_channels + 1)
    arr, p = _ptr_array(rank_bufs)
    ep, keep = _epoch_array(epochs)
    fl = (C.c_uint8 * max(len(epochs), 1))(*[1 if x else 0 for x in in_flight]) if in_flight is not None else None
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_ring_allreduce_sim_inflight(C.byref(desc.c()), p, C.cast(ep, C.c_void_p),
                                                       C.cast(fl, C.c_void_p) if fl is not None else None, len(epochs),
                                                       wp, wb, _ptr(offsets_log), _ptr(plans), _stream(stream))
    del arr, keep, fl
    _check(rc, "r2_ring_allreduce_sim_inflight")


STATIC_WORKSPACE_BYTES = 72 << 20  # R2_STATIC_WORKSPACE_BYTES


def r2_ring_allreduce_sim_static(desc: SimDesc, rank_bufs: Sequence, epochs,
                                 offsets_log: Optional[torch.Tensor] = None, stream=None) -> None:
    """The run whose workspace is the library's own static device array (nothing is allocated)."""
    _check_lists(desc, rank_bufs, epochs)
    arr, p = _ptr_array(rank_bufs)
    ep, keep = _epoch_array(epochs)
    rc = load_library().r2_ring_allreduce_sim_static(C.byref(desc.c()), p, C.cast(ep, C.c_void_p), len(epochs),
                                                     _ptr(offsets_log), _stream(stream))
    del arr, keep
    _check(rc, "r2_ring_allreduce_sim_static")


def r2_collective_sim(desc: SimDesc, rank_bufs: Sequence, epochs, workspace,
                      offsets_log: Optional[torch.Tensor] = None, stream=None,
                      workspace_bytes: Optional[int] = None) -> None:
    _check_lists(desc, rank_bufs, epochs)
    arr, p = _ptr_array(rank_bufs)
    ep, keep = _epoch_array(epochs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_collective_sim(C.byref(desc.c()), p, C.cast(ep, C.c_void_p), len(epochs),
                                          wp, wb, _ptr(offsets_log), _stream(stream))
    del arr, keep
    _check(rc, "r2_collective_sim")


def r2_sendrecv_sim(desc: SimDesc, send_bufs: Sequence, recv_bufs: Sequence, epochs, workspace,
                    offsets_log: Optional[torch.Tensor] = None, stream=None,
                    workspace_bytes: Optional[int] = None) -> None:
    sa, sp = _ptr_array(send_bufs)
    ra, rp = _ptr_array(recv_bufs)
    ep, keep = _epoch_array(epochs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_sendrecv_sim(C.byref(desc.c()), sp, rp, C.cast(ep, C.c_void_p), len(epochs),
                                        wp, wb, _ptr(offsets_log), _stream(stream))
    del sa, ra, keep
    _check(rc, "r2_sendrecv_sim")


def _rails_lists(desc: SimDesc, rank_epochs: Sequence, who: str):
    """The per-rank epoch lists as the C side takes them: (arrays to keep alive, list pointers, list lengths)."""
    if len(rank_epochs) != desc.n_ranks:
        raise ValueError(f"{who}: one epoch list per rank")
    if any(len(w) != desc.n_channels for eps in rank_epochs for _, _, w in eps):
        raise ValueError(f"{who}: one weight per channel in every epoch")
    lists = [_epoch_array(eps) for eps in rank_epochs]
    ptrs = (C.c_void_p * len(lists))(*[C.cast(a, C.c_void_p) for a, _ in lists])
    counts = (C.c_uint32 * len(lists))(*[len(eps) for eps in rank_epochs])
    return lists, ptrs, counts


def r2_ring_rails_sim(desc: SimDesc, rank_bufs: Sequence, rank_epochs: Sequence, workspace,
                      offsets_log: Optional[torch.Tensor] = None, stream=None,
                      workspace_bytes: Optional[int] = None) -> None:
    """rank_epochs[r]: the epoch list [(t_start, fail_mask, weights), ...] of rank r."""
    if len(rank_bufs) != desc.n_ranks:
        raise ValueError("r2_ring_rails_sim: one buffer per rank")
    lists, ptrs, counts = _rails_lists(desc, rank_epochs, "r2_ring_rails_sim")
    arr, p = _ptr_array(rank_bufs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_ring_rails_sim(C.byref(desc.c()), p, C.cast(ptrs, C.c_void_p), C.cast(counts, C.c_void_p),
                                          wp, wb, _ptr(offsets_log), _stream(stream))
    del arr, lists
    _check(rc, "r2_ring_rails_sim")


def r2_rails_resolve_schedule(desc: SimDesc, rank_epochs: Sequence) -> int:
    lists, ptrs, counts = _rails_lists(desc, rank_epochs, "r2_rails_resolve_schedule")
    rc = load_library().r2_rails_resolve_schedule(C.byref(desc.c()), C.cast(ptrs, C.c_void_p), C.cast(counts, C.c_void_p))
    del lists
    if rc < 0:
        raise R2Error(rc, "r2_rails_resolve_schedule")
    return rc


class RailsCall:
    """The arguments of r2_ring_rails_sim marshalled once (see SimCall)."""

    def __init__(self, desc: SimDesc, rank_bufs: Sequence, rank_epochs: Sequence, workspace,
                 offsets_log: Optional[torch.Tensor] = None, stream=None, workspace_bytes: Optional[int] = None):
        if len(rank_bufs) != desc.n_ranks:
            raise ValueError("RailsCall: one buffer per rank")
        self._lists, self._ptrs, self._counts = _rails_lists(desc, rank_epochs, "RailsCall")
        self._fn = load_library().r2_ring_rails_sim
        self._desc = desc.c()
        self._bufs, bufs_p = _ptr_array(rank_bufs)
        wp, wb = _ws(workspace, workspace_bytes)
        self._refs = (rank_bufs, workspace, offsets_log)  # keep the device memory alive
        self._args = (C.byref(self._desc), bufs_p, C.cast(self._ptrs, C.c_void_p), C.cast(self._counts, C.c_void_p),
                      wp, wb, _ptr(offsets_log), _stream(stream))

    def run(self) -> None:
        rc = self._fn(*self._args)
        if rc != R2_OK:
            raise R2Error(rc, "r2_ring_rails_sim")


def static_rails(weights: Sequence[int], fail_masks: Sequence[int]) -> List[list]:
    """Epoch lists for ranks whose channel state does not change during the run."""
    return [[(0, int(m), list(weights))] for m in fail_masks]


def r2_alltoall_sim(desc: SimDesc, send_bufs: Sequence, recv_bufs: Sequence, epochs, workspace,
                    offsets_log: Optional[torch.Tensor] = None, stream=None,
                    workspace_bytes: Optional[int] = None) -> None:
    sa, sp = _ptr_array(send_bufs)
    ra, rp = _ptr_array(recv_bufs)
    ep, keep = _epoch_array(epochs)
    wp, wb = _ws(workspace, workspace_bytes)
    rc = load_library().r2_alltoall_sim(C.byref(desc.c()), sp, rp, C.cast(ep, C.c_void_p), len(epochs),
                                        wp, wb, _ptr(offsets_log), _stream(stream))
    del sa, ra, keep
    _check(rc, "r2_alltoall_sim")
