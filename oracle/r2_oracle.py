"""ctypes front-end of the C oracle (``r2_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Values travel as numpy arrays: fp32 data as
``float32``; bf16 data as ``uint16`` bit patterns; stage memory as ``uint8``.
Nothing here does any of the method's arithmetic: it marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "r2_oracle.c")
_LIB = os.path.join(_HERE, "libr2oracle.so")

F32, BF16 = 0, 1
OP_SUM, OP_COPY, OP_SUM_FORWARD = 0, 1, 2
PHASE_RS, PHASE_AG = 1, 2
PHASE_AR = PHASE_RS | PHASE_AG

_OK, _INVALID, _NO_HEALTHY, _CAPACITY, _NOMEM = 0, -1, -2, -4, -6


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


class NoHealthyChannel(OracleError):
    pass


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-Wall",
               "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Epoch(C.Structure):
    _fields_ = [("t_start", C.c_uint64), ("fail_mask", C.c_uint64),
                ("weights", C.POINTER(C.c_uint32))]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.r2o_partition.restype = C.c_int
        lib.r2o_partition.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint64,
                                      C.c_uint32, C.c_void_p]
        lib.r2o_rollback_plan.restype = C.c_int
        lib.r2o_rollback_plan.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.c_void_p]
        lib.r2o_reduce_copy.restype = C.c_int
        lib.r2o_reduce_copy.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_uint32, C.c_uint64]
        lib.r2o_ring_sim.restype = C.c_int
        lib.r2o_ring_sim.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_int, C.c_uint32,
                                     C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint32, C.c_int,
                                     C.c_void_p, C.c_uint64, C.c_void_p]
        lib.r2o_expected.restype = C.c_int
        lib.r2o_expected.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_int, C.c_uint32,
                                     C.c_int, C.c_void_p]
        lib.r2o_f32_to_bf16.restype = C.c_uint16
        lib.r2o_f32_to_bf16.argtypes = [C.c_float]
        lib.r2o_bf16_to_f32.restype = C.c_float
        lib.r2o_bf16_to_f32.argtypes = [C.c_uint16]
        lib.r2o_num_steps.restype = C.c_uint32
        lib.r2o_num_steps.argtypes = [C.c_uint32, C.c_int]
        lib.r2o_num_transmissions.restype = C.c_uint32
        lib.r2o_num_transmissions.argtypes = [C.c_uint32, C.c_int]
        lib.r2o_threads.restype = C.c_int
        lib.r2o_set_threads.argtypes = [C.c_int]
        _lib = lib
    return _lib


def _check(rc: int, what: str) -> None:
    if rc == _NO_HEALTHY:
        raise NoHealthyChannel(rc, what)
    if rc != _OK:
        raise OracleError(rc, what)


def _np_dtype(dtype: int):
    return np.float32 if dtype == F32 else np.uint16


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def threads() -> int:
    return int(_load().r2o_threads())


def set_threads(n: int) -> None:
    _load().r2o_set_threads(int(n))


def num_steps(R: int, phases: int) -> int:
    return int(_load().r2o_num_steps(R, phases))


def num_transmissions(R: int, phases: int) -> int:
    return int(_load().r2o_num_transmissions(R, phases))


def f32_to_bf16(x: float) -> int:
    return int(_load().r2o_f32_to_bf16(C.c_float(x)))


def bf16_to_f32(h: int) -> float:
    return float(_load().r2o_bf16_to_f32(C.c_uint16(h)))


def partition(weights: Sequence[int], fail_mask: int, nbytes: int, align: int) -> np.ndarray:
    w = np.ascontiguousarray(weights, dtype=np.uint32)
    off = np.zeros(len(w) + 1, dtype=np.uint64)
    rc = _load().r2o_partition(w.ctypes.data, fail_mask, len(w), nbytes, align, off.ctypes.data)
    _check(rc, "partition")
    return off


def rollback_plan(offsets: Sequence[int], weights: Sequence[int], mask_before: int, mask_after: int,
                  align: int) -> np.ndarray:
    """Cut points [C, C+1] of every newly failed channel's slice over the channels still healthy."""
    w = np.ascontiguousarray(weights, dtype=np.uint32)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    n = len(w)
    assert off.shape == (n + 1,)
    plan = np.zeros((n, n + 1), dtype=np.uint64)
    rc = _load().r2o_rollback_plan(off.ctypes.data, w.ctypes.data, mask_before, mask_after, n, align,
                                   plan.ctypes.data)
    _check(rc, "rollback_plan")
    return plan


def reduce_copy(local: np.ndarray, dtype: int, op: int,
                in_stage: Optional[Sequence[np.ndarray]], in_off: Optional[np.ndarray],
                out_stage: Optional[Sequence[np.ndarray]], out_off: Optional[np.ndarray],
                n_channels: int, cap: int) -> None:
    """One fused reduce-copy on one chunk, in place on ``local`` and ``out_stage``."""
    assert local.flags.c_contiguous and local.dtype == _np_dtype(dtype)
    ins = _ptr_array(in_stage) if in_stage is not None else None
    outs = _ptr_array(out_stage) if out_stage is not None else None
    io = np.ascontiguousarray(in_off, dtype=np.uint64) if in_off is not None else None
    oo = np.ascontiguousarray(out_off, dtype=np.uint64) if out_off is not None else None
    rc = _load().r2o_reduce_copy(
        local.ctypes.data, local.nbytes, dtype, op,
        C.cast(ins, C.c_void_p) if ins is not None else None,
        io.ctypes.data if io is not None else None,
        C.cast(outs, C.c_void_p) if outs is not None else None,
        oo.ctypes.data if oo is not None else None,
        n_channels, cap)
    _check(rc, "reduce_copy")


Epoch = Tuple[int, int, Sequence[int]]  # (t_start, fail_mask, weights)


def _epochs(epochs: Sequence[Epoch], n_channels: int):
    keep: List[np.ndarray] = []
    arr = (_Epoch * len(epochs))()
    for i, (t0, mask, w) in enumerate(epochs):
        wa = np.ascontiguousarray(w, dtype=np.uint32)
        assert wa.shape == (n_channels,)
        keep.append(wa)
        arr[i].t_start = t0
        arr[i].fail_mask = mask
        arr[i].weights = wa.ctypes.data_as(C.POINTER(C.c_uint32))
    return arr, keep


def ring_sim(bufs: Sequence[np.ndarray], dtype: int, n_slabs: int, n_channels: int, align: int,
             epochs: Sequence[Epoch], phases: int, cap: Optional[int] = None,
             stage_fill: int = 0xA5):
    """The ring, step by step, in place on ``bufs``.

    Returns ``(offsets_log[T_total, C+1], stage[2, R, S, C, cap])``; stage bytes
    never written keep ``stage_fill``.
    """
    R = len(bufs)
    N = bufs[0].size
    for b in bufs:
        assert b.flags.c_contiguous and b.dtype == _np_dtype(dtype) and b.size == N
    es = bufs[0].itemsize
    chunk_bytes = (N // (n_slabs * R)) * es
    if cap is None:
        cap = max(chunk_bytes, 1)
    T_total = n_slabs * num_transmissions(R, phases)
    log = np.zeros((T_total, n_channels + 1), dtype=np.uint64)
    stage = np.full((2, R, n_slabs, n_channels, cap), stage_fill, dtype=np.uint8)
    ep, keep = _epochs(epochs, n_channels)
    rc = _load().r2o_ring_sim(C.cast(_ptr_array(bufs), C.c_void_p), R, N, dtype, n_slabs,
                              n_channels, align, C.cast(ep, C.c_void_p), len(epochs), phases,
                              stage.ctypes.data, cap, log.ctypes.data)
    del keep
    _check(rc, "ring_sim")
    return log, stage


def expected(inputs: Sequence[np.ndarray], dtype: int, n_slabs: int, phases: int) -> List[np.ndarray]:
    """What every rank must hold afterwards, by the plain definition."""
    R = len(inputs)
    N = inputs[0].size
    for b in inputs:
        assert b.flags.c_contiguous and b.dtype == _np_dtype(dtype) and b.size == N
    outs = [np.empty_like(inputs[0]) for _ in range(R)]
    rc = _load().r2o_expected(C.cast(_ptr_array(inputs), C.c_void_p), R, N, dtype, n_slabs,
                              phases, C.cast(_ptr_array(outs), C.c_void_p))
    _check(rc, "expected")
    return outs
