"""ctypes wrapper around exec.c, the plain CPU schedule executor (oracle side; test infrastructure).

See exec.c for what is computed and the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

from .schedule import Schedule

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "exec.c")
_LIB = os.path.join(_HERE, "liboracle_exec.so")

DTYPES = {"i32": (0, np.int32), "f32": (1, np.float32), "f16": (2, np.float16)}

_lib = None


def build(force: bool = False) -> str:
    """Compile exec.c with gcc (no fast-math, no contraction, OpenMP over elements only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_execute.restype = ctypes.c_int32
        lib.oracle_execute.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                       ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32]
        lib.oracle_f16_to_f32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_f32_to_f16.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        lib.oracle_max_threads.restype = ctypes.c_int32
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def execute(dtype: str, num_chunks: int, elems_per_chunk: int, sched: Schedule,
            bufs: Sequence[np.ndarray], threads: int = 1,
            first_elem: int = 0, num_elems: Optional[int] = None,
            slot: Optional[np.ndarray] = None, slots_per_rank: Optional[int] = None) -> None:
    """Run the schedule in place on P host buffers.

    Default layout: one contiguous array of G*elems_per_chunk per rank, chunk c in slot c.  With `slot`
    (G x P int32, -1 = never held) rank n keeps chunk c in slot[c, n] of a buffer of slots_per_rank chunks.
    """
    code, npdt = DTYPES[dtype]
    P = len(bufs)
    per_rank = num_chunks if slot is None else int(slots_per_rank)
    slot_arr = None if slot is None else np.ascontiguousarray(slot, dtype=np.int32)
    if slot_arr is not None and slot_arr.shape != (num_chunks, P):
        raise ValueError("slot map must be G x P")
    for b in bufs:
        if b.dtype != npdt or not b.flags["C_CONTIGUOUS"] or b.size != per_rank * elems_per_chunk:
            raise ValueError("rank buffer has the wrong dtype, layout or size")
    if num_elems is None:
        num_elems = elems_per_chunk - first_elem
    sends = np.ascontiguousarray(sched.sends, dtype=np.int32)
    ptrs = (ctypes.c_void_p * P)(*[b.ctypes.data for b in bufs])
    rc = _load().oracle_execute(P, num_chunks, elems_per_chunk, code, sched.num_steps, sends.shape[0],
                                sends.ctypes.data, ctypes.cast(ptrs, ctypes.c_void_p),
                                first_elem, num_elems, threads,
                                None if slot_arr is None else slot_arr.ctypes.data, per_rank)
    if rc != 0:
        raise ValueError("oracle_execute rejected its arguments")


def f16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    _load().oracle_f16_to_f32(h.ctypes.data, out.ctypes.data, h.size)
    return out


def f32_to_f16(f: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(f, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    _load().oracle_f32_to_f16(f.ctypes.data, out.ctypes.data, f.size)
    return out


def algorithmic_bytes(sched: Schedule, chunk_bytes: int):
    """Bytes that executing the schedule must move, counted per step.

    A copy group (one (chunk, source) sent to k destinations in a step) reads
    the chunk once and writes it k times: (1 + k) chunks.  A reduce group (k
    sources into one (chunk, destination) in a step) reads k + 1 chunks and
    writes one: (k + 2) chunks.  `unfused` counts every send on its own: 2
    chunks for a copy, 3 for a reduce.
    """
    from collections import Counter
    copy_groups = Counter()
    red_groups = Counter()
    unfused = 0
    for (c, n, m, s, op) in sched.sends.tolist():
        if op == 0:
            copy_groups[(s, c, n)] += 1
            unfused += 2
        else:
            red_groups[(s, c, m)] += 1
            unfused += 3
    fused = sum(1 + k for k in copy_groups.values()) + sum(k + 2 for k in red_groups.values())
    return fused * chunk_bytes, unfused * chunk_bytes
