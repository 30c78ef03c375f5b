"""ctypes binding of libsccl.so: the same names as include/sccl.h, argument marshalling only.

Every step of the hot path runs in the library's kernels; nothing here computes.
There is no CPU fallback: if the library is missing the import of a function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsccl.so")

SCCL_MAX_RANKS = 64
SCCL_OK = 0
STATUS_NAMES = ["SCCL_OK", "SCCL_ERR_INVALID_ARG", "SCCL_ERR_TOPOLOGY", "SCCL_ERR_SEND_NO_SOURCE",
                "SCCL_ERR_SEND_NO_LINK", "SCCL_ERR_BANDWIDTH", "SCCL_ERR_POSTCONDITION", "SCCL_ERR_HAZARD",
                "SCCL_ERR_ALIGNMENT", "SCCL_ERR_OVERLAP", "SCCL_ERR_NOMEM", "SCCL_ERR_DEVICE", "SCCL_ERR_SCRATCH"]
SCCL_STATIC_SCRATCH_BYTES = 256 * 1024
SCCL_I32, SCCL_F32, SCCL_F16 = 0, 1, 2
DTYPE_CODES = {"i32": SCCL_I32, "f32": SCCL_F32, "f16": SCCL_F16}
SCCL_COPY, SCCL_REDUCE_SUM = 0, 1
SCCL_PLAN_HOST_ONLY = 1
SCCL_LOWER_AUTO, SCCL_LOWER_MEMORY, SCCL_LOWER_STAGED = 0, 1, 2


class sccl_edge_t(ctypes.Structure):
    _fields_ = [("src", ctypes.c_int32), ("dst", ctypes.c_int32)]


class sccl_bw_t(ctypes.Structure):
    _fields_ = [("edges", ctypes.POINTER(sccl_edge_t)), ("num_edges", ctypes.c_int32),
                ("chunks_per_round", ctypes.c_int32)]


class sccl_topology_t(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int32), ("bw", ctypes.POINTER(sccl_bw_t)), ("num_bw", ctypes.c_int32)]


class sccl_collective_t(ctypes.Structure):
    _fields_ = [("num_global_chunks", ctypes.c_int32), ("pre", ctypes.c_void_p), ("post", ctypes.c_void_p),
                ("combining", ctypes.c_int32), ("dtype", ctypes.c_int32), ("elems_per_chunk", ctypes.c_int64),
                ("slot", ctypes.c_void_p), ("slots_per_rank", ctypes.c_int32)]


class sccl_send_t(ctypes.Structure):
    _fields_ = [("chunk", ctypes.c_int32), ("src", ctypes.c_int32), ("dst", ctypes.c_int32),
                ("step", ctypes.c_int32), ("op", ctypes.c_int32)]


class sccl_schedule_t(ctypes.Structure):
    _fields_ = [("num_steps", ctypes.c_int32), ("rounds", ctypes.c_void_p), ("sends", ctypes.c_void_p),
                ("num_sends", ctypes.c_int64)]


class sccl_options_t(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("block_threads", ctypes.c_int32),
                ("vectors_per_thread", ctypes.c_int32), ("max_workgroups", ctypes.c_int32),
                ("lowering", ctypes.c_int32), ("slice_vectors", ctypes.c_int32),
                ("staged_threads", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class sccl_stats_t(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int32), ("num_global_chunks", ctypes.c_int32),
                ("num_steps", ctypes.c_int32), ("num_rounds", ctypes.c_int32), ("k", ctypes.c_int32),
                ("num_sends", ctypes.c_int64), ("num_copy_groups", ctypes.c_int64),
                ("num_reduce_groups", ctypes.c_int64), ("max_fan_in", ctypes.c_int32),
                ("max_fan_out", ctypes.c_int32), ("chunks_per_node", ctypes.c_int32), ("chunk_bytes", ctypes.c_int64),
                ("bytes_per_rank", ctypes.c_int64), ("bytes_min", ctypes.c_int64),
                ("bytes_unfused", ctypes.c_int64), ("vector_bytes", ctypes.c_int32),
                ("block_threads", ctypes.c_int32), ("vectors_per_thread", ctypes.c_int32),
                ("num_work_items", ctypes.c_int64), ("grid_workgroups", ctypes.c_int32),
                ("lowering", ctypes.c_int32), ("staged_available", ctypes.c_int32), ("num_cells", ctypes.c_int32),
                ("num_cells_loaded", ctypes.c_int32), ("num_cells_stored", ctypes.c_int32),
                ("num_levels", ctypes.c_int32), ("staged_levels", ctypes.c_int32), ("staged_tasks", ctypes.c_int32),
                ("max_level_tasks", ctypes.c_int32), ("max_chunk_groups", ctypes.c_int32),
                ("slice_vectors", ctypes.c_int32), ("staged_threads", ctypes.c_int32),
                ("staged_lds_bytes", ctypes.c_int32), ("num_slices", ctypes.c_int64),
                ("static_table_bytes", ctypes.c_int64)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


EXPORTS = ["sccl_plan_create", "sccl_plan_create_ex", "sccl_execute", "sccl_execute_stepwise", "sccl_execute_memcpy",
           "sccl_execute_static", "sccl_plan_stats", "sccl_plan_table", "sccl_plan_destroy",
           "sccl_status_string", "sccl_plan_cost", "sccl_select_plan", "sccl_cost_fit", "sccl_cost_fit_intercept"]

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  What is built in-tree is loaded as it is; only when nothing is there is it compiled
    first.  There is no fallback: without the library every call raises."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):                      # nothing built yet: build once, in-tree
            try:
                from . import build as _build
                _build.build_library()
            except Exception as e:
                raise RuntimeError(f"{LIB_PATH} is missing and could not be built ({e}): run `python -m "
                                   "paper_2008_08708_amd.build` (or __graft_entry__.build()); this package has no "
                                   "CPU fallback") from e
        # torch first: it brings its own copy of the HIP runtime (same soname as the system's), and the
        # process must hold exactly one -- the one torch allocates device memory and streams with.
        # Loaded after torch, this library's dependency resolves to that already-loaded runtime.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        L.sccl_plan_create.restype = ctypes.c_int
        L.sccl_plan_create.argtypes = [ctypes.POINTER(sccl_topology_t), ctypes.POINTER(sccl_collective_t),
                                       ctypes.POINTER(sccl_schedule_t), ctypes.POINTER(ctypes.c_void_p)]
        L.sccl_plan_create_ex.restype = ctypes.c_int
        L.sccl_plan_create_ex.argtypes = [ctypes.POINTER(sccl_topology_t), ctypes.POINTER(sccl_collective_t),
                                          ctypes.POINTER(sccl_schedule_t), ctypes.POINTER(sccl_options_t),
                                          ctypes.POINTER(ctypes.c_void_p)]
        L.sccl_execute.restype = ctypes.c_int
        L.sccl_execute.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p]
        for fn in (L.sccl_execute_stepwise, L.sccl_execute_memcpy, L.sccl_execute_static):
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p]
        L.sccl_plan_stats.restype = ctypes.c_int
        L.sccl_plan_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(sccl_stats_t)]
        L.sccl_plan_table.restype = ctypes.c_int
        L.sccl_plan_table.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)]
        L.sccl_plan_destroy.restype = None
        L.sccl_plan_destroy.argtypes = [ctypes.c_void_p]
        L.sccl_status_string.restype = ctypes.c_char_p
        L.sccl_status_string.argtypes = [ctypes.c_int]
        L.sccl_plan_cost.restype = ctypes.c_int
        L.sccl_plan_cost.argtypes = [ctypes.c_void_p, ctypes.c_double, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
        L.sccl_select_plan.restype = ctypes.c_int
        L.sccl_select_plan.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                       ctypes.POINTER(ctypes.c_int32)]
        L.sccl_cost_fit.restype = ctypes.c_int
        L.sccl_cost_fit.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.sccl_cost_fit_intercept.restype = ctypes.c_int
        L.sccl_cost_fit_intercept.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                              ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


class ScclError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        self.name = sccl_status_string(status)
        super().__init__(f"{where}: {self.name}")


# ---- plain descriptions of the three inputs (host data only; what sccl_plan_create marshals)

@dataclass
class Topology:
    num_nodes: int
    bw: List[Tuple[List[Tuple[int, int]], int]]          # [(edges, chunks_per_round)]


@dataclass
class Collective:
    num_global_chunks: int
    pre: np.ndarray                                       # G x P of 0/1
    post: np.ndarray
    combining: bool
    dtype: str                                            # "i32" | "f32" | "f16"
    elems_per_chunk: int
    slot: Optional[np.ndarray] = None                     # optional G x P int32 layout, -1 = never held
    slots_per_rank: int = 0


@dataclass
class Schedule:
    rounds: List[int]
    sends: np.ndarray                                     # (n, 5) int32: chunk, src, dst, step, op


class Plan:
    """Owns an sccl_plan_t*; freed by sccl_plan_destroy or when collected."""

    def __init__(self, handle: int):
        self.handle = ctypes.c_void_p(handle)
        self.num_nodes = 0                                 # P: how many rank buffers an execute call must be given

    def __del__(self):
        try:
            sccl_plan_destroy(self)
        except Exception:
            pass


def sccl_status_string(status: int) -> str:
    return lib().sccl_status_string(int(status)).decode()


def sccl_plan_create(topology: Topology, collective: Collective, schedule: Schedule,
                     options: Optional[dict] = None) -> Plan:
    """sccl_plan_create / sccl_plan_create_ex: marshal the three descriptions and return the plan.

    options: dict with any of the fields of sccl_options_t (flags, block_threads, vectors_per_thread,
    max_workgroups, lowering, slice_vectors, staged_threads).
    Raises ScclError carrying the library's status on failure.
    """
    L = lib()
    keep = []                                              # keeps the ctypes arrays alive during the call
    bws = (sccl_bw_t * max(1, len(topology.bw)))()
    for i, (edges, b) in enumerate(topology.bw):
        arr = (sccl_edge_t * max(1, len(edges)))()
        for j, (s, d) in enumerate(edges):
            arr[j].src, arr[j].dst = int(s), int(d)
        keep.append(arr)
        bws[i].edges = ctypes.cast(arr, ctypes.POINTER(sccl_edge_t))
        bws[i].num_edges = len(edges)
        bws[i].chunks_per_round = int(b)
    topo = sccl_topology_t(int(topology.num_nodes), ctypes.cast(bws, ctypes.POINTER(sccl_bw_t)), len(topology.bw))
    pre = np.ascontiguousarray(collective.pre, dtype=np.uint8)
    post = np.ascontiguousarray(collective.post, dtype=np.uint8)
    slot = None if collective.slot is None else np.ascontiguousarray(collective.slot, dtype=np.int32)
    coll = sccl_collective_t(int(collective.num_global_chunks), pre.ctypes.data, post.ctypes.data,
                             int(bool(collective.combining)), DTYPE_CODES[collective.dtype],
                             int(collective.elems_per_chunk),
                             None if slot is None else slot.ctypes.data, int(collective.slots_per_rank))
    rounds = np.ascontiguousarray(schedule.rounds, dtype=np.int32)
    sends = np.ascontiguousarray(schedule.sends, dtype=np.int32).reshape(-1, 5)
    sched = sccl_schedule_t(len(rounds), rounds.ctypes.data, sends.ctypes.data, sends.shape[0])
    out = ctypes.c_void_p()
    if options:
        o = sccl_options_t(**{k: int(v) for k, v in options.items()})
        st = L.sccl_plan_create_ex(ctypes.byref(topo), ctypes.byref(coll), ctypes.byref(sched), ctypes.byref(o),
                                   ctypes.byref(out))
    else:
        st = L.sccl_plan_create(ctypes.byref(topo), ctypes.byref(coll), ctypes.byref(sched), ctypes.byref(out))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_plan_create")
    plan = Plan(out.value)
    plan.num_nodes = sccl_plan_stats(plan)["num_nodes"]
    return plan


def _device_ptr(b) -> int:
    if hasattr(b, "data_ptr"):
        return int(b.data_ptr())
    return int(b)


def _execute(name: str, plan: Plan, rank_buffers: Sequence, stream) -> None:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    if len(rank_buffers) != plan.num_nodes:                # the library reads exactly P pointers
        raise ValueError(f"{name}: the plan has {plan.num_nodes} ranks, {len(rank_buffers)} buffers were given")
    ptrs = (ctypes.c_void_p * len(rank_buffers))(*[_device_ptr(b) for b in rank_buffers])
    st = getattr(lib(), name)(plan.handle, ptrs, ctypes.c_void_p(int(stream)))
    if st != SCCL_OK:
        raise ScclError(st, name)


def sccl_execute(plan: Plan, rank_buffers: Sequence, stream=None) -> None:
    """Enqueue the plan on `stream` (a torch stream, a raw hipStream_t value, or None for torch's current stream).

    rank_buffers: P device tensors (or raw device addresses).
    """
    _execute("sccl_execute", plan, rank_buffers, stream)


def sccl_execute_stepwise(plan: Plan, rank_buffers: Sequence, stream=None) -> None:
    """One kernel per step (comparator lowering); same arguments and results as sccl_execute."""
    _execute("sccl_execute_stepwise", plan, rank_buffers, stream)


def sccl_execute_memcpy(plan: Plan, rank_buffers: Sequence, stream=None) -> None:
    """One device-to-device copy per COPY send (comparator lowering; plans without REDUCE sends only)."""
    _execute("sccl_execute_memcpy", plan, rank_buffers, stream)


def sccl_execute_static(plan: Plan, rank_buffers: Sequence, stream=None) -> None:
    """sccl_execute without any device allocation: the step table goes into the library's static device array."""
    _execute("sccl_execute_static", plan, rank_buffers, stream)


def sccl_plan_stats(plan: Plan) -> dict:
    s = sccl_stats_t()
    st = lib().sccl_plan_stats(plan.handle, ctypes.byref(s))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_plan_stats")
    return s.as_dict()


def sccl_plan_table(plan: Plan, lowering: int) -> Tuple[np.ndarray, List[int]]:
    """(the step table of the given lowering as int32 words, its four info words)."""
    words = ctypes.c_int64()
    info = (ctypes.c_int32 * 4)()
    st = lib().sccl_plan_table(plan.handle, int(lowering), None, 0, ctypes.byref(words), info)
    if st != SCCL_OK:
        raise ScclError(st, "sccl_plan_table")
    out = np.zeros(max(1, words.value), dtype=np.int32)
    st = lib().sccl_plan_table(plan.handle, int(lowering), out.ctypes.data, words.value, ctypes.byref(words), info)
    if st != SCCL_OK:
        raise ScclError(st, "sccl_plan_table")
    return out[:words.value], [int(x) for x in info]


def sccl_plan_destroy(plan: Plan) -> None:
    if plan.handle:
        lib().sccl_plan_destroy(plan.handle)
        plan.handle = ctypes.c_void_p()


def sccl_plan_cost(plan: Plan, alpha: float, beta: float) -> float:
    """Seconds the paper's (alpha, beta) model gives the plan."""
    out = ctypes.c_double()
    st = lib().sccl_plan_cost(plan.handle, float(alpha), float(beta), ctypes.byref(out))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_plan_cost")
    return out.value


def sccl_select_plan(plans: Sequence[Plan], alpha: float, beta: float) -> int:
    """Index of the plan the cost model prefers."""
    arr = (ctypes.c_void_p * max(1, len(plans)))(*[p.handle for p in plans])
    out = ctypes.c_int32()
    st = lib().sccl_select_plan(arr, len(plans), float(alpha), float(beta), ctypes.byref(out))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_select_plan")
    return out.value


def sccl_cost_fit(a: Sequence[float], b: Sequence[float], t: Sequence[float]) -> Tuple[float, float]:
    """(alpha, beta) of the least-squares fit t = a * alpha + b * beta."""
    aa, bb, tt = (np.ascontiguousarray(x, dtype=np.float64) for x in (a, b, t))
    if not (aa.shape == bb.shape == tt.shape and aa.ndim == 1):
        raise ValueError("a, b, t must be 1-d arrays of one length")
    al, be = ctypes.c_double(), ctypes.c_double()
    st = lib().sccl_cost_fit(aa.size, aa.ctypes.data, bb.ctypes.data, tt.ctypes.data, ctypes.byref(al), ctypes.byref(be))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_cost_fit")
    return al.value, be.value


def sccl_cost_fit_intercept(a: Sequence[float], b: Sequence[float], t: Sequence[float],
                            weights: Optional[Sequence[float]] = None) -> Tuple[float, float, float]:
    """(t0, alpha, beta) of the (weighted) least-squares fit t = t0 + a * alpha + b * beta."""
    aa, bb, tt = (np.ascontiguousarray(x, dtype=np.float64) for x in (a, b, t))
    if not (aa.shape == bb.shape == tt.shape and aa.ndim == 1):
        raise ValueError("a, b, t must be 1-d arrays of one length")
    ww = None if weights is None else np.ascontiguousarray(weights, dtype=np.float64)
    if ww is not None and ww.shape != aa.shape:
        raise ValueError("weights must have the length of the samples")
    t0, al, be = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    st = lib().sccl_cost_fit_intercept(aa.size, aa.ctypes.data, bb.ctypes.data, tt.ctypes.data,
                                       None if ww is None else ww.ctypes.data, ctypes.byref(t0),
                                       ctypes.byref(al), ctypes.byref(be))
    if st != SCCL_OK:
        raise ScclError(st, "sccl_cost_fit_intercept")
    return t0.value, al.value, be.value
