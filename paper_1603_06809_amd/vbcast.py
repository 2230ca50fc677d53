"""Thin ctypes binding over libvbcast.so (declared in include/vbcast.h).

Argument marshalling only: every step of the broadcast, table generation
included, runs in the library's kernels.  torch is used to own device memory
and streams.  There is no fallback: if the library has not been built, loading
fails with an error that says how to build it.
"""

from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvbcast.so")

NATIVE = 0
TUNED = 1
BINOMIAL = 2
SCATTER_RDB = 3
ALGOS = {"native": NATIVE, "tuned": TUNED, "binomial": BINOMIAL, "scatter_rdb": SCATTER_RDB}
ALGO_NAMES = {v: k for k, v in ALGOS.items()}

RING_STEPS = 0
RING_CHAINS = 1
CHAIN_AUTO = 0
CHAIN_INLINE = 1
CHAIN_TABLES = 2

SUCCESS, ERR_ARG, ERR_ROOT, ERR_COUNT, ERR_ALIGN, ERR_HIP, ERR_NOMEM, ERR_LIMIT = range(8)
STATIC_MAX_RANKS = 513

EXPORTS = [
    "vbcast_comm_create", "vbcast_comm_destroy", "bcast_plan", "bcast_run", "bcast_run_static", "bcast_run_steps", "bcast_run_chain_steps",
    "bcast_run_steps_timed", "bcast_run_timed", "bcast_plan_info", "bcast_plan_export", "bcast_plan_export_desc",
    "bcast_plan_export_tiles", "bcast_plan_export_chain", "bcast_plan_census", "bcast_plan_destroy", "vbcast_set_tile_bytes", "vbcast_set_chain_slab_bytes",
    "vbcast_set_ring_executor", "vbcast_set_chain_schedule", "vbcast_set_chain_workgroups_per_cu", "vbcast_set_xcd_count", "vbcast_select_algo",
    "bcast_plan_smp", "bcast_run_smp", "bcast_run_smp_phase", "bcast_smp_subplan",
    "bcast_plan_smp_destroy", "bcast_strerror",
]


class PlanInfo(C.Structure):
    _fields_ = [
        ("P", C.c_int32), ("root", C.c_int32), ("algo", C.c_int32),
        ("n_scatter_steps", C.c_int32), ("n_steps", C.c_int32), ("tile_bytes", C.c_int32),
        ("n", C.c_uint64), ("ss", C.c_uint64),
        ("scatter_rows", C.c_uint64), ("ring_rows", C.c_uint64),
        ("scatter_bytes", C.c_uint64), ("ring_bytes", C.c_uint64),
        ("bytes_moved", C.c_uint64), ("ring_msgs_issued", C.c_uint64),
        ("pairing_mismatches", C.c_uint64), ("n_tiles", C.c_uint64),
        ("run_launches", C.c_uint64),
    ]


class Census(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in (
        "scatter_inter_msgs", "scatter_inter_bytes", "scatter_intra_msgs", "scatter_intra_bytes",
        "ring_inter_msgs", "ring_inter_bytes", "ring_intra_msgs", "ring_intra_bytes")]

    def as_dict(self) -> dict:
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class VbcastError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"vbcast error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Load libvbcast.so once.  torch is imported first so that the HIP runtime
    the library binds to is the one torch already loaded."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with "
            "`python -c 'import __graft_entry__ as g; g.build()'` "
            "(or `python paper_1603_06809_amd/build.py`); there is no CPU fallback")
    import torch  # noqa: F401  (loads libamdhip64 with the soname the library needs)

    L = C.CDLL(LIB_PATH)
    vp, u64p, u32p, i32p = C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32), C.POINTER(C.c_int32)
    L.vbcast_comm_create.argtypes = [C.c_int, C.POINTER(vp), C.c_size_t, C.POINTER(vp)]
    L.vbcast_comm_destroy.argtypes = [vp]
    L.bcast_plan.argtypes = [vp, C.c_size_t, C.c_size_t, C.c_int, C.c_int, vp, C.POINTER(vp)]
    L.bcast_run.argtypes = [vp, vp]
    L.bcast_run_static.argtypes = [vp, C.c_size_t, C.c_size_t, C.c_int, C.c_int, vp]
    L.bcast_run_steps.argtypes = [vp, C.c_int, C.c_int, vp]
    L.bcast_run_chain_steps.argtypes = [vp, C.c_int, C.c_int, vp]
    L.bcast_run_steps_timed.argtypes = [vp, C.c_int, C.c_int, vp, C.POINTER(C.c_float)]
    L.bcast_run_timed.argtypes = [vp, vp, C.POINTER(C.c_float)]
    L.bcast_plan_info.argtypes = [vp, C.POINTER(PlanInfo)]
    L.bcast_plan_export.argtypes = [vp, u64p, u32p, u32p, u64p, u64p, u64p]
    L.bcast_plan_export_desc.argtypes = [vp, u64p, u64p, i32p, i32p, i32p, i32p, i32p]
    L.bcast_plan_export_tiles.argtypes = [vp, C.c_int, u32p, u32p, u32p]
    L.bcast_plan_export_chain.argtypes = [vp, i32p, C.POINTER(C.c_uint8)]
    L.bcast_plan_census.argtypes = [vp, C.c_int, vp, C.POINTER(Census)]
    L.bcast_plan_destroy.argtypes = [vp]
    L.vbcast_set_tile_bytes.argtypes = [C.c_size_t]
    L.vbcast_set_chain_slab_bytes.argtypes = [C.c_size_t]
    L.vbcast_set_ring_executor.argtypes = [C.c_int]
    L.vbcast_set_chain_workgroups_per_cu.argtypes = [C.c_int]
    L.vbcast_set_xcd_count.argtypes = [C.c_int]
    L.vbcast_set_chain_schedule.argtypes = [C.c_int]
    L.bcast_plan_smp.argtypes = [vp, C.c_size_t, C.c_size_t, C.c_int, C.c_int, C.c_int, vp, C.POINTER(vp)]
    L.bcast_run_smp.argtypes = [vp, vp]
    L.bcast_run_smp_phase.argtypes = [vp, C.c_int, vp]
    L.bcast_smp_subplan.argtypes = [vp, C.c_int, i32p, C.POINTER(vp), i32p, i32p, i32p]
    L.bcast_plan_smp_destroy.argtypes = [vp]
    L.vbcast_select_algo.argtypes = [C.c_size_t, C.c_int, C.c_int, C.POINTER(C.c_int)]
    L.bcast_strerror.argtypes = [C.c_int]
    L.bcast_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name != "bcast_strerror":
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def bcast_strerror(code: int) -> str:
    return lib().bcast_strerror(code).decode()


def _check(code: int) -> None:
    if code != SUCCESS:
        raise VbcastError(code, bcast_strerror(code))


def _ptr(arr: Optional[np.ndarray], ctype):
    return None if arr is None else arr.ctypes.data_as(C.POINTER(ctype))


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def vbcast_set_tile_bytes(tile_bytes: int) -> None:
    _check(lib().vbcast_set_tile_bytes(tile_bytes))


def vbcast_set_chain_slab_bytes(slab_bytes: int) -> None:
    _check(lib().vbcast_set_chain_slab_bytes(slab_bytes))


def vbcast_set_ring_executor(mode: int) -> None:
    _check(lib().vbcast_set_ring_executor(mode))


def vbcast_set_chain_workgroups_per_cu(k: int) -> None:
    _check(lib().vbcast_set_chain_workgroups_per_cu(k))


def vbcast_set_chain_schedule(mode: int) -> None:
    _check(lib().vbcast_set_chain_schedule(mode))


def vbcast_set_xcd_count(n_xcd: int) -> None:
    _check(lib().vbcast_set_xcd_count(n_xcd))


def vbcast_select_algo(nbytes: int, P: int, tuned: bool) -> int:
    out = C.c_int()
    _check(lib().vbcast_select_algo(nbytes, P, 1 if tuned else 0, C.byref(out)))
    return out.value


class Comm:
    """vbcast_comm: P rank buffers given as device pointers (ints)."""

    def __init__(self, pointers: Sequence[int], buf_bytes: int):
        self.P = len(pointers)
        arr = (C.c_void_p * max(self.P, 1))(*pointers)
        self._h = C.c_void_p()
        _check(lib().vbcast_comm_create(self.P, arr, buf_bytes, C.byref(self._h)))

    @classmethod
    def from_tensors(cls, bufs) -> "Comm":
        """bufs: list of P uint8 device tensors of equal size (kept alive by the caller)."""
        nbytes = {b.numel() * b.element_size() for b in bufs}
        if len(nbytes) != 1:
            raise ValueError("rank buffers must have equal size")
        return cls([b.data_ptr() for b in bufs], nbytes.pop())

    def destroy(self) -> None:
        if self._h:
            _check(lib().vbcast_comm_destroy(self._h))
            self._h = C.c_void_p()


@dataclass
class Tables:
    step_ptr: np.ndarray
    src: np.ndarray
    dst: np.ndarray
    off: np.ndarray
    len: np.ndarray
    step_bytes: np.ndarray

    def rows_of(self, s: int) -> List[tuple]:
        a, b = int(self.step_ptr[s]), int(self.step_ptr[s + 1])
        return [(int(self.src[k]), int(self.dst[k]), int(self.off[k]), int(self.len[k]))
                for k in range(a, b)]


class Plan:
    """vbcast_plan handle; see bcast_plan in include/vbcast.h."""

    def __init__(self, comm: Comm, count: int, dtype_size: int, root: int, algo: int, stream=None):
        self.comm = comm
        self._h = C.c_void_p()
        _check(lib().bcast_plan(comm._h, count, dtype_size, root, algo,
                                _stream_handle(stream), C.byref(self._h)))

    def info(self) -> PlanInfo:
        out = PlanInfo()
        _check(lib().bcast_plan_info(self._h, C.byref(out)))
        return out

    def run(self, stream=None) -> None:
        _check(lib().bcast_run(self._h, _stream_handle(stream)))

    def run_steps(self, first: int, last: int, stream=None) -> None:
        _check(lib().bcast_run_steps(self._h, first, last, _stream_handle(stream)))

    def run_chain_steps(self, first: int, last: int, stream=None) -> None:
        _check(lib().bcast_run_chain_steps(self._h, first, last, _stream_handle(stream)))

    def run_steps_timed(self, first: int, last: int, stream=None) -> np.ndarray:
        ms = np.zeros(max(last - first, 0), dtype=np.float32)
        _check(lib().bcast_run_steps_timed(self._h, first, last, _stream_handle(stream),
                                           _ptr(ms, C.c_float)))
        return ms

    def run_timed(self, stream=None) -> np.ndarray:
        """One un-graphed run; milliseconds of (table generation, scatter, ring)."""
        ms = np.zeros(3, dtype=np.float32)
        _check(lib().bcast_run_timed(self._h, _stream_handle(stream), _ptr(ms, C.c_float)))
        return ms

    def export(self) -> Tables:
        i = self.info()
        nrows = int(i.scatter_rows + i.ring_rows)
        t = Tables(np.zeros(i.n_steps + 1, np.uint64), np.zeros(nrows, np.uint32),
                   np.zeros(nrows, np.uint32), np.zeros(nrows, np.uint64),
                   np.zeros(nrows, np.uint64), np.zeros(i.n_steps, np.uint64))
        _check(lib().bcast_plan_export(self._h, _ptr(t.step_ptr, C.c_uint64), _ptr(t.src, C.c_uint32),
                                       _ptr(t.dst, C.c_uint32), _ptr(t.off, C.c_uint64),
                                       _ptr(t.len, C.c_uint64), _ptr(t.step_bytes, C.c_uint64)))
        return t

    def export_desc(self) -> dict:
        P = self.info().P
        d = {"chunk_off": np.zeros(P + 1, np.uint64), "chunk_len": np.zeros(P, np.uint64)}
        for k in ("rel", "left", "right", "sw_step", "sw_flag"):
            d[k] = np.zeros(P, np.int32)
        _check(lib().bcast_plan_export_desc(
            self._h, _ptr(d["chunk_off"], C.c_uint64), _ptr(d["chunk_len"], C.c_uint64),
            _ptr(d["rel"], C.c_int32), _ptr(d["left"], C.c_int32), _ptr(d["right"], C.c_int32),
            _ptr(d["sw_step"], C.c_int32), _ptr(d["sw_flag"], C.c_int32)))
        return d

    def export_tiles(self, step: int):
        n = C.c_uint32()
        _check(lib().bcast_plan_export_tiles(self._h, step, C.byref(n), None, None))
        row = np.zeros(n.value, np.uint32)
        idx = np.zeros(n.value, np.uint32)
        _check(lib().bcast_plan_export_tiles(self._h, step, C.byref(n), _ptr(row, C.c_uint32),
                                             _ptr(idx, C.c_uint32)))
        return row, idx

    def export_chain(self):
        """(holder, moves) as [P, n_steps] arrays; see bcast_plan_export_chain."""
        i = self.info()
        holder = np.zeros((i.P, i.n_steps), np.int32)
        moves = np.zeros((i.P, i.n_steps), np.uint8)
        _check(lib().bcast_plan_export_chain(self._h, _ptr(holder, C.c_int32), _ptr(moves, C.c_uint8)))
        return holder, moves

    def census(self, ranks_per_node: int, stream=None) -> dict:
        out = Census()
        _check(lib().bcast_plan_census(self._h, ranks_per_node, _stream_handle(stream), C.byref(out)))
        return out.as_dict()

    def destroy(self) -> None:
        if self._h:
            _check(lib().bcast_plan_destroy(self._h))
            self._h = C.c_void_p()


class SmpPlan:
    """vbcast_smp_plan handle: the three-phase multi-core-aware broadcast."""

    def __init__(self, comm: Comm, count: int, dtype_size: int, root: int, ranks_per_node: int,
                 ring_algo, stream=None):
        self.comm = comm
        self._h = C.c_void_p()
        _check(lib().bcast_plan_smp(comm._h, count, dtype_size, root, ranks_per_node,
                                    ALGOS.get(ring_algo, ring_algo), _stream_handle(stream),
                                    C.byref(self._h)))

    def run(self, stream=None) -> None:
        _check(lib().bcast_run_smp(self._h, _stream_handle(stream)))

    def run_phase(self, phase: int, stream=None) -> None:
        _check(lib().bcast_run_smp_phase(self._h, phase, _stream_handle(stream)))

    def subplans(self):
        """[(phase, members, Plan)] in execution order; the Plan objects are views
        owned by this plan (do not destroy them)."""
        n = C.c_int()
        _check(lib().bcast_smp_subplan(self._h, 0, C.byref(n), None, None, None, None))
        out = []
        for k in range(n.value):
            h, phase, nm = C.c_void_p(), C.c_int(), C.c_int()
            members = np.zeros(self.comm.P, np.int32)
            _check(lib().bcast_smp_subplan(self._h, k, None, C.byref(h), C.byref(phase), C.byref(nm),
                                           _ptr(members, C.c_int32)))
            view = Plan.__new__(Plan)
            view.comm, view._h = self.comm, h
            out.append((phase.value, members[: nm.value].tolist(), view))
        return out

    def destroy(self) -> None:
        if self._h:
            _check(lib().bcast_plan_smp_destroy(self._h))
            self._h = C.c_void_p()


def bcast_plan_smp(comm: Comm, count: int, dtype_size: int, root: int, ranks_per_node: int,
                   ring_algo, stream=None) -> SmpPlan:
    return SmpPlan(comm, count, dtype_size, root, ranks_per_node, ring_algo, stream)


def bcast_plan(comm: Comm, count: int, dtype_size: int, root: int, algo, stream=None) -> Plan:
    """Same name and argument order as the C entry point; ``algo`` may be the
    integer constant or 'native' / 'tuned'."""
    return Plan(comm, count, dtype_size, root, ALGOS.get(algo, algo), stream)


def bcast_run(plan: Plan, stream=None) -> None:
    plan.run(stream)


def bcast_run_static(comm: Comm, count: int, dtype_size: int, root: int, algo, stream=None) -> None:
    """One whole broadcast with the tables in the library's static device array
    (no allocation); see bcast_run_static in include/vbcast.h."""
    _check(lib().bcast_run_static(comm._h, count, dtype_size, root, ALGOS.get(algo, algo),
                                  _stream_handle(stream)))


def bcast_run_steps(plan: Plan, first: int, last: int, stream=None) -> None:
    plan.run_steps(first, last, stream)


def bcast_run_chain_steps(plan: Plan, first: int, last: int, stream=None) -> None:
    plan.run_chain_steps(first, last, stream)
