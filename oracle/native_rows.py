"""ctypes door to oracle/csrc/run_rows.c (test infrastructure, like the rest of
oracle/): byte execution of a schedule with the rows of a step spread over the
host's cores.  The schedule comes from bcast_oracle; nothing here computes it.

Used by bench.py's all-cores CPU baseline and pinned against the plain numpy
execution by tests/test_oracle_pins.py.
"""

from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "csrc", "run_rows.c")
LIB = os.path.join(HERE, "liboracle_rows.so")

_lib = None


def build(verbose: bool = False) -> str:
    """Compile the C file with gcc (always recompiles)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", SOURCE, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout + res.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = C.CDLL(LIB)
        u64p, u32p = C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)
        L.oracle_run_rows.argtypes = [C.POINTER(C.c_void_p), C.c_int64, u64p, u32p, u32p, u64p, u64p,
                                      C.c_int, C.c_int]
        L.oracle_run_rows.restype = C.c_int
        L.oracle_rows_independent.argtypes = [C.c_int64, u64p, u32p, u32p, u64p, u64p]
        L.oracle_rows_independent.restype = C.c_int
        L.oracle_host_threads.restype = C.c_int
        _lib = L
    return _lib


def _arrays(steps):
    step_ptr = np.zeros(len(steps) + 1, np.uint64)
    flat = [r for rows in steps for r in rows]
    step_ptr[1:] = np.cumsum([len(rows) for rows in steps])
    a = np.array(flat, dtype=np.uint64).reshape(-1, 4)
    return (step_ptr, np.ascontiguousarray(a[:, 0].astype(np.uint32)), np.ascontiguousarray(a[:, 1].astype(np.uint32)),
            np.ascontiguousarray(a[:, 2]), np.ascontiguousarray(a[:, 3]))


def _p(arr, t):
    return arr.ctypes.data_as(C.POINTER(t))


def rows_independent(steps) -> bool:
    sp, src, dst, off, ln = _arrays(steps)
    rc = lib().oracle_rows_independent(len(steps), _p(sp, C.c_uint64), _p(src, C.c_uint32), _p(dst, C.c_uint32),
                                       _p(off, C.c_uint64), _p(ln, C.c_uint64))
    if rc < 0:
        raise RuntimeError("oracle_rows_independent: bad arguments")
    return rc == 1


def run_rows(bufs: Sequence[np.ndarray], steps, threads: int, staged: bool) -> None:
    """Apply the steps (lists of (src, dst, off, len) rows) to the uint8 buffers."""
    for b in bufs:
        assert b.dtype == np.uint8 and b.flags.c_contiguous
    sp, src, dst, off, ln = _arrays(steps)
    ptrs = (C.c_void_p * len(bufs))(*[b.ctypes.data for b in bufs])
    rc = lib().oracle_run_rows(ptrs, len(steps), _p(sp, C.c_uint64), _p(src, C.c_uint32), _p(dst, C.c_uint32),
                               _p(off, C.c_uint64), _p(ln, C.c_uint64), 1 if staged else 0, int(threads))
    if rc != 0:
        raise RuntimeError("oracle_run_rows failed")


def host_threads() -> int:
    return int(lib().oracle_host_threads())
