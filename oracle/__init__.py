"""CPU oracle for the ZipLine barrier search -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``zipline_oracle.c`` (plain host C, no GPU code).
Nothing in the product package imports this module; only the tests, the smoke
check and the benchmark's CPU-baseline leg do.  The arithmetic lives entirely
in the C file, whose header states the definition it follows (Section III
"The Problem", Section IV "Naive search" and Algorithm 2 of the paper).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zipline_oracle.c")
_SRC_RANGE = os.path.join(_HERE, "zipline_range_oracle.c")      # the paper's formal objective max(Z) - min(Z)
_LIB = os.path.join(_HERE, "libzipline_oracle.so")
_lib = None

METHODS = {"sweep": 0, "definition": 1, "naive": 2}
RANGE_METHODS = {"sweep": 0, "definition": 1, "naive": 2, "zipline": 3}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC),
                                                                        os.path.getmtime(_SRC_RANGE))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               _SRC, _SRC_RANGE, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.zl_oracle_batch.restype = ctypes.c_int
        lib.zl_oracle_batch.argtypes = [i64p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                        i64p, i32p, i64p, i32p, ctypes.c_int32, ctypes.c_int32,
                                        i32p]
        lib.zl_range_batch.restype = ctypes.c_int
        lib.zl_range_batch.argtypes = lib.zl_oracle_batch.argtypes
        _lib = lib
    return _lib


def zipline_range(ts, method: str = "sweep", threads: int = 0):
    """The search under the paper's formal objective d_Z = max(Z) - min(Z) (Section III).

    Same conventions as :func:`zipline`; the third result is ``dmin[B]`` instead of
    the summed wait.  Methods: "sweep", "definition", "naive", "zipline" (Algorithm 2
    as the paper states it, looking through Z for its minimum).
    """
    return _run(ts, "zl_range_batch", RANGE_METHODS[method], threads)


def zipline(ts, method: str = "sweep", threads: int = 0):
    """Run the oracle on ``ts`` of shape [B, P, R] (or [P, R]) int64.

    Returns ``(barrier[B] int64, iters[B, P] int32, wait[B] int64, rc[B] int32,
    threads_used)``.  ``rc`` is 0 for a valid instance and 1 where a row was
    not non-decreasing (that instance's outputs are left at zero).
    """
    return _run(ts, "zl_oracle_batch", METHODS[method], threads)


def _run(ts, entry: str, method: int, threads: int):
    a = np.ascontiguousarray(np.asarray(ts), dtype=np.int64)
    if a.ndim == 2:
        a = a[None]
    if a.ndim != 3:
        raise ValueError("ts must have shape [B, P, R] or [P, R]")
    B, P, R = a.shape
    if B < 1 or P < 1 or R < 1:
        raise ValueError("B, P and R must all be >= 1")
    lib = _load()
    barrier = np.zeros(B, dtype=np.int64)
    iters = np.zeros((B, P), dtype=np.int32)
    wait = np.zeros(B, dtype=np.int64)
    rc = np.zeros(B, dtype=np.int32)
    used = ctypes.c_int32(0)
    i64p = ctypes.POINTER(ctypes.c_int64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    r = getattr(lib, entry)(a.ctypes.data_as(i64p), B, P, R,
                            barrier.ctypes.data_as(i64p), iters.ctypes.data_as(i32p),
                            wait.ctypes.data_as(i64p), rc.ctypes.data_as(i32p),
                            int(method), int(threads), ctypes.byref(used))
    if r == 2:
        raise ValueError("oracle rejected its arguments")
    return barrier, iters, wait, rc, int(used.value)
