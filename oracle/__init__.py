"""CPU oracle for the ZipLine barrier search -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``zipline_oracle.c`` (plain host C, no GPU code).
Nothing in the product package imports this module; only the tests, the smoke
check and the benchmark's CPU-baseline leg do.  The arithmetic of the search
lives entirely in the C files, whose headers state the definition they follow
(Section III "The Problem", Section IV "Naive search" and Algorithm 2 of the
paper).  Two small steps around the search are written out here in numpy:
the linear prediction of a worker's next R end timestamps (:func:`predicted_rows`)
and the run of supersteps that resumes every worker at the barrier
(:func:`simulate`); the paper describes both only in words (Section I, Section
III, Fig. 1), so both are readings, stated in their docstrings.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zipline_oracle.c")
_SRC_RANGE = os.path.join(_HERE, "zipline_range_oracle.c")      # the paper's formal objective max(Z) - min(Z)
_SRC_GRID = os.path.join(_HERE, "gridscan_oracle.c")            # GridScan and FullGridScan (Section IV, Algorithm 1)
_LIB = os.path.join(_HERE, "libzipline_oracle.so")
_lib = None

METHODS = {"sweep": 0, "definition": 1, "naive": 2}
RANGE_METHODS = {"sweep": 0, "definition": 1, "naive": 2, "latest": 3}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only). Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_RANGE),
                                                                        os.path.getmtime(_SRC_GRID))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               _SRC, _SRC_RANGE, _SRC_GRID, "-o", _LIB]
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
        lib.gs_batch.restype = ctypes.c_int
        lib.gs_batch.argtypes = [i64p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                 i64p, i32p, i64p, i32p, ctypes.c_int32, i32p]
        lib.ebsp_zipline_oracle.restype = ctypes.c_int
        lib.ebsp_zipline_oracle.argtypes = [i64p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, i64p, i32p, i64p, ctypes.c_int32]
        _lib = lib
    return _lib


def zipline_range(ts, method: str = "sweep", threads: int = 0):
    """The search under the paper's formal objective d_Z = max(Z) - min(Z) (Section III).

    Same conventions as :func:`zipline`; the third result is ``dmin[B]`` instead of
    the summed wait.  Methods: "sweep", "definition", "naive", "latest" (the sweep with a
    table of every worker's latest timestamp, searched for its minimum).
    """
    return _run(ts, "zl_range_batch", RANGE_METHODS[method], threads)


def zipline(ts, method: str = "sweep", threads: int = 0):
    """Run the oracle on ``ts`` of shape [B, P, R] (or [P, R]) int64.

    Returns ``(barrier[B] int64, iters[B, P] int32, wait[B] int64, rc[B] int32,
    threads_used)``.  ``rc`` is 0 for a valid instance and 1 where a row was
    not non-decreasing (that instance's outputs are left at zero).
    """
    return _run(ts, "zl_oracle_batch", METHODS[method], threads)


GRID_METHODS = {"scan": 0, "bisect": 1}


def gridscan(ts, full: bool = False, method: str = "scan", threads: int = 0):
    """GridScan (``full=False``) or FullGridScan (``full=True``) of Section IV, Algorithm 1, on ``ts`` [B, P, R] (or [P, R]).

    Returns ``(barrier[B] int64, iters[B, P] int32, dz[B] int64, rc[B] int32, threads_used)``: ``dz`` is the smallest
    ``max(Z) - min(Z)`` the heuristic finds, ``barrier = max(Z*)``, ``iters[p]`` = 1 + the index of worker p's point in Z*.
    Methods: "scan" looks at every point of every other row (the order of work of Algorithm 1), "bisect" finds the
    nearest point by bisection (for larger inputs).
    """
    a = np.ascontiguousarray(np.asarray(ts), dtype=np.int64)
    if a.ndim == 2:
        a = a[None]
    if a.ndim != 3:
        raise ValueError("ts must have shape [B, P, R] or [P, R]")
    B, P, R = a.shape
    lib = _load()
    barrier = np.zeros(B, dtype=np.int64)
    iters = np.zeros((B, P), dtype=np.int32)
    dz = np.zeros(B, dtype=np.int64)
    rc = np.zeros(B, dtype=np.int32)
    used = ctypes.c_int32(0)
    i64p = ctypes.POINTER(ctypes.c_int64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    r = lib.gs_batch(a.ctypes.data_as(i64p), B, P, R, 1 if full else 0, GRID_METHODS[method],
                     barrier.ctypes.data_as(i64p), iters.ctypes.data_as(i32p), dz.ctypes.data_as(i64p),
                     rc.ctypes.data_as(i32p), int(threads), ctypes.byref(used))
    if r == 2:
        raise ValueError("oracle rejected its arguments")
    return barrier, iters, dz, rc, int(used.value)


def zipline_c_abi(ts, threads: int = 0):
    """The summed-wait search through the oracle library's C entry point ``ebsp_zipline_oracle``
    (``include/ebsp_zipline_oracle.h``): the sweep route, host pointers.  Returns ``(barrier, iters, wait, rc)``."""
    a = np.ascontiguousarray(np.asarray(ts), dtype=np.int64)
    if a.ndim != 3:
        raise ValueError("ts must have shape [B, P, R]")
    B, P, R = a.shape
    barrier = np.zeros(B, dtype=np.int64)
    iters = np.zeros((B, P), dtype=np.int32)
    wait = np.zeros(B, dtype=np.int64)
    i64p = ctypes.POINTER(ctypes.c_int64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = _load().ebsp_zipline_oracle(a.ctypes.data_as(i64p), B, P, R, barrier.ctypes.data_as(i64p),
                                     iters.ctypes.data_as(i32p), wait.ctypes.data_as(i64p), int(threads))
    return barrier, iters, wait, int(rc)


def predicted_rows(last_end, interval, R: int) -> np.ndarray:
    """The prediction phase (Section I and Section III: a worker's coming iterations are taken to last
    as long as its most recent one): worker p's i-th coming iteration ends at

        t[..., p, i] = last_end[..., p] + (i + 1) * interval[..., p],   i = 0 .. R-1.

    The paper gives no formula; this linear one is the reading.  int64 in, int64 out, one more axis.
    """
    le = np.asarray(last_end, dtype=np.int64)
    iv = np.asarray(interval, dtype=np.int64)
    out = np.empty(le.shape + (int(R),), dtype=np.int64)
    for i in range(int(R)):
        out[..., i] = le + (i + 1) * iv
    return out


def simulate(last_end0, interval, R: int, sync_cost: int = 0, method: str = "sweep", threads: int = 0):
    """A run of S supersteps (Fig. 1: a superstep is the time between two barriers; Section III: the
    server decides one barrier after the other from the workers' most recent iteration times).

    ``last_end0[B, P]``: the time every worker starts the run at; ``interval[S, B, P]``: worker p's
    iteration time during superstep s.  Superstep s predicts R end timestamps per worker from its
    start time and interval, runs the search over them, and every worker of the instance starts
    superstep s + 1 at ``barrier + sync_cost``.  Readings (the paper states none of them): workers
    run exactly as predicted up to the barrier, all of them resume together, and a synchronisation
    takes a fixed time.  With R = 1 this is BSP with one iteration per superstep.  An instance
    whose rows the search rejects (rc != 0) keeps its start times.

    Returns ``(barrier[S, B], iters[S, B, P], wait[S, B], rc[S, B], threads_used)``.
    """
    start = np.array(last_end0, dtype=np.int64)
    iv = np.asarray(interval, dtype=np.int64)
    if start.ndim != 2 or iv.ndim != 3 or iv.shape[1:] != start.shape:
        raise ValueError("last_end0 must have shape [B, P] and interval [S, B, P]")
    S, B, P = iv.shape
    barrier = np.zeros((S, B), dtype=np.int64)
    iters = np.zeros((S, B, P), dtype=np.int32)
    wait = np.zeros((S, B), dtype=np.int64)
    rc = np.zeros((S, B), dtype=np.int32)
    used = 0
    for s in range(S):
        barrier[s], iters[s], wait[s], rc[s], used = zipline(predicted_rows(start, iv[s], R), method, threads)
        for b in range(B):
            if rc[s, b] == 0:
                start[b, :] = barrier[s, b] + int(sync_cost)
    return barrier, iters, wait, rc, used


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
