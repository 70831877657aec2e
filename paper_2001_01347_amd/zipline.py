"""ctypes binding of libebsp_zipline.so (see include/ebsp_zipline.h and include/ebsp_zipline_bench.h).

Argument marshalling only: every step of the search runs in the HIP kernels.
PyTorch supplies device memory (``torch.empty``) and the current stream.  The
library must have been built (``python -m paper_2001_01347_amd.build`` or
``__graft_entry__.build()``); if it is missing the first call raises -- there
is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libebsp_zipline.so")

EBSP_OK = 0
STATUS_OK, STATUS_UNSORTED, STATUS_OVERFLOW = 0, 1, 2

EXPORTS = ("ebsp_gridscan_workspace_bytes", "ebsp_gridscan_batch", "ebsp_zipline_workspace_bytes", "ebsp_predict_zipline_workspace_bytes", "ebsp_zipline_tune_sweep", "ebsp_zipline_batch", "ebsp_zipline_batch_static",
           "ebsp_zipline_static_scratch_bytes", "ebsp_zipline_range_workspace_bytes",
           "ebsp_zipline_range_batch", "ebsp_predict_zipline_batch", "ebsp_simulate_workspace_bytes",
           "ebsp_simulate_supersteps", "ebsp_zipline_tune", "ebsp_zipline_shape_info", "ebsp_zipline_profile_begin",
           "ebsp_zipline_profile_end", "ebsp_zipline_copy_probe", "ebsp_zipline_read_probe", "ebsp_zipline_memory_info",
           "ebsp_zipline_kernel_count",
           "ebsp_zipline_kernel_name", "ebsp_last_error")

READ_SINK_WORDS = 256     # EBSP_READ_SINK_WORDS of the bench header

_lib = None


class ZipLineError(RuntimeError):
    pass


def load() -> ctypes.CDLL:
    """Load the HIP library (once). Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ZipLineError(f"{LIB_PATH} is missing: build it first "
                               "(python -m paper_2001_01347_amd.build); there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        lib.ebsp_zipline_workspace_bytes.restype = sz
        lib.ebsp_zipline_workspace_bytes.argtypes = [i64, i32, i32]
        lib.ebsp_gridscan_workspace_bytes.restype = sz
        lib.ebsp_gridscan_workspace_bytes.argtypes = [i64, i32, i32, i32]
        lib.ebsp_gridscan_batch.restype = ctypes.c_int
        lib.ebsp_gridscan_batch.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.ebsp_predict_zipline_workspace_bytes.restype = sz
        lib.ebsp_predict_zipline_workspace_bytes.argtypes = [i64, i32, i32]
        lib.ebsp_zipline_tune_sweep.restype = ctypes.c_int
        lib.ebsp_zipline_tune_sweep.argtypes = [i32, i32, i32]
        common = [vp, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.ebsp_zipline_batch.restype = ctypes.c_int
        lib.ebsp_zipline_batch.argtypes = common
        lib.ebsp_zipline_batch_static.restype = ctypes.c_int
        lib.ebsp_zipline_batch_static.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp]
        lib.ebsp_zipline_static_scratch_bytes.restype = sz
        lib.ebsp_zipline_static_scratch_bytes.argtypes = []
        lib.ebsp_zipline_range_workspace_bytes.restype = sz
        lib.ebsp_zipline_range_workspace_bytes.argtypes = [i64, i32, i32]
        lib.ebsp_zipline_range_batch.restype = ctypes.c_int
        lib.ebsp_zipline_range_batch.argtypes = common
        lib.ebsp_predict_zipline_batch.restype = ctypes.c_int
        lib.ebsp_predict_zipline_batch.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.ebsp_simulate_workspace_bytes.restype = sz
        lib.ebsp_simulate_workspace_bytes.argtypes = [i64, i32, i32]
        lib.ebsp_simulate_supersteps.restype = ctypes.c_int
        lib.ebsp_simulate_supersteps.argtypes = [vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.ebsp_zipline_shape_info.restype = ctypes.c_int
        lib.ebsp_zipline_shape_info.argtypes = [i64, i32, i32, ctypes.POINTER(ctypes.c_int64)]
        lib.ebsp_zipline_tune.restype = ctypes.c_int
        lib.ebsp_zipline_tune.argtypes = [i32, i32, i32]
        lib.ebsp_zipline_profile_begin.restype = ctypes.c_int
        lib.ebsp_zipline_profile_begin.argtypes = [i32]
        lib.ebsp_zipline_profile_end.restype = ctypes.c_int
        lib.ebsp_zipline_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        lib.ebsp_zipline_copy_probe.restype = ctypes.c_int
        lib.ebsp_zipline_copy_probe.argtypes = [vp, vp, sz, vp]
        lib.ebsp_zipline_read_probe.restype = ctypes.c_int
        lib.ebsp_zipline_read_probe.argtypes = [vp, sz, vp, vp]
        lib.ebsp_zipline_memory_info.restype = ctypes.c_int
        lib.ebsp_zipline_memory_info.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.ebsp_zipline_kernel_count.restype = ctypes.c_int
        lib.ebsp_zipline_kernel_count.argtypes = []
        lib.ebsp_zipline_kernel_name.restype = ctypes.c_char_p
        lib.ebsp_zipline_kernel_name.argtypes = [ctypes.c_int]
        lib.ebsp_last_error.restype = ctypes.c_char_p
        lib.ebsp_last_error.argtypes = []
        _lib = lib
    return _lib


def ebsp_last_error() -> str:
    return load().ebsp_last_error().decode()


def ebsp_zipline_workspace_bytes(B: int, P: int, R: int) -> int:
    return int(load().ebsp_zipline_workspace_bytes(B, P, R))


def ebsp_predict_zipline_workspace_bytes(B: int, P: int, R: int) -> int:
    return int(load().ebsp_predict_zipline_workspace_bytes(B, P, R))


def ebsp_zipline_tune_sweep(sweep_min: int = 0, slice_keys: int = 0, lines: int = 0) -> None:
    """Which stored-row batches take the one-pass sweep, its slice length and the lines of a window (0 = default); see the header."""
    rc = load().ebsp_zipline_tune_sweep(int(sweep_min), int(slice_keys), int(lines))
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_tune_sweep failed ({rc}): {ebsp_last_error()}")


def ebsp_zipline_range_workspace_bytes(B: int, P: int, R: int) -> int:
    return int(load().ebsp_zipline_range_workspace_bytes(B, P, R))


def ebsp_zipline_shape_info(B: int, P: int, R: int) -> Dict[str, int]:
    """How the library handles a shape: {'multi', 'window_cap', 'bins', 'max_windows', 'window_fill', 'slices'}."""
    info = (ctypes.c_int64 * 6)()
    rc = load().ebsp_zipline_shape_info(B, P, R, info)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_shape_info failed ({rc}): {ebsp_last_error()}")
    return {"multi": int(info[0]), "window_cap": int(info[1]), "bins": int(info[2]), "max_windows": int(info[3]),
            "window_fill": int(info[4]), "slices": int(info[5])}


def ebsp_zipline_tune(window_cap: int = 0, single_max: int = 0, window_fill: int = 0) -> None:
    """Set the process-wide tuning knobs (0 = default); see the header."""
    rc = load().ebsp_zipline_tune(int(window_cap), int(single_max), int(window_fill))
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_tune failed ({rc}): {ebsp_last_error()}")


def ebsp_zipline_kernel_names() -> Tuple[str, ...]:
    lib = load()
    return tuple(lib.ebsp_zipline_kernel_name(i).decode() for i in range(lib.ebsp_zipline_kernel_count()))


def _check_buffer(name: str, t: torch.Tensor, dev: torch.device, dtype: torch.dtype, shape) -> None:
    """A caller-supplied output must be exactly what the kernels will write: anything else would be written out of
    bounds, or at a host address."""
    if not isinstance(t, torch.Tensor) or t.device != dev or t.dtype != dtype or tuple(t.shape) != tuple(shape) \
            or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous {dtype} tensor of shape {tuple(shape)} on {dev}")


def _check_workspace(ws: Optional[torch.Tensor], dev: torch.device, need: int) -> None:
    if ws is None:
        if need:
            raise ValueError(f"this shape needs a workspace of {need} bytes")
        return
    if not isinstance(ws, torch.Tensor) or ws.device != dev or ws.dtype != torch.uint8 or ws.dim() != 1 \
            or not ws.is_contiguous() or ws.numel() < need:
        raise ValueError(f"workspace must be a contiguous 1-D uint8 tensor of at least {need} bytes on {dev}")
    if ws.data_ptr() % 256:
        raise ValueError("workspace must be 256-byte aligned")


def _outputs(dev, B, P, barrier, iters, third, status, lead=()):
    """The four outputs: new tensors where none is given, checked ones where the caller supplies them."""
    shapes = (lead + (B,), lead + (B, P), lead + (B,), lead + (B,))
    dtypes = (torch.int64, torch.int32, torch.int64, torch.int32)
    names = ("barrier", "iters", "wait", "status")
    out = []
    for name, t, shape, dtype in zip(names, (barrier, iters, third, status), shapes, dtypes):
        if t is None:
            t = torch.empty(shape, dtype=dtype, device=dev)
        else:
            _check_buffer(name, t, dev, dtype, shape)
        out.append(t)
    return out


def _check(ts: torch.Tensor) -> Tuple[int, int, int]:
    if ts.dim() != 3 or ts.dtype != torch.int64 or not ts.is_cuda or not ts.is_contiguous():
        raise ValueError("ts must be a contiguous int64 CUDA tensor of shape [B, P, R]")
    return tuple(int(x) for x in ts.shape)


def _prepare(ts, barrier, iters, wait, status, workspace, workspace_bytes=None):
    B, P, R = _check(ts)
    dev = ts.device
    barrier, iters, wait, status = _outputs(dev, B, P, barrier, iters, wait, status)
    need = (workspace_bytes or ebsp_zipline_workspace_bytes)(B, P, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check_workspace(workspace, dev, need)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    stream = torch.cuda.current_stream(dev).cuda_stream
    args = [ts.data_ptr(), B, P, R, barrier.data_ptr(), iters.data_ptr(), wait.data_ptr(),
            status.data_ptr(), ws_ptr, ws_len, stream]
    return args, (barrier, iters, wait, status)


def ebsp_zipline_batch(ts: torch.Tensor, barrier: Optional[torch.Tensor] = None,
                       iters: Optional[torch.Tensor] = None, wait: Optional[torch.Tensor] = None,
                       status: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None):
    """Enqueue the batched search on the current stream of ``ts``'s device.

    Returns ``(barrier[B], iters[B, P], wait[B], status[B])`` device tensors
    (the ones passed in, or new ones).  Does not synchronise.
    """
    args, outs = _prepare(ts, barrier, iters, wait, status, workspace)
    with torch.cuda.device(ts.device):
        rc = load().ebsp_zipline_batch(*args)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_batch failed ({rc}): {ebsp_last_error()}")
    return outs


def ebsp_zipline_static_scratch_bytes() -> int:
    return int(load().ebsp_zipline_static_scratch_bytes())


def ebsp_zipline_batch_static(ts: torch.Tensor, barrier: torch.Tensor, iters: torch.Tensor, wait: torch.Tensor,
                              status: torch.Tensor):
    """``ebsp_zipline_batch`` on the library's own static scratch: nothing is allocated, here or in the library,
    so the caller passes every output.  Returns ``(barrier, iters, wait, status)``.  Does not synchronise."""
    B, P, R = _check(ts)
    barrier, iters, wait, status = _outputs(ts.device, B, P, barrier, iters, wait, status)
    with torch.cuda.device(ts.device):
        rc = load().ebsp_zipline_batch_static(ts.data_ptr(), B, P, R, barrier.data_ptr(), iters.data_ptr(), wait.data_ptr(),
                                              status.data_ptr(), torch.cuda.current_stream(ts.device).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_batch_static failed ({rc}): {ebsp_last_error()}")
    return barrier, iters, wait, status


def ebsp_zipline_range_batch(ts: torch.Tensor, barrier: Optional[torch.Tensor] = None,
                             iters: Optional[torch.Tensor] = None, dmin: Optional[torch.Tensor] = None,
                             status: Optional[torch.Tensor] = None,
                             workspace: Optional[torch.Tensor] = None):
    """The search under the paper's formal objective max(Z) - min(Z); see the header.

    Returns ``(barrier[B], iters[B, P], dmin[B], status[B])`` device tensors.  Does not synchronise.
    """
    args, outs = _prepare(ts, barrier, iters, dmin, status, workspace, ebsp_zipline_range_workspace_bytes)
    with torch.cuda.device(ts.device):
        rc = load().ebsp_zipline_range_batch(*args)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_range_batch failed ({rc}): {ebsp_last_error()}")
    return outs


def ebsp_gridscan_workspace_bytes(B: int, P: int, R: int, full: bool) -> int:
    return int(load().ebsp_gridscan_workspace_bytes(B, P, R, 1 if full else 0))


def ebsp_gridscan_batch(ts: torch.Tensor, full: bool = False, barrier: Optional[torch.Tensor] = None,
                        iters: Optional[torch.Tensor] = None, dz: Optional[torch.Tensor] = None,
                        status: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """GridScan (``full=False``) or FullGridScan (``full=True``), the paper's comparators; see the header.

    Returns ``(barrier[B], iters[B, P], dz[B], status[B])`` device tensors.  Does not synchronise.
    """
    B, P, R = _check(ts)
    dev = ts.device
    barrier, iters, dz, status = _outputs(dev, B, P, barrier, iters, dz, status)
    need = ebsp_gridscan_workspace_bytes(B, P, R, full)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check_workspace(workspace, dev, need)
    with torch.cuda.device(dev):
        rc = load().ebsp_gridscan_batch(ts.data_ptr(), B, P, R, 1 if full else 0, barrier.data_ptr(), iters.data_ptr(),
                                        dz.data_ptr(), status.data_ptr(), workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(),
                                        torch.cuda.current_stream(dev).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_gridscan_batch failed ({rc}): {ebsp_last_error()}")
    return barrier, iters, dz, status


def ebsp_predict_zipline_batch(last_end: torch.Tensor, interval: torch.Tensor, R: int,
                               barrier: Optional[torch.Tensor] = None, iters: Optional[torch.Tensor] = None,
                               wait: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                               workspace: Optional[torch.Tensor] = None):
    """The search over predicted rows ``last_end[b, p] + (i + 1) * interval[b, p]``, i < R; see the header.

    ``last_end`` and ``interval`` are contiguous int64 CUDA tensors of shape [B, P].
    Returns ``(barrier[B], iters[B, P], wait[B], status[B])`` device tensors.  Does not synchronise.
    """
    for t in (last_end, interval):
        if t.dim() != 2 or t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("last_end and interval must be contiguous int64 CUDA tensors of shape [B, P]")
    if last_end.shape != interval.shape or last_end.device != interval.device:
        raise ValueError("last_end and interval must have the same shape and device")
    B, P = (int(x) for x in last_end.shape)
    R = int(R)
    dev = last_end.device
    barrier, iters, wait, status = _outputs(dev, B, P, barrier, iters, wait, status)
    need = ebsp_predict_zipline_workspace_bytes(B, P, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check_workspace(workspace, dev, need)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = load().ebsp_predict_zipline_batch(last_end.data_ptr(), interval.data_ptr(), B, P, R,
                                               barrier.data_ptr(), iters.data_ptr(), wait.data_ptr(),
                                               status.data_ptr(), ws_ptr, ws_len,
                                               torch.cuda.current_stream(dev).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_predict_zipline_batch failed ({rc}): {ebsp_last_error()}")
    return barrier, iters, wait, status


def ebsp_simulate_workspace_bytes(B: int, P: int, R: int) -> int:
    return int(load().ebsp_simulate_workspace_bytes(B, P, R))


def ebsp_simulate_supersteps(last_end0: torch.Tensor, interval: torch.Tensor, R: int, sync_cost: int = 0,
                             barrier: Optional[torch.Tensor] = None, iters: Optional[torch.Tensor] = None,
                             wait: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                             workspace: Optional[torch.Tensor] = None):
    """S supersteps of predict -> search -> resume at the barrier; see the header.

    ``last_end0`` is a contiguous int64 CUDA tensor [B, P], ``interval`` one of shape [S, B, P].
    Returns ``(barrier[S, B], iters[S, B, P], wait[S, B], status[S, B])`` device tensors.  Does not synchronise.
    """
    for t in (last_end0, interval):
        if t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("last_end0 and interval must be contiguous int64 CUDA tensors")
    if last_end0.dim() != 2 or interval.dim() != 3 or interval.shape[1:] != last_end0.shape \
            or interval.device != last_end0.device:
        raise ValueError("last_end0 must have shape [B, P] and interval [S, B, P], on one device")
    S, B, P = (int(x) for x in interval.shape)
    R = int(R)
    dev = last_end0.device
    barrier, iters, wait, status = _outputs(dev, B, P, barrier, iters, wait, status, lead=(S,))
    need = ebsp_simulate_workspace_bytes(B, P, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check_workspace(workspace, dev, need)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_len = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(dev):
        rc = load().ebsp_simulate_supersteps(last_end0.data_ptr(), interval.data_ptr(), int(sync_cost), S, B, P, R,
                                             barrier.data_ptr(), iters.data_ptr(), wait.data_ptr(),
                                             status.data_ptr(), ws_ptr, ws_len,
                                             torch.cuda.current_stream(dev).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_simulate_supersteps failed ({rc}): {ebsp_last_error()}")
    return barrier, iters, wait, status


def ebsp_zipline_copy_probe(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Plain streaming device copy src -> dst (same byte size) on the current stream: a bandwidth yardstick."""
    nbytes = src.numel() * src.element_size()
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
            and dst.numel() * dst.element_size() == nbytes):
        raise ValueError("src and dst must be contiguous CUDA tensors of the same byte size")
    with torch.cuda.device(src.device):
        rc = load().ebsp_zipline_copy_probe(src.data_ptr(), dst.data_ptr(), nbytes,
                                            torch.cuda.current_stream(src.device).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_copy_probe failed ({rc}): {ebsp_last_error()}")


def ebsp_zipline_read_probe(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Plain streaming device read of src on the current stream, summed into sink (READ_SINK_WORDS int64 on the device)."""
    if not (src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.dtype == torch.int64 and sink.is_contiguous()
            and sink.numel() == READ_SINK_WORDS and sink.device == src.device):
        raise ValueError(f"src must be a contiguous CUDA tensor and sink {READ_SINK_WORDS} int64 words on the same device")
    with torch.cuda.device(src.device):
        rc = load().ebsp_zipline_read_probe(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                            torch.cuda.current_stream(src.device).cuda_stream)
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_read_probe failed ({rc}): {ebsp_last_error()}")


def ebsp_zipline_memory_info() -> Tuple[int, int]:
    """(memory clock in kHz, memory bus width in bits) of the current device, as HIP reports them."""
    clk, bus = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = load().ebsp_zipline_memory_info(ctypes.byref(clk), ctypes.byref(bus))
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_memory_info failed ({rc}): {ebsp_last_error()}")
    return int(clk.value), int(bus.value)


def ebsp_zipline_profile_begin(max_calls: int) -> None:
    """Start recording per-kernel HIP events in this thread's following batch calls."""
    rc = load().ebsp_zipline_profile_begin(int(max_calls))
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_profile_begin failed ({rc}): {ebsp_last_error()}")


def ebsp_zipline_profile_end() -> Tuple[Dict[str, float], int]:
    """Synchronise; return ({kernel name: summed ms}, number of profiled calls)."""
    lib = load()
    n = lib.ebsp_zipline_kernel_count()
    ms = (ctypes.c_float * n)()
    calls = ctypes.c_int32(0)
    rc = lib.ebsp_zipline_profile_end(ms, ctypes.byref(calls))
    if rc != EBSP_OK:
        raise ZipLineError(f"ebsp_zipline_profile_end failed ({rc}): {ebsp_last_error()}")
    names = ebsp_zipline_kernel_names()
    return {names[i]: float(ms[i]) for i in range(n)}, int(calls.value)
