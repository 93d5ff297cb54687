"""Thin Python binding of the C ABI in include/rowsum.h (argument marshalling only).

Same rules as binding.py: tensors become device pointers, the current torch stream becomes
the hipStream_t, shapes and dtypes are checked against what the call claims, every arithmetic
step runs in the HIP kernel, and there is no CPU or eager fallback.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

ROWSUM_DTYPE_FP32 = 0
ROWSUM_DTYPE_FP16 = 1
ROWSUM_DTYPE_BF16 = 2

ROWSUM_OK = 0
ROWSUM_ERR_INVALID_ARG = -1
ROWSUM_ERR_LAUNCH = -3

_lib = None


class RowSumError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"rowsum: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.ROWSUM_LIB_PATH


def load() -> ctypes.CDLL:
    """Loads librowsum_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure("rowsum"))
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.rowsum_fwd.argtypes = [vp, vp, i64, i64, i32, vp]
    lib.rowsum_fwd.restype = i32
    lib.rowsum_fwd_tuned.argtypes = [vp, vp, i64, i64, i32, vp, i32]
    lib.rowsum_fwd_tuned.restype = i32
    lib.rowsum_auto_threads_per_row.argtypes = [i64, i32]
    lib.rowsum_auto_threads_per_row.restype = i32
    lib.rowsum_status_string.argtypes = [i32]
    lib.rowsum_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def rowsum_status_string(status: int) -> str:
    return load().rowsum_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != ROWSUM_OK:
        raise RowSumError(status, rowsum_status_string(status))


def _marshal(x, y):
    import torch
    code = {torch.float32: ROWSUM_DTYPE_FP32, torch.float16: ROWSUM_DTYPE_FP16,
            torch.bfloat16: ROWSUM_DTYPE_BF16}.get(x.dtype)
    if code is None:
        raise TypeError(f"rowsum: unsupported input dtype {x.dtype}")
    if x.dim() != 2:
        raise ValueError(f"rowsum: x must be 2-D (M, N), got shape {tuple(x.shape)}")
    M, N = x.shape
    for name, t, dt, shape in (("x", x, x.dtype, (M, N)), ("y", y, torch.float32, (M,))):
        if not t.is_cuda or t.device != x.device:
            raise ValueError(f"rowsum: {name} must live in device memory, on x's device")
        if not t.is_contiguous():
            raise ValueError(f"rowsum: {name} must be contiguous")
        if t.dtype != dt:
            raise ValueError(f"rowsum: {name} must have dtype {dt}, got {t.dtype}")
        if tuple(t.shape) != shape:
            raise ValueError(f"rowsum: {name} must have shape {shape}, got {tuple(t.shape)}")
    return M, N, code, torch.cuda.current_stream(x.device).cuda_stream


def rowsum_fwd(x, y=None):
    """Sums over the last dimension of an (M, N) tensor: float32, shape (M,); returns y."""
    return rowsum_fwd_tuned(x, 0, y)


def rowsum_fwd_tuned(x, threads_per_row: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty(x.shape[0], dtype=torch.float32, device=x.device)
    M, N, code, stream = _marshal(x, y)
    with torch.cuda.device(x.device):
        if threads_per_row == 0:
            rc = lib.rowsum_fwd(x.data_ptr(), y.data_ptr(), M, N, code, stream)
        else:
            rc = lib.rowsum_fwd_tuned(x.data_ptr(), y.data_ptr(), M, N, code, stream,
                                      int(threads_per_row))
    _check(rc)
    return y


def rowsum_auto_threads_per_row(N: int, dtype: int) -> int:
    rc = int(load().rowsum_auto_threads_per_row(int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def bind_rowsum_fwd(x, y, threads_per_row: int = 0):
    """Marshals one call once and returns a zero-argument launcher (for launch loops)."""
    import torch
    lib = load()
    M, N, code, stream = _marshal(x, y)
    xp, yp = x.data_ptr(), y.data_ptr()
    if torch.cuda.current_device() != x.device.index:
        raise ValueError("bind_rowsum_fwd: make the tensors' device current before binding")
    if threads_per_row:
        def launch():
            rc = lib.rowsum_fwd_tuned(xp, yp, M, N, code, stream, int(threads_per_row))
            if rc != ROWSUM_OK:
                _check(rc)
    else:
        def launch():
            rc = lib.rowsum_fwd(xp, yp, M, N, code, stream)
            if rc != ROWSUM_OK:
                _check(rc)
    return launch
