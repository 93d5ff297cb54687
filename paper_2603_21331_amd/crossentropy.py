"""Thin Python binding of the C ABI in include/crossentropy.h (argument marshalling only).

Same rules as binding.py: tensors become device pointers, the current torch stream becomes
the hipStream_t, shapes and dtypes are checked against what the call claims, every arithmetic
step runs in the HIP kernel, and there is no CPU or eager fallback.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

CROSSENTROPY_DTYPE_FP32 = 0
CROSSENTROPY_DTYPE_FP16 = 1
CROSSENTROPY_DTYPE_BF16 = 2

CROSSENTROPY_OK = 0
CROSSENTROPY_ERR_INVALID_ARG = -1
CROSSENTROPY_ERR_UNSUPPORTED = -2
CROSSENTROPY_ERR_LAUNCH = -3

_lib = None


class CrossEntropyError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"crossentropy: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.CROSSENTROPY_LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libcrossentropy_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure("crossentropy"))
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.crossentropy_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp]
    lib.crossentropy_fwd.restype = i32
    lib.crossentropy_fwd_tuned.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, i32]
    lib.crossentropy_fwd_tuned.restype = i32
    lib.crossentropy_auto_threads_per_row.argtypes = [i64, i32]
    lib.crossentropy_auto_threads_per_row.restype = i32
    lib.crossentropy_status_string.argtypes = [i32]
    lib.crossentropy_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def crossentropy_status_string(status: int) -> str:
    return load().crossentropy_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != CROSSENTROPY_OK:
        raise CrossEntropyError(status, crossentropy_status_string(status))


def _marshal(x, target, loss, lse):
    import torch
    code = {torch.float32: CROSSENTROPY_DTYPE_FP32, torch.float16: CROSSENTROPY_DTYPE_FP16,
            torch.bfloat16: CROSSENTROPY_DTYPE_BF16}.get(x.dtype)
    if code is None:
        raise TypeError(f"crossentropy: unsupported logits dtype {x.dtype}")
    if x.dim() != 2:
        raise ValueError(f"crossentropy: x must be 2-D (M, N), got shape {tuple(x.shape)}")
    M, N = x.shape
    named = [("x", x, x.dtype, (M, N)), ("target", target, torch.int64, (M,)),
             ("loss", loss, torch.float32, (M,))]
    if lse is not None:
        named.append(("lse", lse, torch.float32, (M,)))
    for name, t, dt, shape in named:
        if not t.is_cuda or t.device != x.device:
            raise ValueError(f"crossentropy: {name} must live in device memory, on x's device")
        if not t.is_contiguous():
            raise ValueError(f"crossentropy: {name} must be contiguous")
        if t.dtype != dt:
            raise ValueError(f"crossentropy: {name} must have dtype {dt}, got {t.dtype}")
        if tuple(t.shape) != shape:
            raise ValueError(f"crossentropy: {name} must have shape {shape}, got {tuple(t.shape)}")
    return M, N, code, torch.cuda.current_stream(x.device).cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def crossentropy_fwd(x, target, loss=None, lse=None):
    """Per-row loss (float32, shape (M,)) of (M, N) logits and int64 targets; returns loss.
    Pass an (M,) float32 tensor as lse to also receive the log-sum-exp of each row."""
    return crossentropy_fwd_tuned(x, target, 0, loss, lse)


def crossentropy_fwd_tuned(x, target, threads_per_row: int, loss=None, lse=None):
    import torch
    lib = load()
    if loss is None:
        loss = torch.empty(x.shape[0], dtype=torch.float32, device=x.device)
    M, N, code, stream = _marshal(x, target, loss, lse)
    with torch.cuda.device(x.device):
        if threads_per_row == 0:
            rc = lib.crossentropy_fwd(x.data_ptr(), target.data_ptr(), loss.data_ptr(), _ptr(lse),
                                      M, N, code, stream)
        else:
            rc = lib.crossentropy_fwd_tuned(x.data_ptr(), target.data_ptr(), loss.data_ptr(),
                                            _ptr(lse), M, N, code, stream, int(threads_per_row))
    _check(rc)
    return loss


def crossentropy_auto_threads_per_row(N: int, dtype: int) -> int:
    rc = int(load().crossentropy_auto_threads_per_row(int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def bind_crossentropy_fwd(x, target, loss, lse=None, threads_per_row: int = 0):
    """Marshals one call once and returns a zero-argument launcher (for launch loops)."""
    import torch
    lib = load()
    M, N, code, stream = _marshal(x, target, loss, lse)
    xp, tp, lp, sp = x.data_ptr(), target.data_ptr(), loss.data_ptr(), _ptr(lse)
    if torch.cuda.current_device() != x.device.index:
        raise ValueError("bind_crossentropy_fwd: make the tensors' device current before binding")
    if threads_per_row:
        def launch():
            rc = lib.crossentropy_fwd_tuned(xp, tp, lp, sp, M, N, code, stream, int(threads_per_row))
            if rc != CROSSENTROPY_OK:
                _check(rc)
    else:
        def launch():
            rc = lib.crossentropy_fwd(xp, tp, lp, sp, M, N, code, stream)
            if rc != CROSSENTROPY_OK:
                _check(rc)
    return launch
