"""Thin Python binding of the C ABI in include/softmax.h (argument marshalling only).

Same rules as binding.py: tensors become device pointers, the current torch
stream becomes the hipStream_t, shapes are checked against what the call claims,
every arithmetic step runs in the HIP kernels, and there is no CPU or eager
fallback: a missing library or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

SOFTMAX_DTYPE_FP32 = 0
SOFTMAX_DTYPE_FP16 = 1
SOFTMAX_DTYPE_BF16 = 2

SOFTMAX_OK = 0
SOFTMAX_ERR_INVALID_ARG = -1
SOFTMAX_ERR_UNSUPPORTED = -2
SOFTMAX_ERR_LAUNCH = -3

SOFTMAX_VARIANT_AUTO = 0
SOFTMAX_VARIANT_WAVE = 1
SOFTMAX_VARIANT_BLOCK = 2
SOFTMAX_VARIANT_GENERIC = 3
SOFTMAX_VARIANT_SUBWAVE = 4
SOFTMAX_VARIANT_UNALIGNED = 5
SOFTMAX_VARIANT_STREAM = 6
SOFTMAX_VARIANT_PACKED = 7

VARIANT_NAMES = {0: "auto", 1: "wave", 2: "block", 3: "generic", 4: "subwave", 5: "unaligned", 6: "stream", 7: "packed"}

_lib = None


class SoftmaxError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"softmax: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.SOFTMAX_LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libsoftmax_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure("softmax"))
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.softmax_fwd.argtypes = [vp, vp, i64, i64, i32, vp]
    lib.softmax_fwd.restype = i32
    lib.softmax_fwd_variant.argtypes = [vp, vp, i64, i64, i32, vp, i32]
    lib.softmax_fwd_variant.restype = i32
    lib.softmax_fwd_tuned.argtypes = [vp, vp, i64, i64, i32, vp, i32]
    lib.softmax_fwd_tuned.restype = i32
    lib.softmax_auto_threads_per_row.argtypes = [i64, i32]
    lib.softmax_auto_threads_per_row.restype = i32
    lib.softmax_register_max_n.argtypes = [i32]
    lib.softmax_register_max_n.restype = i64
    lib.softmax_status_string.argtypes = [i32]
    lib.softmax_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def softmax_status_string(status: int) -> str:
    return load().softmax_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != SOFTMAX_OK:
        raise SoftmaxError(status, softmax_status_string(status))


def _marshal(x, y):
    import torch
    code = {torch.float32: SOFTMAX_DTYPE_FP32, torch.float16: SOFTMAX_DTYPE_FP16,
            torch.bfloat16: SOFTMAX_DTYPE_BF16}.get(x.dtype)
    if code is None:
        raise TypeError(f"softmax: unsupported tensor dtype {x.dtype}")
    if x.dim() != 2:
        raise ValueError(f"softmax: x must be 2-D (M, N), got shape {tuple(x.shape)}")
    for name, t in (("x", x), ("y", y)):
        if not t.is_cuda:
            raise ValueError(f"softmax: {name} must live in device memory")
        if not t.is_contiguous():
            raise ValueError(f"softmax: {name} must be contiguous (leading dimension N)")
        if t.dtype != x.dtype or t.device != x.device:
            raise ValueError(f"softmax: {name} must match x in dtype and device")
    if tuple(y.shape) != tuple(x.shape):
        raise ValueError(f"softmax: y must have shape {tuple(x.shape)}, got {tuple(y.shape)}")
    M, N = x.shape
    return M, N, code, torch.cuda.current_stream(x.device).cuda_stream


def softmax_fwd(x, y=None):
    """y = softmax(x, dim=-1) on the current stream; returns y."""
    return softmax_fwd_variant(x, SOFTMAX_VARIANT_AUTO, y)


def softmax_fwd_variant(x, variant: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, y)
    with torch.cuda.device(x.device):
        if variant == SOFTMAX_VARIANT_AUTO:
            rc = lib.softmax_fwd(x.data_ptr(), y.data_ptr(), M, N, code, stream)
        else:
            rc = lib.softmax_fwd_variant(x.data_ptr(), y.data_ptr(), M, N, code, stream, int(variant))
    _check(rc)
    return y


def softmax_fwd_tuned(x, threads_per_row: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, y)
    with torch.cuda.device(x.device):
        rc = lib.softmax_fwd_tuned(x.data_ptr(), y.data_ptr(), M, N, code, stream,
                                   int(threads_per_row))
    _check(rc)
    return y


def softmax_auto_threads_per_row(N: int, dtype: int) -> int:
    rc = int(load().softmax_auto_threads_per_row(int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def softmax_register_max_n(dtype: int) -> int:
    return int(load().softmax_register_max_n(int(dtype)))


def bind_softmax_fwd(x, y, variant: int = SOFTMAX_VARIANT_AUTO, threads_per_row: int = 0):
    """Marshals one call once and returns a zero-argument launcher (for launch loops)."""
    import torch
    lib = load()
    M, N, code, stream = _marshal(x, y)
    xp, yp = x.data_ptr(), y.data_ptr()
    if threads_per_row:
        fn, last = lib.softmax_fwd_tuned, int(threads_per_row)
    else:
        fn, last = lib.softmax_fwd_variant, int(variant)
    if torch.cuda.current_device() != x.device.index:
        raise ValueError("bind_softmax_fwd: make the tensors' device current before binding")

    def launch():
        rc = fn(xp, yp, M, N, code, stream, last)
        if rc != SOFTMAX_OK:
            _check(rc)

    return launch
