"""Thin Python binding of the C ABI in include/layernorm.h (argument marshalling only).

Same rules as binding.py: tensors become device pointers, the current torch
stream becomes the hipStream_t, shapes are checked against what the call claims,
every arithmetic step runs in the HIP kernels, and there is no CPU or eager
fallback: a missing library or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

LAYERNORM_DTYPE_FP32 = 0
LAYERNORM_DTYPE_FP16 = 1
LAYERNORM_DTYPE_BF16 = 2

LAYERNORM_OK = 0
LAYERNORM_ERR_INVALID_ARG = -1
LAYERNORM_ERR_UNSUPPORTED = -2
LAYERNORM_ERR_LAUNCH = -3

LAYERNORM_VARIANT_AUTO = 0
LAYERNORM_VARIANT_WAVE = 1
LAYERNORM_VARIANT_BLOCK = 2
LAYERNORM_VARIANT_GENERIC = 3
LAYERNORM_VARIANT_SUBWAVE = 4
LAYERNORM_VARIANT_UNALIGNED = 5
LAYERNORM_VARIANT_STREAM = 6
LAYERNORM_VARIANT_PACKED = 7
LAYERNORM_VARIANT_QUEUE = 8

VARIANT_NAMES = {0: "auto", 1: "wave", 2: "block", 3: "generic", 4: "subwave", 5: "unaligned", 6: "stream", 7: "packed",
                 8: "queue"}

_lib = None


class LayerNormError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"layernorm: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.LAYERNORM_LIB_PATH


def load() -> ctypes.CDLL:
    """Loads liblayernorm_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure("layernorm"))
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    f32 = ctypes.c_float
    lib.layernorm_fwd.argtypes = [vp, vp, vp, vp, i64, i64, f32, i32, vp]
    lib.layernorm_fwd.restype = i32
    lib.layernorm_fwd_variant.argtypes = [vp, vp, vp, vp, i64, i64, f32, i32, vp, i32]
    lib.layernorm_fwd_variant.restype = i32
    lib.layernorm_fwd_tuned.argtypes = [vp, vp, vp, vp, i64, i64, f32, i32, vp, i32]
    lib.layernorm_fwd_tuned.restype = i32
    lib.layernorm_auto_threads_per_row.argtypes = [i64, i32]
    lib.layernorm_auto_threads_per_row.restype = i32
    lib.layernorm_unaligned_walk_grid.argtypes = [vp, vp, vp, vp, i64, i64, i32]
    lib.layernorm_unaligned_walk_grid.restype = i64
    ip = ctypes.POINTER(ctypes.c_int)
    lib.layernorm_queue_plan.argtypes = [i64, i64, i32, ip, ip, ip, ip]
    lib.layernorm_queue_plan.restype = i32
    lib.layernorm_register_max_n.argtypes = [i32]
    lib.layernorm_register_max_n.restype = i64
    lib.layernorm_status_string.argtypes = [i32]
    lib.layernorm_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def layernorm_status_string(status: int) -> str:
    return load().layernorm_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != LAYERNORM_OK:
        raise LayerNormError(status, layernorm_status_string(status))


def _marshal(x, w, b, y):
    import torch
    code = {torch.float32: LAYERNORM_DTYPE_FP32, torch.float16: LAYERNORM_DTYPE_FP16,
            torch.bfloat16: LAYERNORM_DTYPE_BF16}.get(x.dtype)
    if code is None:
        raise TypeError(f"layernorm: unsupported tensor dtype {x.dtype}")
    if x.dim() != 2:
        raise ValueError(f"layernorm: x must be 2-D (M, N), got shape {tuple(x.shape)}")
    M, N = x.shape
    named = [("x", x), ("w", w), ("y", y)] + ([("b", b)] if b is not None else [])
    for name, t in named:
        if not t.is_cuda:
            raise ValueError(f"layernorm: {name} must live in device memory")
        if not t.is_contiguous():
            raise ValueError(f"layernorm: {name} must be contiguous (leading dimension N)")
        if t.dtype != x.dtype or t.device != x.device:
            raise ValueError(f"layernorm: {name} must match x in dtype and device")
    if tuple(w.shape) != (N,) or (b is not None and tuple(b.shape) != (N,)):
        raise ValueError(f"layernorm: w and b must have shape ({N},)")
    if tuple(y.shape) != (M, N):
        raise ValueError(f"layernorm: y must have shape {(M, N)}, got {tuple(y.shape)}")
    return M, N, code, torch.cuda.current_stream(x.device).cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def layernorm_fwd(x, w, b, eps: float, y=None):
    """y = layer_norm(x, w, b) over the last dimension on the current stream (b may be None)."""
    return layernorm_fwd_variant(x, w, b, eps, LAYERNORM_VARIANT_AUTO, y)


def layernorm_fwd_variant(x, w, b, eps: float, variant: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, b, y)
    with torch.cuda.device(x.device):
        if variant == LAYERNORM_VARIANT_AUTO:
            rc = lib.layernorm_fwd(x.data_ptr(), w.data_ptr(), _ptr(b), y.data_ptr(), M, N, eps,
                                   code, stream)
        else:
            rc = lib.layernorm_fwd_variant(x.data_ptr(), w.data_ptr(), _ptr(b), y.data_ptr(), M, N,
                                           eps, code, stream, int(variant))
    _check(rc)
    return y


def layernorm_fwd_tuned(x, w, b, eps: float, threads_per_row: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, b, y)
    with torch.cuda.device(x.device):
        rc = lib.layernorm_fwd_tuned(x.data_ptr(), w.data_ptr(), _ptr(b), y.data_ptr(), M, N, eps,
                                     code, stream, int(threads_per_row))
    _check(rc)
    return y


def layernorm_auto_threads_per_row(N: int, dtype: int) -> int:
    rc = int(load().layernorm_auto_threads_per_row(int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def layernorm_unaligned_walk_grid(x, w, b, y) -> int:
    M, N, code, _ = _marshal(x, w, b, y)
    rc = int(load().layernorm_unaligned_walk_grid(x.data_ptr(), w.data_ptr(), _ptr(b), y.data_ptr(), M, N, code))
    if rc < 0:
        _check(rc)
    return rc


def layernorm_queue_plan(M: int, N: int, dtype: int):
    """(auto_takes_it, threads, grid, shards, block_rows) of LAYERNORM_VARIANT_QUEUE for M x N on the
    current device; raises if the variant cannot run such rows."""
    out = [ctypes.c_int(0) for _ in range(4)]
    rc = int(load().layernorm_queue_plan(int(M), int(N), int(dtype), *[ctypes.byref(o) for o in out]))
    if rc < 0:
        _check(rc)
    return (rc == 1, out[0].value, out[1].value, out[2].value, out[3].value)


def layernorm_register_max_n(dtype: int) -> int:
    return int(load().layernorm_register_max_n(int(dtype)))


def bind_layernorm_fwd(x, w, b, y, eps: float, variant: int = LAYERNORM_VARIANT_AUTO,
                       threads_per_row: int = 0):
    """Marshals one call once and returns a zero-argument launcher (for launch loops)."""
    import torch
    lib = load()
    M, N, code, stream = _marshal(x, w, b, y)
    xp, wp, bp, yp = x.data_ptr(), w.data_ptr(), _ptr(b), y.data_ptr()
    eps_c = ctypes.c_float(eps)
    if threads_per_row:
        fn, last = lib.layernorm_fwd_tuned, int(threads_per_row)
    else:
        fn, last = lib.layernorm_fwd_variant, int(variant)
    if torch.cuda.current_device() != x.device.index:
        raise ValueError("bind_layernorm_fwd: make the tensors' device current before binding")

    def launch():
        rc = fn(xp, wp, bp, yp, M, N, eps_c, code, stream, last)
        if rc != LAYERNORM_OK:
            _check(rc)

    return launch
