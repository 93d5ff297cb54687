"""Thin Python binding of the C ABI in include/rmsnorm.h.

Argument marshalling only: tensors become device pointers, the current torch
stream becomes the hipStream_t, and shapes are checked against what the call
claims so that a kernel is never launched on buffers smaller than its grid
assumes.  Every arithmetic step runs in the HIP kernels.  There is no CPU or
eager fallback: if the library cannot be loaded, or a call fails, this raises.
"""
from __future__ import annotations

import ctypes

from . import build as _build

RMSNORM_DTYPE_FP32 = 0
RMSNORM_DTYPE_FP16 = 1
RMSNORM_DTYPE_BF16 = 2

RMSNORM_OK = 0
RMSNORM_ERR_INVALID_ARG = -1
RMSNORM_ERR_UNSUPPORTED = -2
RMSNORM_ERR_LAUNCH = -3
RMSNORM_ERR_TOO_LARGE = -4

RMSNORM_VARIANT_AUTO = 0
RMSNORM_VARIANT_WAVE = 1
RMSNORM_VARIANT_BLOCK = 2
RMSNORM_VARIANT_GENERIC = 3
RMSNORM_VARIANT_UNALIGNED = 4
RMSNORM_VARIANT_SUBWAVE = 5
RMSNORM_VARIANT_STREAM = 6
RMSNORM_VARIANT_PACKED = 7
RMSNORM_VARIANT_QUEUE = 8

VARIANT_NAMES = {0: "auto", 1: "wave", 2: "block", 3: "generic", 4: "unaligned", 5: "subwave", 6: "stream", 7: "packed",
                 8: "queue"}

_lib = None


class RmsnormError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"rmsnorm: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Loads librmsnorm_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_build.ensure("rmsnorm"))
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    lib.rmsnorm_fwd.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp]
    lib.rmsnorm_fwd.restype = i32
    lib.rmsnorm_fwd_variant.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp, i32]
    lib.rmsnorm_fwd_variant.restype = i32
    lib.rmsnorm_fwd_tuned.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp, i32]
    lib.rmsnorm_fwd_tuned.restype = i32
    lib.rmsnorm_fwd_workspace.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp, vp, i64]
    lib.rmsnorm_fwd_workspace.restype = i32
    lib.rmsnorm_fwd_static.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp]
    lib.rmsnorm_fwd_static.restype = i32
    lib.rmsnorm_fwd_queue_tuned.argtypes = [vp, vp, vp, i64, i64, f32, i32, vp, vp, i64, i32, i32, i32, i32]
    lib.rmsnorm_fwd_queue_tuned.restype = i32
    lib.rmsnorm_workspace_bytes.argtypes = []
    lib.rmsnorm_workspace_bytes.restype = i64
    ip = ctypes.POINTER(ctypes.c_int)
    lib.rmsnorm_queue_plan.argtypes = [i64, i64, i32, ip, ip, ip, ip]
    lib.rmsnorm_queue_plan.restype = i32
    lib.rmsnorm_auto_threads_per_row.argtypes = [i64, i32]
    lib.rmsnorm_auto_threads_per_row.restype = i32
    lib.rmsnorm_auto_threads_for_batch.argtypes = [i64, i64, i32]
    lib.rmsnorm_auto_threads_for_batch.restype = i32
    lib.rmsnorm_select_variant.argtypes = [vp, vp, vp, i64, i64, i32]
    lib.rmsnorm_select_variant.restype = i32
    lib.rmsnorm_unaligned_walk_grid.argtypes = [vp, vp, vp, i64, i64, i32]
    lib.rmsnorm_unaligned_walk_grid.restype = i64
    lib.rmsnorm_wave_max_n.argtypes = [i32]
    lib.rmsnorm_wave_max_n.restype = i64
    lib.rmsnorm_block_max_n.argtypes = [i32]
    lib.rmsnorm_block_max_n.restype = i64
    lib.rmsnorm_unaligned_max_n.argtypes = [i32]
    lib.rmsnorm_unaligned_max_n.restype = i64
    lib.rmsnorm_status_string.argtypes = [i32]
    lib.rmsnorm_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def rmsnorm_status_string(status: int) -> str:
    return load().rmsnorm_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != RMSNORM_OK:
        raise RmsnormError(status, rmsnorm_status_string(status))


def dtype_code(t) -> int:
    import torch
    code = {torch.float32: RMSNORM_DTYPE_FP32, torch.float16: RMSNORM_DTYPE_FP16,
            torch.bfloat16: RMSNORM_DTYPE_BF16}.get(t.dtype)
    if code is None:
        raise TypeError(f"rmsnorm: unsupported tensor dtype {t.dtype}")
    return code


def _marshal(x, w, y):
    """Checks the tensors against the ABI's layout rules; returns (M, N, dtype, stream)."""
    import torch
    if x.dim() != 2:
        raise ValueError(f"rmsnorm: x must be 2-D (M, N), got shape {tuple(x.shape)}")
    M, N = x.shape
    for name, t in (("x", x), ("w", w), ("y", y)):
        if not t.is_cuda:
            raise ValueError(f"rmsnorm: {name} must live in device memory")
        if not t.is_contiguous():
            raise ValueError(f"rmsnorm: {name} must be contiguous (leading dimension N)")
        if t.dtype != x.dtype or t.device != x.device:
            raise ValueError(f"rmsnorm: {name} must match x in dtype and device")
    if tuple(w.shape) != (N,):
        raise ValueError(f"rmsnorm: w must have shape ({N},), got {tuple(w.shape)}")
    if tuple(y.shape) != (M, N):
        raise ValueError(f"rmsnorm: y must have shape {(M, N)}, got {tuple(y.shape)}")
    stream = torch.cuda.current_stream(x.device).cuda_stream
    return M, N, dtype_code(x), stream


def rmsnorm_fwd(x, w, eps: float, y=None):
    """y = x * rsqrt(mean(x^2, -1) + eps) * w on the current stream; returns y."""
    return rmsnorm_fwd_variant(x, w, eps, RMSNORM_VARIANT_AUTO, y)


def rmsnorm_fwd_variant(x, w, eps: float, variant: int, y=None):
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, y)
    with torch.cuda.device(x.device):
        if variant == RMSNORM_VARIANT_AUTO:
            rc = lib.rmsnorm_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps, code, stream)
        else:
            rc = lib.rmsnorm_fwd_variant(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps,
                                         code, stream, int(variant))
    _check(rc)
    return y


def rmsnorm_fwd_tuned(x, w, eps: float, threads_per_row: int, y=None):
    """rmsnorm_fwd with the number of threads sharing one row forced (64 .. 1024)."""
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, y)
    with torch.cuda.device(x.device):
        rc = lib.rmsnorm_fwd_tuned(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps, code,
                                   stream, int(threads_per_row))
    _check(rc)
    return y


def rmsnorm_workspace_bytes() -> int:
    return int(load().rmsnorm_workspace_bytes())


def new_workspace(device):
    """A zero-filled workspace for rmsnorm_fwd_workspace on `device` (the caller owns it)."""
    import torch
    return torch.zeros(rmsnorm_workspace_bytes() // 4, dtype=torch.int32, device=device)


def _workspace_args(workspace, x):
    if not (workspace.is_cuda and workspace.is_contiguous() and workspace.device == x.device):
        raise ValueError("rmsnorm: the workspace must be a contiguous tensor on the device of x")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def rmsnorm_fwd_workspace(x, w, eps: float, workspace, y=None):
    """The work-queue kernel on the caller's workspace (see new_workspace); returns y."""
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, y)
    wp, wbytes = _workspace_args(workspace, x)
    with torch.cuda.device(x.device):
        rc = lib.rmsnorm_fwd_workspace(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps, code,
                                       stream, wp, wbytes)
    _check(rc)
    return y


def rmsnorm_fwd_static(x, w, eps: float, y=None):
    """The work-queue kernel on the library's own fixed counters (allocates nothing; calls that
    overlap on one GPU race); returns y."""
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, y)
    with torch.cuda.device(x.device):
        rc = lib.rmsnorm_fwd_static(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps, code, stream)
    _check(rc)
    return y


def rmsnorm_fwd_queue_tuned(x, w, eps: float, workspace, grid: int, shards: int, block_rows: int,
                            prefetch: bool, y=None):
    """rmsnorm_fwd_workspace with the launch shape forced."""
    import torch
    lib = load()
    if y is None:
        y = torch.empty_like(x)
    M, N, code, stream = _marshal(x, w, y)
    wp, wbytes = _workspace_args(workspace, x)
    with torch.cuda.device(x.device):
        rc = lib.rmsnorm_fwd_queue_tuned(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, eps, code,
                                         stream, wp, wbytes, int(grid), int(shards), int(block_rows),
                                         1 if prefetch else 0)
    _check(rc)
    return y


def rmsnorm_queue_plan(M: int, N: int, dtype: int):
    """(auto_takes_it, grid, shards, block_rows, prefetch) of RMSNORM_VARIANT_QUEUE for M x N on
    the current device; raises if the variant cannot run such rows."""
    out = [ctypes.c_int(0) for _ in range(4)]
    rc = int(load().rmsnorm_queue_plan(int(M), int(N), int(dtype), *[ctypes.byref(o) for o in out]))
    if rc < 0:
        _check(rc)
    return (rc == 1, out[0].value, out[1].value, out[2].value, bool(out[3].value))


def rmsnorm_auto_threads_per_row(N: int, dtype: int) -> int:
    rc = int(load().rmsnorm_auto_threads_per_row(int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def rmsnorm_auto_threads_for_batch(M: int, N: int, dtype: int) -> int:
    rc = int(load().rmsnorm_auto_threads_for_batch(int(M), int(N), int(dtype)))
    if rc < 0:
        _check(rc)
    return rc


def rmsnorm_select_variant(x, w, y) -> int:
    M, N, code, _ = _marshal(x, w, y)
    rc = load().rmsnorm_select_variant(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, code)
    if rc < 0:
        _check(rc)
    return rc


def rmsnorm_unaligned_walk_grid(x, w, y) -> int:
    M, N, code, _ = _marshal(x, w, y)
    rc = int(load().rmsnorm_unaligned_walk_grid(x.data_ptr(), w.data_ptr(), y.data_ptr(), M, N, code))
    if rc < 0:
        _check(rc)
    return rc


def rmsnorm_wave_max_n(dtype: int) -> int:
    return int(load().rmsnorm_wave_max_n(int(dtype)))


def rmsnorm_block_max_n(dtype: int) -> int:
    return int(load().rmsnorm_block_max_n(int(dtype)))


def rmsnorm_unaligned_max_n(dtype: int) -> int:
    return int(load().rmsnorm_unaligned_max_n(int(dtype)))


def bind_rmsnorm_fwd(x, w, y, eps: float, variant: int = RMSNORM_VARIANT_AUTO,
                     threads_per_row: int = 0):
    """Marshals one call once and returns a zero-argument launcher for it.

    For launch loops (benchmarks, serving steps) where the per-call tensor checks
    of rmsnorm_fwd would dominate the host side.  The launcher enqueues on the
    stream that was current when it was bound and raises on a non-zero status.
    The tensors must outlive every use of the launcher.
    """
    import torch
    lib = load()
    M, N, code, stream = _marshal(x, w, y)
    xp, wp, yp = x.data_ptr(), w.data_ptr(), y.data_ptr()
    eps_c = ctypes.c_float(eps)
    if threads_per_row:
        fn, last = lib.rmsnorm_fwd_tuned, int(threads_per_row)
    else:
        fn, last = lib.rmsnorm_fwd_variant, int(variant)
    if torch.cuda.current_device() != x.device.index:
        raise ValueError("bind_rmsnorm_fwd: make the tensors' device current before binding")

    def launch():
        rc = fn(xp, wp, yp, M, N, eps_c, code, stream, last)
        if rc != RMSNORM_OK:
            _check(rc)

    return launch
