"""Thin Python binding of the C ABI in include/measure.h (argument marshalling only): the
streaming copy of known traffic that the benchmark uses to scale the hardware counters and as
the practical bandwidth ceiling."""
from __future__ import annotations

import ctypes

from . import build as _build

MEASURE_OK = 0
MEASURE_ERR_INVALID_ARG = -1
MEASURE_ERR_LAUNCH = -3

_lib = None


class MeasureError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"measure: {text} (status {status})")
        self.status = status


def library_path() -> str:
    return _build.MEASURE_LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libmeasure_hip.so (rebuilt first if it is missing or does not match its sources)."""
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.ensure("measure"))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.measure_copy.argtypes = [vp, vp, i64, vp]
        lib.measure_copy.restype = i32
        lib.measure_staged_copy.argtypes = [vp, vp, i64, vp]
        lib.measure_staged_copy.restype = i32
        lib.measure_status_string.argtypes = [i32]
        lib.measure_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def measure_status_string(status: int) -> str:
    return load().measure_status_string(int(status)).decode()


def measure_copy(src, dst) -> None:
    """dst <- src, byte for byte, with the library's streaming copy kernel, on the current stream."""
    _copy("measure_copy", src, dst)


def measure_staged_copy(src, dst) -> None:
    """dst <- src through LDS tiles (the staging of the short-row kernels), on the current stream."""
    _copy("measure_staged_copy", src, dst)


def _copy(entry: str, src, dst) -> None:
    import torch
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError(f"{entry}: contiguous device tensors required")
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError(f"{entry}: size mismatch")
    stream = torch.cuda.current_stream(src.device).cuda_stream
    with torch.cuda.device(src.device):
        rc = getattr(load(), entry)(src.data_ptr(), dst.data_ptr(), nbytes, stream)
    if rc != MEASURE_OK:
        raise MeasureError(rc, measure_status_string(rc))
