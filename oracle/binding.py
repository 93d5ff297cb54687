"""ctypes access to the C++ oracle (host memory only).  Test infrastructure."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

FP32, FP16, BF16 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rmsnorm_oracle.cpp")
_LIB = os.path.join(_HERE, "librmsnorm_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compiles the oracle with the host compiler.  No GPU toolchain involved."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # RMSNORM_ORACLE_LIB lets the mutation test (tests/test_oracle_mutants.py) point the
        # pins at a deliberately broken build of the oracle; nothing else sets it.
        lib = ctypes.CDLL(os.environ.get("RMSNORM_ORACLE_LIB") or build(force=False))
        vp, i64, dbl, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_int
        lib.rmsnorm_oracle.argtypes = [vp, vp, vp, i64, i64, dbl, i32, i32]
        lib.rmsnorm_oracle.restype = i32
        lib.rmsnorm_oracle_rstd.argtypes = [vp, vp, i64, i64, dbl, i32]
        lib.rmsnorm_oracle_rstd.restype = i32
        lib.rmsnorm_oracle_decode.argtypes = [vp, vp, i64, i32]
        lib.rmsnorm_oracle_decode.restype = i32
        lib.rmsnorm_oracle_encode.argtypes = [vp, vp, i64, i32]
        lib.rmsnorm_oracle_encode.restype = i32
        lib.rmsnorm_oracle_hardware_threads.argtypes = []
        lib.rmsnorm_oracle_hardware_threads.restype = i32
        _lib = lib
    return _lib


def _storage_dtype(dtype: int):
    if dtype == FP32:
        return np.float32
    if dtype in (FP16, BF16):
        return np.uint16
    raise ValueError(f"unknown dtype code {dtype}")


def _as_storage(a, dtype: int) -> np.ndarray:
    a = np.asarray(a)
    want = _storage_dtype(dtype)
    if a.dtype != want:
        raise TypeError(f"dtype code {dtype} wants a {np.dtype(want).name} array "
                        f"(bit patterns for 16-bit types), got {a.dtype}")
    return np.ascontiguousarray(a)


def eps_as_passed(eps: float) -> float:
    """The GPU entry point takes eps as a float; the oracle uses that float, widened."""
    return float(np.float32(eps))


def rmsnorm_oracle(x, w, eps: float, dtype: int, nthreads: int = 0) -> np.ndarray:
    """y = rmsnorm(x, w) for an (M, N) x and an (N,) w in storage form; returns storage form."""
    x = _as_storage(x, dtype)
    w = _as_storage(w, dtype)
    if x.ndim != 2 or w.ndim != 1 or w.shape[0] != x.shape[1]:
        raise ValueError(f"shape mismatch: x {x.shape}, w {w.shape}")
    M, N = x.shape
    y = np.empty_like(x)
    rc = _load().rmsnorm_oracle(x.ctypes.data, w.ctypes.data, y.ctypes.data, M, N,
                                eps_as_passed(eps), dtype, nthreads)
    if rc != 0:
        raise ValueError(f"rmsnorm_oracle rejected its arguments (rc={rc})")
    return y


def rmsnorm_oracle_rstd(x, eps: float, dtype: int) -> np.ndarray:
    x = _as_storage(x, dtype)
    M, N = x.shape
    r = np.empty(M, dtype=np.float64)
    rc = _load().rmsnorm_oracle_rstd(x.ctypes.data, r.ctypes.data, M, N, eps_as_passed(eps), dtype)
    if rc != 0:
        raise ValueError(f"rmsnorm_oracle_rstd rejected its arguments (rc={rc})")
    return r


def decode(bits, dtype: int) -> np.ndarray:
    b = _as_storage(bits, dtype)
    out = np.empty(b.shape, dtype=np.float64)
    rc = _load().rmsnorm_oracle_decode(b.ctypes.data, out.ctypes.data, b.size, dtype)
    if rc != 0:
        raise ValueError("decode failed")
    return out


def encode(values, dtype: int) -> np.ndarray:
    v = np.ascontiguousarray(np.asarray(values, dtype=np.float64))
    out = np.empty(v.shape, dtype=_storage_dtype(dtype))
    rc = _load().rmsnorm_oracle_encode(v.ctypes.data, out.ctypes.data, v.size, dtype)
    if rc != 0:
        raise ValueError("encode failed")
    return out


def hardware_threads() -> int:
    return int(_load().rmsnorm_oracle_hardware_threads())
