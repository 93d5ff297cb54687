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
_SOFTMAX_SRC = os.path.join(_HERE, "softmax_oracle.cpp")
_SOFTMAX_LIB = os.path.join(_HERE, "libsoftmax_oracle.so")
_LAYERNORM_SRC = os.path.join(_HERE, "layernorm_oracle.cpp")
_LAYERNORM_LIB = os.path.join(_HERE, "liblayernorm_oracle.so")
_CE_SRC = os.path.join(_HERE, "crossentropy_oracle.cpp")
_CE_LIB = os.path.join(_HERE, "libcrossentropy_oracle.so")
_ROWSUM_SRC = os.path.join(_HERE, "rowsum_oracle.cpp")
_ROWSUM_LIB = os.path.join(_HERE, "librowsum_oracle.so")
_lib = None
_rowsum_lib = None
_softmax_lib = None
_layernorm_lib = None
_ce_lib = None


def _compile(src: str, lib: str, force: bool) -> str:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread",
               "-Wall", "-Wextra", "-o", lib, src]
        subprocess.run(cmd, check=True)
    return lib


def build(force: bool = True) -> str:
    """Compiles the oracles with the host compiler.  No GPU toolchain involved."""
    _compile(_SOFTMAX_SRC, _SOFTMAX_LIB, force)
    _compile(_LAYERNORM_SRC, _LAYERNORM_LIB, force)
    _compile(_CE_SRC, _CE_LIB, force)
    _compile(_ROWSUM_SRC, _ROWSUM_LIB, force)
    return _compile(_SRC, _LIB, force)


def _load():
    global _lib
    if _lib is None:
        # RMSNORM_ORACLE_LIB lets the mutation test (tests/test_oracle_mutants.py) point the
        # pins at a deliberately broken build of the oracle; nothing else sets it.
        lib = ctypes.CDLL(os.environ.get("RMSNORM_ORACLE_LIB") or _compile(_SRC, _LIB, False))
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


# ------------------------------------------------------------------ row softmax

def _load_softmax():
    global _softmax_lib
    if _softmax_lib is None:
        # SOFTMAX_ORACLE_LIB: same hook as RMSNORM_ORACLE_LIB, for the softmax mutation test.
        lib = ctypes.CDLL(os.environ.get("SOFTMAX_ORACLE_LIB")
                          or _compile(_SOFTMAX_SRC, _SOFTMAX_LIB, False))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.softmax_oracle.argtypes = [vp, vp, i64, i64, i32, i32]
        lib.softmax_oracle.restype = i32
        _softmax_lib = lib
    return _softmax_lib


def softmax_oracle(x, dtype: int, nthreads: int = 0) -> np.ndarray:
    """Row softmax of an (M, N) x in storage form; returns storage form."""
    x = _as_storage(x, dtype)
    if x.ndim != 2:
        raise ValueError(f"x must be 2-D, got shape {x.shape}")
    M, N = x.shape
    y = np.empty_like(x)
    rc = _load_softmax().softmax_oracle(x.ctypes.data, y.ctypes.data, M, N, dtype, nthreads)
    if rc != 0:
        raise ValueError(f"softmax_oracle rejected its arguments (rc={rc})")
    return y


# ------------------------------------------------------------------ row LayerNorm

def _load_layernorm():
    global _layernorm_lib
    if _layernorm_lib is None:
        # LAYERNORM_ORACLE_LIB: the mutation test's hook, as for the other oracles.
        lib = ctypes.CDLL(os.environ.get("LAYERNORM_ORACLE_LIB")
                          or _compile(_LAYERNORM_SRC, _LAYERNORM_LIB, False))
        vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.layernorm_oracle.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, dbl, i32, i32]
        lib.layernorm_oracle.restype = i32
        _layernorm_lib = lib
    return _layernorm_lib


def layernorm_oracle(x, w, b, eps: float, dtype: int, nthreads: int = 0, stats: bool = False):
    """LayerNorm of an (M, N) x with (N,) w and optional (N,) b (None = no bias), storage form.

    Returns y, or (y, mean, rstd) with the fp64 row statistics when stats is true."""
    x = _as_storage(x, dtype)
    w = _as_storage(w, dtype)
    if b is not None:
        b = _as_storage(b, dtype)
    if x.ndim != 2 or w.shape != (x.shape[1],) or (b is not None and b.shape != w.shape):
        raise ValueError(f"shape mismatch: x {x.shape}, w {w.shape}, b {None if b is None else b.shape}")
    M, N = x.shape
    y = np.empty_like(x)
    mean = np.empty(M, dtype=np.float64) if stats else None
    rstd = np.empty(M, dtype=np.float64) if stats else None
    rc = _load_layernorm().layernorm_oracle(
        x.ctypes.data, w.ctypes.data, None if b is None else b.ctypes.data, y.ctypes.data,
        None if mean is None else mean.ctypes.data, None if rstd is None else rstd.ctypes.data,
        M, N, eps_as_passed(eps), dtype, nthreads)
    if rc != 0:
        raise ValueError(f"layernorm_oracle rejected its arguments (rc={rc})")
    return (y, mean, rstd) if stats else y


# ------------------------------------------------------------------ row cross-entropy

def _load_crossentropy():
    global _ce_lib
    if _ce_lib is None:
        # CROSSENTROPY_ORACLE_LIB: the mutation test's hook, as for the other oracles.
        lib = ctypes.CDLL(os.environ.get("CROSSENTROPY_ORACLE_LIB") or _compile(_CE_SRC, _CE_LIB, False))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.crossentropy_oracle.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32]
        lib.crossentropy_oracle.restype = i32
        _ce_lib = lib
    return _ce_lib


def crossentropy_oracle(x, target, dtype: int, nthreads: int = 0, with_lse: bool = False):
    """Per-row loss (float32, M entries) of (M, N) logits in storage form and int64 targets.

    Returns loss, or (loss, lse) with the fp64 log-sum-exp of each row when with_lse is true."""
    x = _as_storage(x, dtype)
    target = np.ascontiguousarray(np.asarray(target))
    if target.dtype != np.int64:
        raise TypeError(f"targets must be int64, got {target.dtype}")
    if x.ndim != 2 or target.shape != (x.shape[0],):
        raise ValueError(f"shape mismatch: x {x.shape}, target {target.shape}")
    M, N = x.shape
    loss = np.empty(M, dtype=np.float32)
    lse = np.empty(M, dtype=np.float64) if with_lse else None
    rc = _load_crossentropy().crossentropy_oracle(
        x.ctypes.data, target.ctypes.data, loss.ctypes.data,
        None if lse is None else lse.ctypes.data, M, N, dtype, nthreads)
    if rc != 0:
        raise ValueError(f"crossentropy_oracle rejected its arguments (rc={rc})")
    return (loss, lse) if with_lse else loss


# ------------------------------------------------------------------ row sum

def _load_rowsum():
    global _rowsum_lib
    if _rowsum_lib is None:
        # ROWSUM_ORACLE_LIB: the mutation test's hook, as for the other oracles.
        lib = ctypes.CDLL(os.environ.get("ROWSUM_ORACLE_LIB") or _compile(_ROWSUM_SRC, _ROWSUM_LIB, False))
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.rowsum_oracle.argtypes = [vp, vp, vp, i64, i64, i32, i32]
        lib.rowsum_oracle.restype = i32
        _rowsum_lib = lib
    return _rowsum_lib


def rowsum_oracle(x, dtype: int, nthreads: int = 0, with_abs: bool = False):
    """Sum over the last dimension of an (M, N) x in storage form: float32, M entries.

    Returns y, or (y, abs_sum) with the fp64 sums of absolute values when with_abs is true."""
    x = _as_storage(x, dtype)
    if x.ndim != 2:
        raise ValueError(f"x must be 2-D, got shape {x.shape}")
    M, N = x.shape
    y = np.empty(M, dtype=np.float32)
    a = np.empty(M, dtype=np.float64) if with_abs else None
    rc = _load_rowsum().rowsum_oracle(x.ctypes.data, y.ctypes.data,
                                      None if a is None else a.ctypes.data, M, N, dtype, nthreads)
    if rc != 0:
        raise ValueError(f"rowsum_oracle rejected its arguments (rc={rc})")
    return (y, a) if with_abs else y
