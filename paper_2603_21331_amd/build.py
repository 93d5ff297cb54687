"""Builds the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "librmsnorm_hip.so")
SOFTMAX_LIB_PATH = os.path.join(_HERE, "libsoftmax_hip.so")

SOURCES = ["rmsnorm_api.hip"]
HEADERS = ["rmsnorm_kernels.h", "vec_io.h", "wave_reduce.h", "packed_rows.h", "launch_util.h"]
LAYERNORM_LIB_PATH = os.path.join(_HERE, "liblayernorm_hip.so")
LAYERNORM_SOURCES = ["layernorm_api.hip"]
LAYERNORM_HEADERS = ["layernorm_kernels.h", "vec_io.h", "wave_reduce.h", "packed_rows.h", "launch_util.h"]
CROSSENTROPY_LIB_PATH = os.path.join(_HERE, "libcrossentropy_hip.so")
CROSSENTROPY_SOURCES = ["crossentropy_api.hip"]
CROSSENTROPY_HEADERS = ["crossentropy_kernels.h", "vec_io.h", "wave_reduce.h", "packed_rows.h"]
ROWSUM_LIB_PATH = os.path.join(_HERE, "librowsum_hip.so")
ROWSUM_SOURCES = ["rowsum_api.hip"]
ROWSUM_HEADERS = ["rowsum_kernels.h", "vec_io.h", "wave_reduce.h", "packed_rows.h"]
SOFTMAX_SOURCES = ["softmax_api.hip"]
SOFTMAX_HEADERS = ["softmax_kernels.h", "vec_io.h", "wave_reduce.h", "packed_rows.h", "launch_util.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-Wall",
    # packed-fp32 VALU forms are kept off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(sources, lib_path: str, verbose: bool) -> str:
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", lib_path,
           *[os.path.join(CSRC, s) for s in sources]]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in proc.stderr.splitlines() if noise not in ln)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return lib_path


def build(verbose: bool = False) -> str:
    """Compiles csrc/ into librmsnorm_hip.so, libsoftmax_hip.so, liblayernorm_hip.so,
    libcrossentropy_hip.so and librowsum_hip.so next to this file; returns the path of the
    RMSNorm library."""
    _compile(ROWSUM_SOURCES, ROWSUM_LIB_PATH, verbose)
    _compile(SOFTMAX_SOURCES, SOFTMAX_LIB_PATH, verbose)
    _compile(LAYERNORM_SOURCES, LAYERNORM_LIB_PATH, verbose)
    _compile(CROSSENTROPY_SOURCES, CROSSENTROPY_LIB_PATH, verbose)
    return _compile(SOURCES, LIB_PATH, verbose)


def build_softmax(verbose: bool = False) -> str:
    return _compile(SOFTMAX_SOURCES, SOFTMAX_LIB_PATH, verbose)


def build_layernorm(verbose: bool = False) -> str:
    return _compile(LAYERNORM_SOURCES, LAYERNORM_LIB_PATH, verbose)


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps.append(os.path.join(ROOT, "include", "rmsnorm.h"))
    return any(os.path.getmtime(d) > built for d in deps)


def build_crossentropy(verbose: bool = False) -> str:
    return _compile(CROSSENTROPY_SOURCES, CROSSENTROPY_LIB_PATH, verbose)


def build_rowsum(verbose: bool = False) -> str:
    return _compile(ROWSUM_SOURCES, ROWSUM_LIB_PATH, verbose)


if __name__ == "__main__":
    print(build(verbose=True))
