"""Builds the HIP libraries for gfx950 with hipcc (cross-compiles without a GPU), and tells a
built library that no longer matches its sources from one that does.

Every library carries a build id: a hash over the compiler flags and the contents of every file
it is built from (its .hip source, the csrc headers it includes, its public header).  The id is
compiled into the library as a string, so it can be read back from the file without loading
it, and it does not depend on modification times (a copy of the tree to another machine keeps
it valid).  `ensure(name)` is what the bindings call before loading: a missing or stale library
is rebuilt if hipcc is there, otherwise the call raises and names the stale file.
"""
from __future__ import annotations

import hashlib
import os
import re
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")

_COMMON = ["vec_io.h", "wave_reduce.h", "packed_rows.h", "launch_util.h", "dispatch_util.h", "queue_slots.h", "build_id.h"]

# name -> (library file, source, csrc headers, public header)
LIBRARIES = {
    "rmsnorm": ("librmsnorm_hip.so", "rmsnorm_api.hip", ["rmsnorm_kernels.h"] + _COMMON, "rmsnorm.h"),
    "softmax": ("libsoftmax_hip.so", "softmax_api.hip", ["softmax_kernels.h"] + _COMMON, "softmax.h"),
    "layernorm": ("liblayernorm_hip.so", "layernorm_api.hip", ["layernorm_kernels.h"] + _COMMON, "layernorm.h"),
    "crossentropy": ("libcrossentropy_hip.so", "crossentropy_api.hip",
                     ["crossentropy_kernels.h"] + _COMMON, "crossentropy.h"),
    "rowsum": ("librowsum_hip.so", "rowsum_api.hip", ["rowsum_kernels.h"] + _COMMON, "rowsum.h"),
    "measure": ("libmeasure_hip.so", "measure_api.hip", ["vec_io.h", "launch_util.h", "build_id.h"], "measure.h"),
}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-Wall",
    # packed-fp32 VALU forms are kept off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]

BUILD_ID_MARKER = b"RMS_BUILD_ID:"


def lib_path(name: str) -> str:
    return os.path.join(_HERE, LIBRARIES[name][0])


# Paths under their old names (the bindings and the benchmark refer to them).
LIB_PATH = lib_path("rmsnorm")
SOFTMAX_LIB_PATH = lib_path("softmax")
LAYERNORM_LIB_PATH = lib_path("layernorm")
CROSSENTROPY_LIB_PATH = lib_path("crossentropy")
ROWSUM_LIB_PATH = lib_path("rowsum")
MEASURE_LIB_PATH = lib_path("measure")


def dependencies(name: str) -> list:
    """Every file the library is built from, in a fixed order."""
    _, source, headers, public = LIBRARIES[name]
    return [os.path.join(CSRC, source)] + [os.path.join(CSRC, h) for h in headers] + \
        [os.path.join(INCLUDE, public)]


def source_id(name: str) -> str:
    """Hash of the flags and of the contents of the library's dependencies, as they are now."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for path in dependencies(name):
        h.update(b"\0" + os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:32]


def built_id(name: str):
    """The build id compiled into the library file, None if there is no file or no id in it."""
    try:
        with open(lib_path(name), "rb") as f:
            blob = f.read()
    except OSError:
        return None
    m = re.search(re.escape(BUILD_ID_MARKER) + rb"([0-9a-f]{32})", blob)
    return m.group(1).decode() if m else None


def is_stale(name: str = "rmsnorm") -> bool:
    """True if the library is missing or was built from other sources than the present ones."""
    return built_id(name) != source_id(name)


def hipcc():
    """Path of hipcc, or None if this machine has none."""
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    return shutil.which("hipcc")


def compile_library(name: str, verbose: bool = False) -> str:
    cc = hipcc()
    if cc is None:
        raise RuntimeError(f"no hipcc on this machine: cannot build {lib_path(name)}")
    _, source, _, _ = LIBRARIES[name]
    cmd = [cc, *HIPCC_FLAGS, f'-DRMS_BUILD_ID="{source_id(name)}"', "-I", INCLUDE, "-o", lib_path(name),
           os.path.join(CSRC, source)]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in proc.stderr.splitlines() if noise not in ln)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return lib_path(name)


def build(verbose: bool = False, jobs: int = 0) -> str:
    """Compiles every library, whether or not a built one is there (several hipcc processes side
    by side: the libraries do not depend on each other); returns the path of the RMSNorm
    library."""
    from concurrent.futures import ThreadPoolExecutor
    names = ["rmsnorm", "layernorm", "softmax", "crossentropy", "rowsum", "measure"]   # longest first
    jobs = jobs or max(1, min(len(names), (os.cpu_count() or 2) // 2))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for path in pool.map(lambda n: compile_library(n, verbose), names):
            pass
    return lib_path("rmsnorm")


def ensure(name: str) -> str:
    """Path of an up-to-date library: builds it if it is missing or stale; on a machine without
    hipcc a missing or stale library is an error that names the file."""
    if is_stale(name):
        path = lib_path(name)
        if hipcc() is None:
            state = "is missing" if not os.path.exists(path) else \
                f"is stale (built from other sources than the present {', '.join(os.path.basename(d) for d in dependencies(name))})"
            raise RuntimeError(f"{path} {state} and this machine has no hipcc to rebuild it")
        compile_library(name)
    return lib_path(name)


if __name__ == "__main__":
    print(build(verbose=True))
