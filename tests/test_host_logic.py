"""The launch arithmetic the kernels rely on, checked on the CPU: the XCD row permutation, the
cut of rows that are not 16-byte aligned and the slot each lane holds, the selection of kernel
instantiations, lane groups and tiles of the LDS-staged kernels, and the grids.  The checks are
C++ (tests/host/host_logic.hip includes the libraries' own headers); hipcc builds them into a host
program that touches no GPU."""
import os
import subprocess

import pytest

from paper_2603_21331_amd import build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_logic(tmp_path):
    cc = build.hipcc()
    if cc is None:
        pytest.skip("no hipcc on this machine")
    exe = str(tmp_path / "host_logic")
    cmd = [cc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-Wall",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", build.CSRC, "-I", build.INCLUDE, "-o", exe, os.path.join(HERE, "host", "host_logic.hip")]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout[-3000:] + run.stderr[-1000:]
