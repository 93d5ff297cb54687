"""More streams than the libraries have blocks of counters for their work-queue kernels (32 per
device): the 33rd and 34th stream run the kernels that need no counters, with the same bits.  Runs
in a child process, because the tables of stream slots are per process and this test fills them."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_streams_beyond_the_counter_blocks(gpu_device):
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    proc = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "stream_slots_child.py")],
                          capture_output=True, text=True, cwd=ROOT, env=env, timeout=280)
    tail = (proc.stdout[-2000:] + "\n" + proc.stderr[-2000:])
    assert proc.returncode == 0, tail
    assert proc.stdout.strip().endswith("ok"), tail
