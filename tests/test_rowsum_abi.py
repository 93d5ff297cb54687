"""Host-side checks of the row-sum C ABI that need no GPU."""
import os
import re

import pytest

from paper_2603_21331_amd import rowsum as rs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rowsum.h")
P = 0x10000
BIG = 1 << 24


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(rowsum_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = rs.load()
    names = declared_functions()
    assert "rowsum_fwd" in names and "rowsum_fwd_tuned" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in rowsum.h but not exported"
        assert hasattr(rs, name), f"binding lacks {name}"


def test_enum_values_match_the_header():
    for name, value in re.findall(r"\b(ROWSUM_[A-Z0-9_]+)\s*=\s*(-?\d+)", open(HEADER).read()):
        assert getattr(rs, name) == int(value), name


@pytest.mark.parametrize("args", [dict(x=0), dict(y=0), dict(M=-1), dict(N=0), dict(N=-3), dict(dtype=3),
                                  dict(dtype=-1), dict(x=P + 1, dtype=1), dict(x=P + 2, dtype=0),
                                  dict(y=P + BIG + 2), dict(N=1 << 32), dict(M=1 << 40, N=1 << 30)])
def test_invalid_arguments_are_rejected_without_a_launch(args):
    lib = rs.load()
    a = dict(x=P, y=P + BIG, M=4, N=8, dtype=2)
    a.update(args)
    call = (a["x"], a["y"], a["M"], a["N"], a["dtype"], None)
    assert lib.rowsum_fwd(*call) == rs.ROWSUM_ERR_INVALID_ARG
    assert lib.rowsum_fwd_tuned(*call, 256) == rs.ROWSUM_ERR_INVALID_ARG


def test_empty_batch_and_bad_thread_counts():
    lib = rs.load()
    assert lib.rowsum_fwd(None, None, 0, 16, 2, None) == rs.ROWSUM_OK
    assert lib.rowsum_fwd_tuned(None, None, 0, 16, 2, None, 64) == rs.ROWSUM_OK
    for bad in (0, 1, 2, 3, 4, 24, 100, 1088, 2048, -64):   # 2: a valid code, but not for 4096 elements
        assert lib.rowsum_fwd_tuned(P, P + BIG, 4, 4096, 2, None, bad) == rs.ROWSUM_ERR_INVALID_ARG
    # the LDS-staged kernel (code 2) takes at most 1024 elements, at any alignment
    assert lib.rowsum_fwd_tuned(P + 2, P + BIG, 4, 1025, 1, None, 2) == rs.ROWSUM_ERR_INVALID_ARG
    assert lib.rowsum_fwd_tuned(P + 2, P + BIG, 0, 1024, 1, None, 2) == rs.ROWSUM_OK
    # several rows per wavefront: only aligned rows of at most 8 vectors per lane
    assert lib.rowsum_fwd_tuned(P, P + BIG, 0, 512, 2, None, 8) == rs.ROWSUM_OK            # 64 vectors
    assert lib.rowsum_fwd_tuned(P, P + BIG, 4, 520, 2, None, 8) == rs.ROWSUM_ERR_INVALID_ARG
    assert lib.rowsum_fwd_tuned(P, P + BIG, 4, 100, 2, None, 8) == rs.ROWSUM_ERR_INVALID_ARG  # 200-byte rows
    assert lib.rowsum_fwd_tuned(P + 2, P + BIG, 4, 64, 2, None, 16) == rs.ROWSUM_ERR_INVALID_ARG


def test_automatic_threads_per_row():
    auto = rs.rowsum_auto_threads_per_row
    # just past the LDS-staged kernel's 1024 elements: one wavefront per row
    assert auto(1032, 1) == 64 and auto(2048, 1) == 64 and auto(1028, 0) == 64 and auto(2048, 0) == 192
    # (rows of up to 1024 elements never get here: they go through LDS, see below)
    # longer rows: two or three vectors per thread, whole wavefronts, at most 768 threads
    assert auto(4096, 1) == 192 and auto(8192, 1) == 384
    assert auto(4096, 0) == 384 and auto(8192, 0) == 768 and auto(8192, 2) == 384
    assert auto(32000, 1) == 768 and auto(65536, 1) == 768 and auto(1 << 30, 2) == 768
    assert auto(1025, 2) == 64 and auto(1031, 0) == 64                          # not 16-byte rows
    # up to 1024 elements: through LDS, aligned or not
    assert auto(1, 1) == 2 and auto(7, 0) == 2 and auto(16, 2) == 2 and auto(8, 0) == 2
    assert auto(17, 1) == 2 and auto(64, 1) == 2 and auto(120, 2) == 2 and auto(511, 0) == 2 and auto(1023, 1) == 2
    assert auto(128, 1) == 2 and auto(512, 2) == 2 and auto(1024, 1) == 2 and auto(1024, 0) == 2
    with pytest.raises(rs.RowSumError):
        auto(0, 1)
    with pytest.raises(rs.RowSumError):
        auto(8, 5)
    assert rs.rowsum_status_string(0) == "ok" and rs.rowsum_status_string(-1)
