"""Host-side checks of the cross-entropy C ABI that need no GPU."""
import os
import re

import pytest

from paper_2603_21331_amd import crossentropy as ce

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "crossentropy.h")
P = 0x10000
BIG = 1 << 24


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(crossentropy_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = ce.load()
    names = declared_functions()
    assert "crossentropy_fwd" in names and "crossentropy_fwd_tuned" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in crossentropy.h but not exported"
        assert hasattr(ce, name), f"binding lacks {name}"


def test_enum_values_match_the_header():
    for name, value in re.findall(r"\b(CROSSENTROPY_[A-Z0-9_]+)\s*=\s*(-?\d+)", open(HEADER).read()):
        assert getattr(ce, name) == int(value), name


@pytest.mark.parametrize("args", [dict(x=0), dict(t=0), dict(loss=0), dict(M=-1), dict(N=0), dict(N=-3),
                                  dict(dtype=3), dict(dtype=-1), dict(x=P + 1, dtype=1), dict(x=P + 2, dtype=0),
                                  dict(t=P + BIG + 4), dict(loss=P + 2 * BIG + 2), dict(lse=P + 3 * BIG + 1),
                                  dict(N=1 << 32), dict(M=1 << 40, N=1 << 30)])
def test_invalid_arguments_are_rejected_without_a_launch(args):
    lib = ce.load()
    a = dict(x=P, t=P + BIG, loss=P + 2 * BIG, lse=P + 3 * BIG, M=4, N=8, dtype=2)
    a.update(args)
    call = (a["x"], a["t"], a["loss"], a["lse"], a["M"], a["N"], a["dtype"], None)
    assert lib.crossentropy_fwd(*call) == ce.CROSSENTROPY_ERR_INVALID_ARG
    assert lib.crossentropy_fwd_tuned(*call, 256) == ce.CROSSENTROPY_ERR_INVALID_ARG


def test_empty_batch_and_bad_thread_counts():
    lib = ce.load()
    assert lib.crossentropy_fwd(None, None, None, None, 0, 16, 2, None) == ce.CROSSENTROPY_OK
    assert lib.crossentropy_fwd_tuned(None, None, None, None, 0, 16, 2, None, 64) == ce.CROSSENTROPY_OK
    for bad in (0, 1, 3, 4, 24, 48, 100, 1088, 2048, -64, -1):
        assert lib.crossentropy_fwd_tuned(P, P + BIG, P + 2 * BIG, None, 4, 4096, 2, None, bad) == \
            ce.CROSSENTROPY_ERR_INVALID_ARG


def test_lane_groups_refuse_rows_they_cannot_take():
    """8, 16 or 32 lanes per row need 16-byte aligned rows of at most 8 vectors per lane."""
    lib = ce.load()
    f = lib.crossentropy_fwd_tuned
    for lanes, n_too_long in ((8, 520), (16, 1032), (32, 2056)):
        assert f(P, P + BIG, P + 2 * BIG, None, 4, n_too_long, 2, None, lanes) == ce.CROSSENTROPY_ERR_UNSUPPORTED
        assert f(P, P + BIG, P + 2 * BIG, None, 4, n_too_long // 2 + 4, 0, None, lanes) == ce.CROSSENTROPY_ERR_UNSUPPORTED
        assert f(P, P + BIG, P + 2 * BIG, None, 4, 100, 1, None, lanes) == ce.CROSSENTROPY_ERR_UNSUPPORTED  # 200-byte rows
        assert f(P + 2, P + BIG, P + 2 * BIG, None, 4, 64, 1, None, lanes) == ce.CROSSENTROPY_ERR_UNSUPPORTED  # base off by 2 bytes
        assert f(P, P + BIG, P + 2 * BIG, None, 0, 64, 1, None, lanes) == ce.CROSSENTROPY_OK  # empty batch
    assert "thread count" in ce.crossentropy_status_string(ce.CROSSENTROPY_ERR_UNSUPPORTED)
    # the LDS-staged kernel (code 2): any alignment, at most 1024 classes
    assert f(P + 2, P + BIG, P + 2 * BIG, None, 4, 1025, 1, None, 2) == ce.CROSSENTROPY_ERR_UNSUPPORTED
    assert f(P, P + BIG, P + 2 * BIG, None, 4, 4096, 0, None, 2) == ce.CROSSENTROPY_ERR_UNSUPPORTED
    assert f(P + 2, P + BIG, P + 2 * BIG, None, 0, 100, 1, None, 2) == ce.CROSSENTROPY_OK
    # 1 was one lane per row once; the LDS-staged kernel covers those rows now
    assert f(P, P + BIG, P + 2 * BIG, None, 4, 10, 1, None, 1) == ce.CROSSENTROPY_ERR_INVALID_ARG


def test_automatic_threads_per_row():
    auto = ce.crossentropy_auto_threads_per_row
    for dtype in (0, 1, 2):
        for n in (1, 7, 10, 31):             # a handful of classes: through LDS, one lane per row
            assert auto(n, dtype) == 2
        for n in (65, 130, 511, 1001):       # up to 1024 classes, not whole 16-byte vectors: through LDS
            assert auto(n, dtype) == 2
        for n in (1025, 1031):               # longer rows that are not whole 16-byte vectors: a workgroup
            assert auto(n, dtype) in (64, 128)
    # from 32 classes up to 256 bytes per row: through LDS, aligned or not
    assert auto(32, 1) == 2 and auto(64, 1) == 2 and auto(128, 2) == 2 and auto(32, 0) == 2 and auto(60, 0) == 2
    # few classes in whole vectors: lane groups, at most 32 / 64 / 256 (fp32: 128) vectors per row
    assert auto(136, 1) == 8 and auto(256, 2) == 8 and auto(264, 2) == 16
    assert auto(512, 1) == 16 and auto(520, 1) == 32 and auto(1000, 1) == 32 and auto(1024, 2) == 32
    assert auto(2048, 1) == 32 and auto(2056, 2) == 64
    assert auto(128, 0) == 2 and auto(512, 0) == 2 and auto(1024, 0) == 2 and auto(1028, 0) == 128   # fp32: through LDS up to 1024
    # about 8 16-byte vectors per thread for the 16-bit types and 4 for fp32, in whole wavefronts
    assert auto(2064, 1) == 64 and auto(4096, 2) == 64 and auto(8192, 1) == 128 and auto(12288, 2) == 192
    assert auto(16384, 1) == 256 and auto(32000, 1) == 512 and auto(50257, 2) == 512
    assert auto(65536, 1) == 1024 and auto(131072, 2) == 1024 and auto(1 << 30, 1) == 1024
    assert auto(2048, 0) == 128 and auto(4096, 0) == 256 and auto(8192, 0) == 512
    assert auto(16000, 0) == 512 and auto(32000, 0) == 1024 and auto(65536, 0) == 1024
    with pytest.raises(ce.CrossEntropyError):
        auto(0, 1)
    with pytest.raises(ce.CrossEntropyError):
        auto(8, 5)
    assert ce.crossentropy_status_string(0) == "ok" and ce.crossentropy_status_string(-1)
