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
    for bad in (0, 1, 32, 100, 1088, 2048, -64):
        assert lib.crossentropy_fwd_tuned(P, P + BIG, P + 2 * BIG, None, 4, 4096, 2, None, bad) == \
            ce.CROSSENTROPY_ERR_INVALID_ARG


def test_automatic_threads_per_row():
    auto = ce.crossentropy_auto_threads_per_row
    for dtype in (0, 1, 2):
        for n in (1, 7, 128, 1000):
            assert auto(n, dtype) == 64
    # about 8 16-byte vectors per thread for the 16-bit types and 4 for fp32, in whole wavefronts
    assert auto(2048, 1) == 64 and auto(4096, 2) == 64 and auto(8192, 1) == 128 and auto(12288, 2) == 192
    assert auto(16384, 1) == 256 and auto(32000, 1) == 512 and auto(50257, 2) == 512
    assert auto(65536, 1) == 1024 and auto(131072, 2) == 1024 and auto(1 << 30, 1) == 1024
    assert auto(1024, 0) == 64 and auto(4096, 0) == 256 and auto(8192, 0) == 512
    assert auto(16000, 0) == 512 and auto(32000, 0) == 1024 and auto(65536, 0) == 1024
    with pytest.raises(ce.CrossEntropyError):
        auto(0, 1)
    with pytest.raises(ce.CrossEntropyError):
        auto(8, 5)
    assert ce.crossentropy_status_string(0) == "ok" and ce.crossentropy_status_string(-1)
