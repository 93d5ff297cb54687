"""Host-side checks of the softmax C ABI that need no GPU."""
import os
import re

import pytest

from paper_2603_21331_amd import softmax

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "softmax.h")
P = 0x10000
BIG = 1 << 24


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(softmax_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = softmax.load()
    names = declared_functions()
    assert "softmax_fwd" in names and "softmax_fwd_tuned" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in softmax.h but not exported"
        assert hasattr(softmax, name), f"binding lacks {name}"


def test_enum_values_match_the_header():
    for name, value in re.findall(r"\b(SOFTMAX_[A-Z0-9_]+)\s*=\s*(-?\d+)", open(HEADER).read()):
        assert getattr(softmax, name) == int(value), name


@pytest.mark.parametrize("args", [dict(x=0), dict(y=0), dict(M=-1), dict(N=0), dict(dtype=3),
                                  dict(dtype=-1), dict(x=P + 1, dtype=1), dict(M=1 << 40, N=1 << 40)])
def test_invalid_arguments_are_rejected_without_a_launch(args):
    lib = softmax.load()
    a = dict(x=P, y=P + BIG, M=4, N=8, dtype=2)
    a.update(args)
    assert lib.softmax_fwd(a["x"], a["y"], a["M"], a["N"], a["dtype"], None) == softmax.SOFTMAX_ERR_INVALID_ARG
    assert lib.softmax_fwd_variant(a["x"], a["y"], a["M"], a["N"], a["dtype"], None, 3) == \
        softmax.SOFTMAX_ERR_INVALID_ARG


def test_empty_batch_unknown_variant_and_unsupported_shapes():
    lib = softmax.load()
    assert lib.softmax_fwd(None, None, 0, 16, 2, None) == softmax.SOFTMAX_OK
    assert lib.softmax_fwd_variant(P, P + BIG, 4, 8, 2, None, 1000) == softmax.SOFTMAX_ERR_INVALID_ARG
    assert lib.softmax_fwd_variant(P, P + BIG, 4, 8, 2, None, -1) == softmax.SOFTMAX_ERR_INVALID_ARG
    for bad in (0, 4, 128, 2048):
        assert lib.softmax_fwd_tuned(P, P + BIG, 4, 4096, 2, None, bad) == softmax.SOFTMAX_ERR_INVALID_ARG
    # unaligned rows and over-long rows are refused by the register-resident kernels
    for v in (1, 2, 4):
        assert lib.softmax_fwd_variant(P, P + BIG, 4, 7, 2, None, v) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P, P + BIG, 4, 4096, 2, None, 1) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P, P + BIG, 4, 1024, 2, None, 4) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_tuned(P, P + BIG, 4, 4096, 2, None, 64) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_tuned(P, P + BIG, 1, 65544, 2, None, 1024) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P, P + BIG, 1, 65544, 2, None, 2) == softmax.SOFTMAX_ERR_UNSUPPORTED
    # the element-aligned kernel takes any alignment but not rows past the register limit
    assert lib.softmax_fwd_variant(P, P + BIG, 1, 65544, 2, None, 5) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P, P + BIG, 0, 1023, 2, None, 5) == softmax.SOFTMAX_OK
    # the streaming kernel takes any N below 2^31
    assert lib.softmax_fwd_variant(P, P + BIG, 0, 1 << 30, 2, None, 6) == softmax.SOFTMAX_OK
    assert lib.softmax_fwd_variant(P, P + BIG, 1, 1 << 31, 2, None, 6) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P, P + BIG, 1, 8, 2, None, 8) == softmax.SOFTMAX_ERR_INVALID_ARG
    # the LDS-staged kernel takes at most 1024 elements, x and y at any offsets
    for dtype in (0, 1, 2):
        assert lib.softmax_fwd_variant(P, P + BIG, 4, 1025, dtype, None, 7) == softmax.SOFTMAX_ERR_UNSUPPORTED
    assert lib.softmax_fwd_variant(P + 2, P + BIG + 18, 0, 77, 2, None, 7) == softmax.SOFTMAX_OK


def test_automatic_threads_per_row():
    auto = softmax.softmax_auto_threads_per_row
    # aligned rows that the automatic path sends through LDS report 1: rows of at most 64
    # bytes, and 5 vectors on 8 lanes, 9 or 10 on 16
    assert auto(8, 1) == 1 and auto(32, 2) == 1 and auto(16, 0) == 1 and auto(40, 2) == 1
    assert auto(72, 2) == 1 and auto(80, 1) == 1 and auto(96, 1) == 16 and auto(48, 2) == 8
    assert auto(64, 1) == 8 and auto(128, 2) == 16 and auto(256, 1) == 32 and auto(512, 1) == 64
    assert auto(192, 1) == 16 and auto(256, 1) == 32 and auto(384, 2) == 32 and auto(448, 2) == 64
    assert auto(96, 0) == 16 and auto(128, 0) == 32 and auto(192, 0) == 32 and auto(224, 0) == 64
    assert auto(2048, 2) == 64 and auto(4096, 1) == 256 and auto(5632, 1) == 256
    assert auto(5696, 1) == 512 and auto(8192, 1) == 512 and auto(4096, 0) == 512
    assert auto(16384, 2) == 256 and auto(16448, 2) == 1024 and auto(32768, 1) == 1024 and auto(65536, 2) == 1024
    assert auto(65544, 2) == 0 and auto(1023, 1) == 0
    assert auto(8192, 0) == 256 and auto(8224, 0) == 1024 and auto(32768, 0) == 1024 and auto(32772, 0) == 0
    # rows of 256 bytes to 64 KiB that are a multiple of 16 bytes but not of the 128-byte line: through
    # LDS up to 1.5 KiB (1), then the element-addressed kernel's thread counts; longer ones as before
    assert auto(200, 1) == 1 and auto(392, 2) == 1 and auto(100, 0) == 1 and auto(760, 1) == 1
    assert auto(776, 1) == 64 and auto(2040, 1) == 64 and auto(5640, 1) == 256 and auto(8200, 1) == 256
    assert auto(16392, 2) == 512 and auto(8196, 0) == 512 and auto(32760, 2) == 512
    assert auto(32776, 2) == 1024 and auto(40952, 2) == 1024
    assert softmax.softmax_register_max_n(1) == 65536 and softmax.softmax_register_max_n(0) == 32768
    with pytest.raises(softmax.SoftmaxError):
        auto(0, 1)
    assert softmax.softmax_status_string(0) == "ok" and softmax.softmax_status_string(-2)
