"""Host-side checks of the layernorm C ABI that need no GPU."""
import os
import re

import pytest

from paper_2603_21331_amd import layernorm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "layernorm.h")
P = 0x10000
BIG = 1 << 24


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(layernorm_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = layernorm.load()
    names = declared_functions()
    assert "layernorm_fwd" in names and "layernorm_fwd_tuned" in names
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in layernorm.h but not exported"
        assert hasattr(layernorm, name), f"binding lacks {name}"


def test_enum_values_match_the_header():
    for name, value in re.findall(r"\b(LAYERNORM_[A-Z0-9_]+)\s*=\s*(-?\d+)", open(HEADER).read()):
        assert getattr(layernorm, name) == int(value), name


@pytest.mark.parametrize("args", [dict(x=0), dict(y=0), dict(w=0), dict(eps=-1.0), dict(eps=float("nan")),
                                  dict(b=P + 3 * BIG + 1, dtype=1), dict(M=-1), dict(N=0), dict(dtype=3),
                                  dict(dtype=-1), dict(x=P + 1, dtype=1), dict(M=1 << 40, N=1 << 40)])
def test_invalid_arguments_are_rejected_without_a_launch(args):
    lib = layernorm.load()
    a = dict(x=P, w=P + 2 * BIG, b=P + 3 * BIG, y=P + BIG, M=4, N=8, eps=1e-5, dtype=2)
    a.update(args)
    assert lib.layernorm_fwd(a["x"], a["w"], a["b"], a["y"], a["M"], a["N"], a["eps"], a["dtype"], None) == \
        layernorm.LAYERNORM_ERR_INVALID_ARG
    assert lib.layernorm_fwd_variant(a["x"], a["w"], a["b"], a["y"], a["M"], a["N"], a["eps"], a["dtype"],
                                     None, 3) == layernorm.LAYERNORM_ERR_INVALID_ARG


def test_empty_batch_unknown_variant_and_unsupported_shapes():
    lib = layernorm.load()
    W, B, Y = P + 2 * BIG, P + 3 * BIG, P + BIG
    assert lib.layernorm_fwd(None, None, None, None, 0, 16, 1e-5, 2, None) == layernorm.LAYERNORM_OK
    assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 8, 1e-5, 2, None, 1000) == layernorm.LAYERNORM_ERR_INVALID_ARG
    assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 8, 1e-5, 2, None, 9) == layernorm.LAYERNORM_ERR_INVALID_ARG
    # the LDS-staged kernel takes at most 1024 elements, x and y at any offsets
    for dtype in (0, 1, 2):
        assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 1025, 1e-5, dtype, None, 7) == layernorm.LAYERNORM_ERR_UNSUPPORTED
    assert lib.layernorm_fwd_variant(P + 2, W, B, Y + 18, 0, 77, 1e-5, 2, None, 7) == layernorm.LAYERNORM_OK
    assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 8, 1e-5, 2, None, -1) == layernorm.LAYERNORM_ERR_INVALID_ARG
    for bad in (0, 4, 128, 2048):
        assert lib.layernorm_fwd_tuned(P, W, B, Y, 4, 4096, 1e-5, 2, None, bad) == layernorm.LAYERNORM_ERR_INVALID_ARG
    for v in (1, 2, 4):
        assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 7, 1e-5, 2, None, v) == layernorm.LAYERNORM_ERR_UNSUPPORTED
        # a misaligned bias pointer alone also rules the vector kernels out
        assert lib.layernorm_fwd_variant(P, W, B + 2, Y, 4, 64, 1e-5, 2, None, v) == layernorm.LAYERNORM_ERR_UNSUPPORTED
    assert lib.layernorm_fwd_variant(P, W, B, Y, 4, 4096, 1e-5, 2, None, 1) == layernorm.LAYERNORM_ERR_UNSUPPORTED
    assert lib.layernorm_fwd_variant(P, W, None, Y, 4, 1024, 1e-5, 2, None, 4) == layernorm.LAYERNORM_ERR_UNSUPPORTED
    assert lib.layernorm_fwd_tuned(P, W, B, Y, 1, 65544, 1e-5, 2, None, 1024) == layernorm.LAYERNORM_ERR_UNSUPPORTED


def test_automatic_threads_per_row():
    auto = layernorm.layernorm_auto_threads_per_row
    # aligned rows that the automatic path sends through LDS report 1: rows of at most 64
    # bytes, and 5 vectors on 8 lanes, 9 or 10 on 16
    assert auto(8, 1) == 1 and auto(32, 2) == 1 and auto(16, 0) == 1 and auto(40, 2) == 1
    assert auto(72, 2) == 1 and auto(80, 1) == 1 and auto(96, 1) == 16 and auto(48, 2) == 8
    assert auto(64, 1) == 8 and auto(128, 2) == 16 and auto(256, 1) == 16 and auto(512, 1) == 32
    assert auto(264, 1) == 32 and auto(576, 2) == 64
    # rows of 1 to 32 KiB that are a multiple of 16 bytes but not of the 128-byte line: through LDS up
    # to 1.75 KiB (1), then the element-addressed kernel's thread counts; longer ones as before
    assert auto(520, 2) == 1 and auto(260, 0) == 1 and auto(888, 1) == 1 and auto(904, 1) == 64
    assert auto(2056, 1) == 256 and auto(8200, 2) == 256 and auto(1028, 0) == 256 and auto(16376, 1) == 256
    assert auto(16392, 1) == 1024
    assert auto(32, 0) == 8 and auto(64, 0) == 16 and auto(96, 0) == 16 and auto(128, 0) == 32
    assert auto(192, 0) == 32 and auto(256, 0) == 64
    # past one wavefront: the smallest workgroup whose threads hold at most 24 elements of a
    # 16-bit type (16 of fp32), which runs the resident kernel ...
    assert auto(2048, 2) == 64 and auto(4096, 1) == 256 and auto(5120, 1) == 256 and auto(6144, 2) == 256
    assert auto(8192, 1) == 512 and auto(12288, 2) == 512 and auto(16384, 2) == 1024 and auto(24576, 1) == 1024
    assert auto(4096, 0) == 256 and auto(8192, 0) == 512 and auto(16384, 0) == 1024
    # ... and beyond that the smallest one that holds the row in at most 8 chunks per thread
    assert auto(24584, 1) == 512 and auto(32768, 1) == 512 and auto(65536, 2) == 1024
    assert auto(65544, 2) == 0 and auto(1023, 1) == 0
    assert auto(16388, 0) == 1024 and auto(32768, 0) == 1024 and auto(32772, 0) == 0
    assert layernorm.layernorm_register_max_n(1) == 65536 and layernorm.layernorm_register_max_n(0) == 32768
    with pytest.raises(layernorm.LayerNormError):
        auto(0, 1)
    assert layernorm.layernorm_status_string(0) == "ok" and layernorm.layernorm_status_string(-2)


def test_unaligned_walk_grid_query():
    """The grid of the walking form: a multiple of the compute units (256 without a device) near
    48 KiB of rows in flight per compute unit, chosen so that the rows divide evenly; 0 where
    the one-row-per-workgroup form runs."""
    lib = layernorm.load()
    X, W, B, Y = P, P + 2 * BIG, P + 3 * BIG, P + 8 * BIG
    q = lib.layernorm_unaligned_walk_grid
    assert q(X, W, B, Y, 8192, 4097, 1) == 1024 and q(X, W, B, Y, 16384, 8191, 2) == 768
    assert q(X, W, B, Y, 4096, 20481, 2) == 256 and q(X, W, None, Y, 8192, 4097, 1) == 1024
    assert q(X + 6, W + 2, B + 4, Y + 22, 8192, 4097, 1) == 1024   # same offset from a line
    assert q(X, W, B, Y + 2, 8192, 4097, 1) == 1024                # different offsets: cut at x's lines
    assert q(X, W, B, Y, 8192, 4097, 0) == 768                     # fp32 walks too
    assert q(X, W, B, Y, 8192, 1027, 0) == 0 and q(X, W, B, Y, 8192, 1028, 0) == 2048
    assert q(X, W, B, Y, 2048, 16387, 0) == 256 and q(X, W, B, Y, 2048, 16388, 0) == 0
    assert q(X, W, B, Y, 3000, 4097, 1) == 0                       # too few rows
    assert q(X, W, B, Y, 16384, 2055, 1) == 0 and q(X, W, B, Y, 16384, 2056, 1) > 0
    assert q(X, W, B, Y, 2048, 32775, 1) == 256 and q(X, W, B, Y, 2048, 32776, 1) == 0
    assert q(X, W, B, Y, 8192, 0, 1) == layernorm.LAYERNORM_ERR_INVALID_ARG
    assert q(0, W, B, Y, 8192, 4097, 1) == layernorm.LAYERNORM_ERR_INVALID_ARG


def test_queue_plan_query():
    """Where the automatic path takes the work-queue form of the resident kernel: launches of a few
    hundred megabytes of rows that 256 or 512 threads hold (thresholds by row length), never rows one
    wavefront takes or rows of more than 2048 vectors."""
    plan = layernorm.layernorm_queue_plan
    FP32, FP16, BF16 = 0, 1, 2
    MiB = 1 << 20
    # 256 threads: 128 MiB of x from rows of 6 KiB up, 192 MiB for shorter ones
    assert plan(16384, 4096, FP16)[:2] == (True, 256) and not plan(16383, 4096, FP16)[0]
    assert plan(128 * MiB // (5120 * 2) + 1, 5120, FP16)[0] and not plan(128 * MiB // (5120 * 2), 5120, FP16)[0]
    assert plan(32768, 3072, FP16)[0] and not plan(32767, 3072, FP16)[0]          # 6 KiB rows: 192 MiB
    assert plan(8192, 4096, FP32)[:2] == (True, 256) and not plan(8191, 4096, FP32)[0]
    # 12 to 16 KiB rows of a 16-bit type in 256 threads (weight and bias kept packed): 192 MiB
    assert plan(12288, 8192, BF16)[:2] == (True, 256) and not plan(12287, 8192, BF16)[0]
    assert plan(14044, 7168, FP16)[:2] == (True, 256) and not plan(14043, 7168, FP16)[0]
    # 512 threads: rows beyond 20 KiB from 96 MiB, up to 20 KiB from 256 MiB
    assert plan(4096, 12288, BF16)[:2] == (True, 512) and not plan(4095, 12288, BF16)[0]
    assert plan(13108, 10240, FP16)[0] and not plan(13107, 10240, FP16)[0]
    assert plan(3072, 8192, FP32)[:2] == (True, 512) and not plan(3071, 8192, FP32)[0]
    assert plan(3072, 16384, BF16)[:2] == (True, 512) and not plan(3071, 16384, BF16)[0]
    # rows one wavefront takes can run it but never do on the automatic path
    assert plan(1 << 22, 2048, FP16)[:2] == (False, 256)
    # shards, blocks of at most 128 KiB of rows, grids that are whole numbers of shards
    for M, N, dt, shards, block_rows in ((1000, 4096, FP16, 16, 16), (1000, 5120, FP16, 16, 8), (1000, 3072, FP16, 16, 16),
                                         (1000, 12288, BF16, 8, 4), (1000, 8192, FP32, 8, 4), (1000, 512, FP32, 16, 64)):
        _, threads, grid, s, br = plan(M, N, dt)
        assert (s, br) == (shards, block_rows) and grid % s == 0 and grid >= s, (M, N, dt)
    lib = layernorm.load()
    for M, N, dt in ((4, 16392, FP16), (4, 8196, FP32), (4, 65536, BF16), (4, 4100, FP16), (0, 4096, FP16), (1 << 30, 4096, FP16)):
        assert lib.layernorm_queue_plan(M, N, dt, None, None, None, None) == layernorm.LAYERNORM_ERR_UNSUPPORTED, (M, N, dt)
    for M, N, dt in ((4, 0, FP16), (-1, 4096, FP16), (4, 4096, 3)):
        assert lib.layernorm_queue_plan(M, N, dt, None, None, None, None) == layernorm.LAYERNORM_ERR_INVALID_ARG
