"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2603_21331_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rmsnorm.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rmsnorm_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    assert "rmsnorm_fwd" in names and "rmsnorm_fwd_variant" in names
    assert "rmsnorm_status_string" in names


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in rmsnorm.h but not exported"


def test_binding_has_the_same_names_as_the_header():
    for name in declared_functions():
        assert hasattr(binding, name), f"binding lacks {name}"


def test_enum_values_match_the_header():
    text = open(HEADER).read()
    for name, value in re.findall(r"\b(RMSNORM_[A-Z0-9_]+)\s*=\s*(-?\d+)", text):
        assert getattr(binding, name) == int(value), name


def test_status_strings():
    assert binding.rmsnorm_status_string(0) == "ok"
    for s in (-1, -2, -3, 77):
        assert binding.rmsnorm_status_string(s)


def test_limits():
    assert binding.rmsnorm_wave_max_n(binding.RMSNORM_DTYPE_BF16) == 8192
    assert binding.rmsnorm_wave_max_n(binding.RMSNORM_DTYPE_FP16) == 8192
    assert binding.rmsnorm_wave_max_n(binding.RMSNORM_DTYPE_FP32) == 8192
    assert binding.rmsnorm_block_max_n(binding.RMSNORM_DTYPE_BF16) >= 32768
    assert binding.rmsnorm_unaligned_max_n(binding.RMSNORM_DTYPE_BF16) == 131079
    assert binding.rmsnorm_unaligned_max_n(binding.RMSNORM_DTYPE_FP32) == 65539
    assert binding.rmsnorm_wave_max_n(9) == 0 and binding.rmsnorm_block_max_n(-1) == 0
    assert binding.rmsnorm_unaligned_max_n(5) == 0


# The calls below never reach the device: argument checks come first, and the
# pointers are fake addresses that are never dereferenced on the host.
P = 0x10000


@pytest.mark.parametrize("args", [
    dict(x=0),                       # null x
    dict(w=0),                       # null w
    dict(y=0),                       # null y
    dict(M=-1),
    dict(N=0),
    dict(N=-5),
    dict(dtype=3),
    dict(dtype=-1),
    dict(eps=-1e-6),
    dict(eps=float("nan")),
    dict(x=P + 1, dtype=1),          # not element-aligned
    dict(y=P + 2, dtype=0),
    dict(M=1 << 40, N=1 << 40),      # M * N overflows
])
def test_invalid_arguments_are_rejected_without_a_launch(args):
    lib = binding.load()
    a = dict(x=P, w=P + 4096, y=P + 8192, M=4, N=8, eps=1e-6, dtype=2)
    a.update(args)
    rc = lib.rmsnorm_fwd(a["x"], a["w"], a["y"], a["M"], a["N"], a["eps"], a["dtype"], None)
    assert rc == binding.RMSNORM_ERR_INVALID_ARG
    rc = lib.rmsnorm_fwd_variant(a["x"], a["w"], a["y"], a["M"], a["N"], a["eps"], a["dtype"],
                                 None, binding.RMSNORM_VARIANT_GENERIC)
    assert rc == binding.RMSNORM_ERR_INVALID_ARG


def test_empty_batch_is_a_successful_no_op():
    lib = binding.load()
    assert lib.rmsnorm_fwd(None, None, None, 0, 16, 1e-6, 2, None) == binding.RMSNORM_OK


def test_unknown_variant_and_unsupported_shapes():
    lib = binding.load()
    assert lib.rmsnorm_fwd_variant(P, P + 4096, P + 8192, 4, 8, 1e-6, 2, None, 1000) == \
        binding.RMSNORM_ERR_INVALID_ARG
    assert lib.rmsnorm_fwd_variant(P, P + 4096, P + 8192, 4, 8, 1e-6, 2, None, -1) == \
        binding.RMSNORM_ERR_INVALID_ARG
    # too long for the element-aligned register kernel
    assert lib.rmsnorm_fwd_variant(P, P + (1 << 22), P + (2 << 22), 1, 131081, 1e-6, 2, None,
                                   binding.RMSNORM_VARIANT_UNALIGNED) == binding.RMSNORM_ERR_UNSUPPORTED
    # a row of 7 bf16 elements is not 16-byte aligned: the vector kernels must refuse
    for v in (binding.RMSNORM_VARIANT_WAVE, binding.RMSNORM_VARIANT_BLOCK):
        assert lib.rmsnorm_fwd_variant(P, P + 4096, P + 8192, 4, 7, 1e-6, 2, None, v) == \
            binding.RMSNORM_ERR_UNSUPPORTED
    # more than 1 KiB per row is too long for the several-rows-per-wavefront kernel
    assert lib.rmsnorm_fwd_variant(P, P + (1 << 20), P + (2 << 20), 4, 1024, 1e-6, 2, None,
                                   binding.RMSNORM_VARIANT_SUBWAVE) == binding.RMSNORM_ERR_UNSUPPORTED
    # too long for one wavefront's registers
    assert lib.rmsnorm_fwd_variant(P, P + (1 << 20), P + (2 << 20), 4, 8200, 1e-6, 2, None,
                                   binding.RMSNORM_VARIANT_WAVE) == binding.RMSNORM_ERR_UNSUPPORTED
    # misaligned base pointer
    assert lib.rmsnorm_fwd_variant(P + 2, P + 4096, P + 8192, 4, 8, 1e-6, 2, None,
                                   binding.RMSNORM_VARIANT_WAVE) == binding.RMSNORM_ERR_UNSUPPORTED
    # more than 1024 elements per row is too long for the LDS-staged kernel
    for dtype in (0, 1, 2):
        assert lib.rmsnorm_fwd_variant(P, P + (1 << 20), P + (2 << 20), 4, 1025, 1e-6, dtype, None,
                                       binding.RMSNORM_VARIANT_PACKED) == binding.RMSNORM_ERR_UNSUPPORTED
    assert lib.rmsnorm_fwd_variant(P, P + (1 << 20), P + (2 << 20), 0, 512, 1e-6, 2, None,
                                   binding.RMSNORM_VARIANT_PACKED) == binding.RMSNORM_OK


def test_tuned_entry_argument_checks():
    lib = binding.load()
    f = lib.rmsnorm_fwd_tuned
    big = 1 << 22
    for bad in (0, 4, 48, 96, 2048, -64):
        assert f(P, P + big, P + 2 * big, 4, 4096, 1e-6, 2, None, bad) == binding.RMSNORM_ERR_INVALID_ARG
    # 4096 bf16 = 512 vectors: 64 threads -> 8 chunks (ok); 16384 bf16 with 64 threads -> 32 (too many)
    assert f(P, P + big, P + 2 * big, 4, 16384, 1e-6, 2, None, 64) == binding.RMSNORM_ERR_UNSUPPORTED
    assert f(P, P + big, P + 2 * big, 4, 16384, 1e-6, 2, None, 128) == binding.RMSNORM_ERR_UNSUPPORTED
    assert f(P, P + big, P + 2 * big, 4, 1023, 1e-6, 2, None, 256) == binding.RMSNORM_ERR_UNSUPPORTED
    assert f(P, P + big, P + 2 * big, 0, 4096, 1e-6, 2, None, 256) == binding.RMSNORM_OK
    assert f(0, P + big, P + 2 * big, 4, 4096, 1e-6, 2, None, 256) == binding.RMSNORM_ERR_INVALID_ARG


def test_automatic_threads_per_row():
    auto = binding.rmsnorm_auto_threads_per_row
    bf16, fp16, fp32 = binding.RMSNORM_DTYPE_BF16, binding.RMSNORM_DTYPE_FP16, binding.RMSNORM_DTYPE_FP32
    assert auto(8192, bf16) == 512          # headline shape: 2 chunks per thread
    assert auto(4096, bf16) == 512          # exactly one vector per thread
    assert auto(4104, bf16) == 256 and auto(4088, bf16) == 256
    assert auto(2048, bf16) == 256 and auto(2040, bf16) == 64 and auto(2056, bf16) == 256
    assert auto(512, bf16) == 64
    assert auto(256, bf16) == 32
    assert auto(128, bf16) == 16
    assert auto(64, fp16) == 8
    # aligned rows that the automatic path sends through LDS report 1 (RMSNORM_VARIANT_PACKED):
    # rows of at most 64 bytes, and 5 vectors on 8 lanes, 9 or 10 on 16
    assert auto(8, fp16) == 1 and auto(32, bf16) == 1 and auto(16, fp32) == 1 and auto(40, bf16) == 1
    assert auto(40, fp16) == 1 and auto(72, bf16) == 1 and auto(80, fp16) == 1 and auto(96, fp16) == 16
    assert auto(48, bf16) == 8 and auto(24, fp32) == 8
    assert auto(128, fp32) == 32
    assert auto(192, bf16) == 32            # 384 bytes: three whole lines
    # rows that are a multiple of 16 bytes but not of the 128-byte line, beyond 256 bytes: through
    # LDS up to 2 KiB (1), then the element-addressed kernel's thread counts
    assert auto(200, bf16) == 1 and auto(136, fp16) == 1 and auto(1000, fp16) == 1 and auto(260, fp32) == 1
    assert auto(1032, fp16) == 64 and auto(2040, bf16) == 64 and auto(4088, bf16) == 256 and auto(8184, fp16) == 256
    assert auto(16392, bf16) == 512 and auto(131064, bf16) == 1024
    assert auto(1024, fp32) == 256 and auto(2048, fp32) == 512 and auto(1020, fp32) == 64
    assert auto(768, fp16) == 64
    assert auto(5120, fp16) == 256
    assert auto(5632, fp16) == 256 and auto(5696, fp16) == 512
    assert auto(13824, fp16) == 512
    assert auto(8192, fp32) == 512
    assert auto(16384, bf16) == 512 and auto(16448, bf16) == 1024
    assert auto(32768, bf16) == 1024
    assert auto(65536, fp16) == 1024
    assert auto(131072, bf16) == 1024
    assert auto(131080, bf16) == 0          # too long for registers
    assert auto(1023, bf16) == 0            # rows not 16-byte aligned
    with pytest.raises(binding.RmsnormError):
        auto(0, bf16)
    with pytest.raises(binding.RmsnormError):
        auto(64, 7)


def test_dispatch_choice_is_visible_without_a_launch():
    lib = binding.load()
    sel = lib.rmsnorm_select_variant
    assert sel(P, P + 65536, P + 131072, 16, 8192, 2) == binding.RMSNORM_VARIANT_BLOCK
    assert sel(P, P + 65536, P + 131072, 16, 768, 1) == binding.RMSNORM_VARIANT_WAVE
    assert sel(P, P + 65536, P + 131072, 16, 13824, 1) == binding.RMSNORM_VARIANT_BLOCK
    assert sel(P, P + 65536, P + 131072, 16, 1984, 2) == binding.RMSNORM_VARIANT_WAVE
    # 16-byte aligned rows beyond 256 bytes that are not whole 128-byte lines: through LDS up to
    # 2 KiB, the element-addressed kernel beyond, also where the work-queue kernel would run
    assert sel(P, P + 65536, P + 131072, 16, 2040, 2) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 200, 2) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 1000, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 1032, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 260, 0) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + (1 << 22), P + (1 << 30), 16384, 8184, 2) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + (1 << 22), P + (1 << 30), 16384, 8192, 2) == binding.RMSNORM_VARIANT_QUEUE
    assert lib.rmsnorm_queue_plan(16384, 8184, 2, None, None, None, None) == 0
    assert sel(P, P + 65536, P + 131072, 16, 136, 1) == binding.RMSNORM_VARIANT_PACKED
    # whole-line rows of 2 KiB and more written to a y that starts off the 64-byte pieces of the
    # lines: element-addressed too
    assert sel(P, P + (1 << 22), P + (1 << 30) + 16, 16384, 8192, 2) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P + 16, P + (1 << 22), P + (1 << 30), 16384, 8192, 2) == binding.RMSNORM_VARIANT_QUEUE
    assert sel(P, P + (1 << 22), P + (1 << 30) + 64, 16384, 8192, 2) == binding.RMSNORM_VARIANT_QUEUE
    assert sel(P, P + (1 << 22), P + (1 << 30) + 48, 16, 1024, 2) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + (1 << 22), P + (1 << 30) + 48, 16, 512, 2) == binding.RMSNORM_VARIANT_WAVE
    # rows of whole half lines: through LDS while short, the aligned kernels beyond
    assert sel(P, P + 65536, P + 131072, 16, 544, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 2080, 1) == binding.RMSNORM_VARIANT_BLOCK
    assert sel(P, P + 65536, P + 131072, 16, 2072, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 120, 1) == binding.RMSNORM_VARIANT_SUBWAVE   # 240 bytes: below the rule
    assert sel(P, P + 65536, P + 131072, 16, 128, 2) == binding.RMSNORM_VARIANT_SUBWAVE
    assert sel(P, P + 65536, P + 131072, 16, 48, 2) == binding.RMSNORM_VARIANT_SUBWAVE
    assert sel(P, P + 65536, P + 131072, 16, 40, 2) == binding.RMSNORM_VARIANT_PACKED   # 5 vectors on 8 lanes
    assert sel(P, P + 65536, P + 131072, 16, 72, 1) == binding.RMSNORM_VARIANT_PACKED   # 9 vectors on 16 lanes
    assert sel(P, P + 65536, P + 131072, 16, 96, 1) == binding.RMSNORM_VARIANT_SUBWAVE
    # aligned rows of at most 64 bytes go through LDS like the unaligned ones
    assert sel(P, P + 65536, P + 131072, 16, 32, 2) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 8, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 16, 0) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 24, 0) == binding.RMSNORM_VARIANT_SUBWAVE
    assert sel(P, P + 65536, P + 131072, 16, 1023, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 4097, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P + 2, P + 65536, P + 131072, 16, 2048, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 1025, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 513, 1) == binding.RMSNORM_VARIANT_PACKED
    # short rows that are not 16-byte aligned go through LDS several at a time
    assert sel(P, P + 65536, P + 131072, 16, 511, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P + 2, P + 65536, P + 131072 + 18, 16, 512, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P + 2, P + 65536, P + 131072, 16, 512, 1) == binding.RMSNORM_VARIANT_PACKED  # x - y not a multiple of 16
    # only y off a boundary: rows of 1 KiB and more keep the register kernel (aligned loads)
    assert sel(P, P + 65536, P + 131072 + 2, 16, 512, 1) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072 + 2, 16, 504, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072 + 4, 16, 256, 0) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536 + 2, P + 131072 + 2, 16, 512, 1) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 197, 2) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 3, 0) == binding.RMSNORM_VARIANT_PACKED
    assert sel(P, P + 65536, P + 131072, 16, 512, 1) == binding.RMSNORM_VARIANT_WAVE
    assert sel(P, P + 65536, P + 131072, 16, 131079, 2) == binding.RMSNORM_VARIANT_UNALIGNED
    assert sel(P, P + 65536, P + 131072, 16, 131081, 2) == binding.RMSNORM_VARIANT_STREAM
    assert sel(P, P + 65536, P + 131072, 16, 1 << 20, 2) == binding.RMSNORM_VARIANT_STREAM
    assert sel(P, P + 65536, P + (1 << 33), 2, 1 << 31, 2) == binding.RMSNORM_VARIANT_GENERIC
    assert sel(P, P + 65536, P + 131072, 16, 0, 2) == binding.RMSNORM_ERR_INVALID_ARG


def test_unaligned_walk_grid_query():
    """The grid of the walking form: a multiple of the compute units (256 without a device) near
    26 KiB of rows in flight per compute unit, chosen so that the rows divide evenly; 0 where
    the one-row-per-workgroup form runs."""
    lib = binding.load()
    X, W, Y = P, P + (1 << 30), P + (2 << 30)
    q = lib.rmsnorm_unaligned_walk_grid
    assert q(X, W, Y, 8192, 4097, 1) == 1024 and q(X, W, Y, 16384, 8191, 2) == 512
    assert q(X, W, Y, 16384, 1025, 1) == 13 * 256 and q(X, W, Y, 8191, 1537, 1) == 8 * 256
    assert q(X, W, Y, 3000, 4097, 1) == 768 and q(X, W, Y, 4096, 20481, 2) == 256
    assert q(X + 6, W + 2, Y + 22, 8192, 4097, 1) == 1024      # same offset from a line
    assert q(X, W, Y + 2, 8192, 4097, 1) == 1024               # different offsets: cut at x's lines
    assert q(X, W, Y, 8192, 4097, 0) == 512 and q(X, W, Y, 16384, 4097, 0) == 512   # fp32 walks too
    # two or three rows per workgroup are enough where the grid is close to the best one
    assert q(X, W, Y, 2048, 4097, 1) == 1024 and q(X, W, Y, 1024, 8191, 2) == 512
    assert q(X, W, Y, 1500, 4097, 1) == 0 and q(X, W, Y, 768, 8191, 2) == 0    # too few rows
    assert q(X, W, Y, 1061, 131079, 1) == 0                    # more than 8 groups per thread
    assert q(X, W, Y, 1061, 57343, 1) == 256 and q(X, W, Y, 1061, 65535, 1) == 0   # 1024 threads: 7
    assert q(X, W, Y, 4, 1 << 20, 1) == 0                      # does not fit in registers
    assert q(X, W, Y, 0, 4097, 1) == 0
    assert q(X, W, Y, 8192, 0, 1) == binding.RMSNORM_ERR_INVALID_ARG
    assert q(X, W, Y, 8192, 4097, 7) == binding.RMSNORM_ERR_INVALID_ARG
    assert q(0, W, Y, 8192, 4097, 1) == binding.RMSNORM_ERR_INVALID_ARG


def test_queue_plan_and_dispatch_threshold():
    """The work-queue kernel's launch shape and the sizes at which the automatic path takes it,
    without a launch (off a GPU machine the library assumes MI355X's 256 compute units)."""
    bf16, fp32 = binding.RMSNORM_DTYPE_BF16, binding.RMSNORM_DTYPE_FP32
    takes, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(16384, 8192, bf16)
    assert takes and (grid, shards, block_rows, prefetch) == (512, 16, 8, False)
    assert grid % shards == 0
    takes, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(16384, 16384, bf16)
    assert takes and (grid, shards, block_rows, prefetch) == (512, 8, 4, False)
    takes, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(16384, 20480, bf16)
    assert takes and (grid, shards, block_rows, prefetch) == (256, 8, 2, True)
    assert binding.rmsnorm_queue_plan(3276, 20480, bf16)[0] is False      # 128 MiB of 40 KiB rows
    takes, grid, shards, block_rows, prefetch = binding.rmsnorm_queue_plan(16384, 4096, fp32)
    assert takes and (grid, shards, block_rows, prefetch) == (512, 16, 8, False)
    # a block is the largest power of two of rows within 128 KiB
    assert binding.rmsnorm_queue_plan(100000, 5120, bf16)[3] == 8        # 10 KiB rows
    assert binding.rmsnorm_queue_plan(100000, 32768, bf16)[3] == 2       # 64 KiB rows
    # small launches stay with one workgroup per row; rows under 16 KiB take the kernel from 320 MiB on
    assert binding.rmsnorm_queue_plan(4096, 8192, bf16)[0] is False
    assert binding.rmsnorm_queue_plan(6144, 8192, bf16)[0] is True
    assert binding.rmsnorm_queue_plan(32767, 5120, bf16)[0] is False
    assert binding.rmsnorm_queue_plan(32768, 5120, bf16)[0] is True
    assert binding.rmsnorm_queue_plan(1 << 20, 4160, bf16)[0] is True      # 8320 bytes: 65 lines
    assert binding.rmsnorm_queue_plan(40000, 4160, bf16)[0] is False
    # rows that are not whole 128-byte lines never: the element-addressed kernel takes those
    assert binding.rmsnorm_queue_plan(1 << 20, 4104, bf16)[0] is False
    assert binding.rmsnorm_queue_plan(16384, 8184, bf16)[0] is False
    lib = binding.load()
    plan = lib.rmsnorm_queue_plan
    assert plan(16, 4096, bf16, None, None, None, None) == binding.RMSNORM_ERR_UNSUPPORTED   # 512 vectors
    assert plan(16, 32776, bf16, None, None, None, None) == binding.RMSNORM_ERR_UNSUPPORTED  # 4097 vectors
    assert plan(16, 8191, bf16, None, None, None, None) == binding.RMSNORM_ERR_UNSUPPORTED   # not aligned
    assert plan(1 << 30, 8192, bf16, None, None, None, None) == binding.RMSNORM_ERR_UNSUPPORTED
    assert plan(16, 8192, 7, None, None, None, None) == binding.RMSNORM_ERR_INVALID_ARG
    assert plan(-1, 8192, bf16, None, None, None, None) == binding.RMSNORM_ERR_INVALID_ARG
    sel = lib.rmsnorm_select_variant
    assert sel(P, P + 65536, P + 131072, 16384, 8192, 2) == binding.RMSNORM_VARIANT_QUEUE
    assert sel(P, P + 65536, P + 131072, 4096, 8192, 2) == binding.RMSNORM_VARIANT_BLOCK
    assert sel(P, P + 65536, P + 131072, 16384, 4096, 2) == binding.RMSNORM_VARIANT_BLOCK   # 8 KiB rows
    assert sel(P, P + 65536, P + 131072 + 2, 16384, 8192, 2) == binding.RMSNORM_VARIANT_UNALIGNED


def test_workspace_entry_argument_checks():
    lib = binding.load()
    assert binding.rmsnorm_workspace_bytes() == 4096
    f = lib.rmsnorm_fwd_workspace
    W = P + (1 << 24)
    assert f(P, P + 65536, P + 131072, 4, 8192, 1e-6, 2, None, None, 4096) == binding.RMSNORM_ERR_INVALID_ARG
    assert f(P, P + 65536, P + 131072, 4, 8192, 1e-6, 2, None, W, 4095) == binding.RMSNORM_ERR_INVALID_ARG
    assert f(P, P + 65536, P + 131072, 4, 8192, 1e-6, 2, None, W + 2, 8192) == binding.RMSNORM_ERR_INVALID_ARG
    assert f(P, P + 65536, P + 131072, 4, 4096, 1e-6, 2, None, W, 4096) == binding.RMSNORM_ERR_UNSUPPORTED
    assert f(P, P + 65536, P + 131072, 4, 8191, 1e-6, 2, None, W, 4096) == binding.RMSNORM_ERR_UNSUPPORTED
    assert f(P, P + 65536, P + 131072, 0, 8192, 1e-6, 2, None, W, 4096) == binding.RMSNORM_OK
    assert f(None, P + 65536, P + 131072, 4, 8192, 1e-6, 2, None, W, 4096) == binding.RMSNORM_ERR_INVALID_ARG
    g = lib.rmsnorm_fwd_queue_tuned
    for grid, shards, block_rows in [(10, 16, 8), (48, 32, 8), (64, 0, 8), (64, 33, 8), (64, 16, 3),
                                     (64, 16, 0), (0, 1, 1), (1 << 17, 1, 1), (64, 16, 1 << 17)]:
        assert g(P, P + 65536, P + 131072, 4, 8192, 1e-6, 2, None, W, 4096, grid, shards, block_rows, 0) == \
            binding.RMSNORM_ERR_INVALID_ARG, (grid, shards, block_rows)


def test_thread_count_follows_the_batch_size():
    """Batches of one to three rounds of resident workgroups run with narrower workgroups when
    the whole batch then fits on the GPU at once (256 compute units assumed off a GPU machine: a
    round is 1024 workgroups of 512 threads, 2048 of 256, 4096 of 128)."""
    f = binding.rmsnorm_auto_threads_for_batch
    bf16, fp16, fp32 = binding.RMSNORM_DTYPE_BF16, binding.RMSNORM_DTYPE_FP16, binding.RMSNORM_DTYPE_FP32
    # N = 8192 in a 16-bit type: 1024 vectors, 512 threads by default
    assert [f(M, 8192, bf16) for M in (1, 1024, 1025, 1536, 2048, 2049, 3072, 3073, 16384)] == \
        [512, 512, 256, 256, 256, 512, 512, 512, 512]                      # 128 threads would need 8 chunks
    # N = 4096: 512 vectors
    assert [f(M, 4096, fp16) for M in (1024, 1025, 2048, 2049, 3072, 3073, 4096)] == \
        [512, 256, 256, 128, 128, 512, 512]
    # N = 2048: 256 vectors, 256 threads by default, a round of 2048
    assert [f(M, 2048, bf16) for M in (2048, 2049, 4096, 4097, 6144, 6145)] == [256, 128, 128, 256, 256, 256]
    assert f(1536, 4096, fp32) == 256 and f(3000, 2048, fp32) == 128
    # rows that need more than 4 chunks in the narrower workgroup keep the default
    assert f(3000, 5120, bf16) == 256 and f(1200, 32768, bf16) == 1024
    # rows of one wavefront or less, and the special return codes, pass through
    for N in (512, 128, 40, 8, 1023, 131080):
        assert f(5000, N, bf16) == binding.rmsnorm_auto_threads_per_row(N, bf16)
    with pytest.raises(binding.RmsnormError):
        f(-1, 8192, bf16)
    with pytest.raises(binding.RmsnormError):
        f(16, 0, bf16)
