"""GPU parity tests of the LDS-staged kernels for short rows that are not 16-byte aligned
(several rows per workgroup): odd lengths from 1 to 1024 (attention rows of 77, 197, 257
entries), row counts that end inside a tile, inside a lane-group pass and inside a
wavefront, base pointers off a 16-byte boundary, in place, and aligned shapes forced onto
the kernel.  Each output is compared with the CPU oracle element by element, and the
guard elements around y must stay untouched."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import binding, inputs

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
# every lane-group size (1, 2, 4 ... 64 lanes of up to 16 elements) at its limits and inside
LENGTHS = [1, 3, 7, 16, 17, 31, 32, 33, 50, 63, 64, 65, 77, 127, 129, 197, 255, 257, 300, 511, 512, 513, 777, 1023, 1024]


def offset_view(a, dtype, device, off, shape):
    """The array on the device, `off` elements past a 16-byte boundary."""
    buf = torch.zeros(a.size + 16, dtype=H.torch_dtype(dtype), device=device)
    view = buf[off:off + a.size].view(*shape)
    view.copy_(H.to_device(a.reshape(shape), dtype, device))
    return view


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", LENGTHS)
def test_rmsnorm_packed_lengths(gpu_device, N, dtype):
    rows_per_tile = 16384 // (N * inputs.DTYPE_BYTES[dtype])
    M = 2 * rows_per_tile + 5 if rows_per_tile < 3000 else 4099     # two full tiles and a partial one
    case = inputs.random_case(6, 900 + 2 * dtype, M, N, dtype, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, dtype)
    H.check_case(case, gpu_device, variants=(binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_PACKED,
                                             binding.RMSNORM_VARIANT_GENERIC), want=want)
    # x and y the same distance off a 16-byte boundary (w anywhere): still the LDS-staged kernel
    per16 = 16 // inputs.DTYPE_BYTES[dtype]
    xd = offset_view(case["x"], dtype, gpu_device, 1, (M, N))
    wd = offset_view(case["w"], dtype, gpu_device, 3, (N,))
    for mode in (binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_PACKED):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1 + per16)
        H.say(f"rmsnorm packed offset bases {inputs.DTYPE_NAMES[dtype]} {M}x{N} mode={mode}")
        binding.rmsnorm_fwd_variant(xd, wd, 1e-6, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=1 + per16)
        compare.check_parity(H.to_host(y, dtype), want, dtype, f"packed offset bases mode {mode}")
    assert binding.rmsnorm_select_variant(xd, wd, y) == binding.RMSNORM_VARIANT_PACKED
    # x and y at different distances: the same kernel, with element-aligned stores
    for mode in (binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_PACKED):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=2)
        assert binding.rmsnorm_select_variant(xd, wd, y) == binding.RMSNORM_VARIANT_PACKED
        binding.rmsnorm_fwd_variant(xd, wd, 1e-6, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=2)
        compare.check_parity(H.to_host(y, dtype), want, dtype, "x and y at different offsets")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M", [1, 2, 31, 33, 64, 1000])
def test_rmsnorm_packed_row_counts(gpu_device, M, dtype):
    """Fewer rows than a tile, than a pass of the lane groups, than a wavefront."""
    N = 77
    case = inputs.random_case(6, 920 + 2 * dtype, M, N, dtype, 1e-5)
    H.check_case(case, gpu_device, variants=(binding.RMSNORM_VARIANT_AUTO, binding.RMSNORM_VARIANT_PACKED))


@pytest.mark.parametrize("dtype", DTYPES)
def test_rmsnorm_packed_in_place_and_deterministic(gpu_device, dtype):
    M, N = 3001, 197
    case = inputs.random_case(6, 940 + 2 * dtype, M, N, dtype, 1e-6)
    want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, dtype)
    wd = H.to_device(case["w"], dtype, gpu_device)
    xd = H.to_device(case["x"], dtype, gpu_device)
    first = H.to_host(binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_PACKED), dtype).copy()
    compare.check_parity(first, want, dtype, "packed")
    for _ in range(2):
        again = H.to_host(binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_PACKED), dtype)
        assert np.array_equal(again.view(np.uint8), first.view(np.uint8))
    H.say("rmsnorm packed in place")
    binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_PACKED, xd)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(xd, dtype).view(np.uint8), first.view(np.uint8))


def test_rmsnorm_packed_more_tiles_than_the_grid(gpu_device):
    """The grid stops at 8192 workgroups; with 8 rows of 2 KiB per tile, 65536 + 13 rows are 8194
    tiles: the workgroups take two tiles each, the last of them a partial one, and some only one."""
    M, N = 8192 * 8 + 13, 511
    case = inputs.random_case(6, 960, M, N, inputs.FP32, 1e-6)
    H.check_case(case, gpu_device, variants=(binding.RMSNORM_VARIANT_PACKED,))


# ---- softmax -----------------------------------------------------------------------------------
import test_softmax_gpu as SM
from paper_2603_21331_amd import softmax


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", LENGTHS)
def test_softmax_packed_lengths(gpu_device, N, dtype):
    rows_per_tile = 16384 // (N * inputs.DTYPE_BYTES[dtype])
    M = 2 * rows_per_tile + 5 if rows_per_tile < 3000 else 4099
    case = inputs.softmax_case(6, 1000 + 2 * dtype, M, N, dtype, 2.5)
    if N > 2:                       # masked scores and one fully masked row (NaN by definition)
        neg_inf = {inputs.FP32: np.float32(-np.inf), inputs.FP16: 0xFC00, inputs.BF16: 0xFF80}[dtype]
        case["x"][::5, N // 2] = neg_inf
        case["x"][7, :] = neg_inf
    want = oracle.softmax_oracle(case["x"], dtype)
    SM.check(case, gpu_device, modes=(0, softmax.SOFTMAX_VARIANT_PACKED, softmax.SOFTMAX_VARIANT_GENERIC), want=want)
    per16 = 16 // inputs.DTYPE_BYTES[dtype]
    xd = offset_view(case["x"], dtype, gpu_device, 1, (M, N))
    for mode in (0, softmax.SOFTMAX_VARIANT_PACKED):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1 + 2 * per16)
        H.say(f"softmax packed offset bases {inputs.DTYPE_NAMES[dtype]} {M}x{N} mode={mode}")
        softmax.softmax_fwd_variant(xd, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=1 + 2 * per16)
        compare.check_softmax_parity(H.to_host(y, dtype), want, dtype, f"softmax packed offset bases mode {mode}")
    for mode in (0, softmax.SOFTMAX_VARIANT_PACKED):     # the same kernel, element-aligned stores
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=2)
        softmax.softmax_fwd_variant(xd, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=2)
        compare.check_softmax_parity(H.to_host(y, dtype), want, dtype, "softmax, x and y at different offsets")


@pytest.mark.parametrize("dtype", DTYPES)
def test_softmax_packed_attention_shapes_in_place(gpu_device, dtype):
    """Square attention-score blocks with odd context lengths, in place, twice for determinism."""
    for n in (77, 197, 257):
        M = 12 * n
        case = inputs.softmax_case(6, 1020 + 2 * dtype, M, n, dtype, 3.0)
        want = oracle.softmax_oracle(case["x"], dtype)
        xd = H.to_device(case["x"], dtype, gpu_device)
        first = H.to_host(softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_PACKED), dtype).copy()
        compare.check_softmax_parity(first, want, dtype, f"softmax packed {n}")
        again = H.to_host(softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_PACKED), dtype)
        assert np.array_equal(again.view(np.uint8), first.view(np.uint8))
        H.say(f"softmax packed in place n={n}")
        softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_PACKED, xd)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_host(xd, dtype).view(np.uint8), first.view(np.uint8))


def test_softmax_packed_more_tiles_than_the_grid(gpu_device):
    """The grid stops at 32768 workgroups; fp16 rows of 1001 elements go 4 to a tile, so
    131072 + 13 rows are 32772 tiles: two for most workgroups, the last of all a partial one."""
    M, N = 32768 * 4 + 13, 1001
    case = inputs.softmax_case(6, 1030, M, N, inputs.FP16, 2.0)
    SM.check(case, gpu_device, modes=(0, softmax.SOFTMAX_VARIANT_PACKED))


# ---- LayerNorm ---------------------------------------------------------------------------------
import test_layernorm_gpu as LN
from paper_2603_21331_amd import layernorm


def test_layernorm_packed_more_tiles_than_the_grid(gpu_device):
    """The grid stops at 4096 workgroups; with 8 rows of 2 KiB per tile, 32768 + 13 rows are 4098
    tiles: two for most workgroups (weight and bias fetched once, the second tile requested while
    the first is worked on), the last of all a partial one."""
    M, N = 4096 * 8 + 13, 511
    case = inputs.layernorm_case(6, 1080, M, N, inputs.FP32, 1e-5, mean=1.0, std=2.0)
    LN.check(case, gpu_device, modes=(0, layernorm.LAYERNORM_VARIANT_PACKED))


@pytest.mark.parametrize("bias", [True, False])
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", LENGTHS)
def test_layernorm_packed_lengths(gpu_device, N, dtype, bias):
    rows_per_tile = 16384 // (N * inputs.DTYPE_BYTES[dtype])
    M = 2 * rows_per_tile + 5 if rows_per_tile < 3000 else 4099
    case = inputs.layernorm_case(6, 1040 + 4 * dtype, M, N, dtype, 1e-5, mean=3.0, std=2.0, bias=bias)
    LN.check(case, gpu_device, modes=(0, layernorm.LAYERNORM_VARIANT_PACKED, layernorm.LAYERNORM_VARIANT_GENERIC))


@pytest.mark.parametrize("dtype", DTYPES)
def test_layernorm_packed_offset_bases_and_in_place(gpu_device, dtype):
    M, N = 3001, 197
    case = inputs.layernorm_case(6, 1060 + 4 * dtype, M, N, dtype, 1e-5, mean=-2.0, std=0.5)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    bias64 = LN.scale_of(case, mean, rstd)
    per16 = 16 // inputs.DTYPE_BYTES[dtype]
    xd = offset_view(case["x"], dtype, gpu_device, 3, (M, N))
    wd = offset_view(case["w"], dtype, gpu_device, 1, (N,))
    bd = offset_view(case["b"], dtype, gpu_device, 2, (N,))
    for mode in (0, layernorm.LAYERNORM_VARIANT_PACKED):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=3 + per16)
        H.say(f"layernorm packed offset bases {inputs.DTYPE_NAMES[dtype]} mode={mode}")
        layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=3 + per16)
        compare.check_layernorm_parity(H.to_host(y, dtype), want, bias64, dtype, f"layernorm packed offset mode {mode}")
    first = H.to_host(y, dtype).copy()
    for mode in (0, layernorm.LAYERNORM_VARIANT_PACKED):  # y at another offset: element-aligned stores
        whole, y2 = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1)
        layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, mode, y2)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=1)
        compare.check_layernorm_parity(H.to_host(y2, dtype), want, bias64, dtype, "layernorm, y at another offset")
    H.say("layernorm packed in place")
    layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, layernorm.LAYERNORM_VARIANT_PACKED, xd)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(xd, dtype).view(np.uint8), first.view(np.uint8))


# ---- every row length, every instantiation ---------------------------------------------------
# Lane groups of 1 to 64 lanes with 1 to 16 elements per lane are separate instantiations; the
# lengths 1 .. 1024 visit every one of them, with the row ending at every position of a lane's
# last step.  37 rows: more than a pass of the widest groups, fewer than one of the narrowest.
from paper_2603_21331_amd import crossentropy as ce, rowsum as rs

ALL_LENGTHS = list(range(1, 1025))


@pytest.mark.parametrize("dtype", DTYPES)
def test_rmsnorm_packed_every_length(gpu_device, dtype):
    M = 37
    for N in ALL_LENGTHS:
        case = inputs.random_case(7, 1100 + 2 * dtype, M, N, dtype, 1e-6)
        want = oracle.rmsnorm_oracle(case["x"], case["w"], 1e-6, dtype)
        xd, wd = H.to_device(case["x"], dtype, gpu_device), H.to_device(case["w"], dtype, gpu_device)
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
        H.say(f"rmsnorm packed every length: {inputs.DTYPE_NAMES[dtype]} N={N}")
        binding.rmsnorm_fwd_variant(xd, wd, 1e-6, binding.RMSNORM_VARIANT_PACKED, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), f"N={N}: wrote outside y"
        compare.check_parity(H.to_host(y, dtype), want, dtype, f"rmsnorm packed N={N}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_softmax_packed_every_length(gpu_device, dtype):
    M = 37
    for N in ALL_LENGTHS:
        case = inputs.softmax_case(7, 1120 + 2 * dtype, M, N, dtype, 2.0)
        want = oracle.softmax_oracle(case["x"], dtype)
        xd = H.to_device(case["x"], dtype, gpu_device)
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
        H.say(f"softmax packed every length: {inputs.DTYPE_NAMES[dtype]} N={N}")
        softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_PACKED, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), f"N={N}: wrote outside y"
        compare.check_softmax_parity(H.to_host(y, dtype), want, dtype, f"softmax packed N={N}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_layernorm_packed_every_length(gpu_device, dtype):
    M = 37
    for N in ALL_LENGTHS:
        case = inputs.layernorm_case(7, 1140 + 4 * dtype, M, N, dtype, 1e-5, mean=1.0, std=2.0)
        want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
        bias64 = LN.scale_of(case, mean, rstd)
        xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device)
        H.say(f"layernorm packed every length: {inputs.DTYPE_NAMES[dtype]} N={N}")
        layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, layernorm.LAYERNORM_VARIANT_PACKED, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), f"N={N}: wrote outside y"
        compare.check_layernorm_parity(H.to_host(y, dtype), want, bias64, dtype, f"layernorm packed N={N}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_crossentropy_and_rowsum_packed_every_length(gpu_device, dtype):
    M = 37
    for N in ALL_LENGTHS:
        case = inputs.crossentropy_case(7, 1160 + 4 * dtype, M, N, dtype, 2.0, ignore_every=9)
        t = np.asarray(case["target"], dtype=np.int64)
        want_loss = oracle.crossentropy_oracle(case["x"], t, dtype)
        want_sum, want_abs = oracle.rowsum_oracle(case["x"], dtype, with_abs=True)
        xd = H.to_device(case["x"], dtype, gpu_device)
        td = torch.from_numpy(t).to(gpu_device)
        H.say(f"cross-entropy and row sum packed every length: {inputs.DTYPE_NAMES[dtype]} N={N}")
        loss = ce.crossentropy_fwd_tuned(xd, td, 2)
        total = rs.rowsum_fwd_tuned(xd, 2)
        torch.cuda.synchronize()
        compare.check_crossentropy_parity(loss.cpu().numpy(), want_loss, f"cross-entropy packed N={N}",
                                          exact_zero=(t < 0) | (t >= N))
        compare.check_rowsum_parity(total.cpu().numpy(), want_sum, want_abs, N, f"row sum packed N={N}")
