"""GPU parity tests of LayerNorm forward against its CPU oracle, through the C ABI: the paper's
five stages (Section 4) in compact form.  Its stability probe for normalisations is near-zero
variance; rows with a mean far larger than their spread are added."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import inputs, layernorm

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
THREADS = (8, 16, 32, 64, 256, 512, 1024)
MODES = (0, 1, 2, 3, 4, 5, 6, 7, 8) + tuple(("threads", g) for g in THREADS)


def mode_name(m):
    return f"threads{m[1]}" if isinstance(m, tuple) else layernorm.VARIANT_NAMES[m]


def launch(xd, wd, bd, eps, mode, y):
    if isinstance(mode, tuple):
        return layernorm.layernorm_fwd_tuned(xd, wd, bd, eps, mode[1], y)
    return layernorm.layernorm_fwd_variant(xd, wd, bd, eps, mode, y)


def scale_of(case, mean, rstd):
    dtype = case["dtype"]
    return compare.layernorm_scale(inputs.storage_to_f64(case["x"], dtype), inputs.storage_to_f64(case["w"], dtype),
                                   None if case["b"] is None else inputs.storage_to_f64(case["b"], dtype), mean, rstd)


def check(case, device, modes=MODES, want=None):
    dtype, eps = case["dtype"], case["eps"]
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], eps, dtype, stats=True)
    xd = H.to_device(case["x"], dtype, device)
    wd = H.to_device(case["w"], dtype, device)
    bd = None if case["b"] is None else H.to_device(case["b"], dtype, device)
    bias64 = scale_of(case, mean, rstd)
    M, N = case["x"].shape
    stats, ran = {}, 0
    for m in modes:
        whole, y = H.alloc_guarded(M, N, dtype, device)
        H.say(f"{case['name']}: {inputs.DTYPE_NAMES[dtype]} {M}x{N} bias={bd is not None} mode={mode_name(m)}")
        try:
            launch(xd, wd, bd, eps, m, y)
        except layernorm.LayerNormError as e:
            if e.status == layernorm.LAYERNORM_ERR_UNSUPPORTED and m != 0:
                continue
            raise
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype), "wrote outside y"
        ran += 1
        stats[mode_name(m)] = compare.check_layernorm_parity(H.to_host(y, dtype), want, bias64, dtype,
                                                             f"{case['name']} [{mode_name(m)}]")
    assert ran >= 2
    return stats


@pytest.mark.parametrize("dtype", DTYPES)
def test_smoke_128x128(gpu_device, dtype):
    check(inputs.layernorm_case(0, 1400 + 4 * dtype, 128, 128, dtype), gpu_device)


SWEEP = [("tiny", 70, 8), ("head_64", 1031, 64), ("dim_128", 4099, 128), ("dim_200", 333, 200),
         ("dim_512", 515, 512), ("ragged_1000", 301, 1000), ("dim_2048", 517, 2048),
         ("standard_4096", 1024, 4096), ("hidden_5120", 259, 5120), ("wide_8192", 259, 8192),
         ("wide_16384", 67, 16384), ("limit_16bit", 9, 65536), ("past_limit", 5, 65544), ("long_131072", 5, 131072),
         ("long_odd_262145", 3, 262145), ("tall", 8192, 1024)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("name,M,N", SWEEP, ids=[s[0] for s in SWEEP])
def test_shape_sweep(gpu_device, name, M, N, dtype):
    check(inputs.layernorm_case(1, 1410 + 4 * dtype, M, N, dtype, mean=0.3, std=1.5), gpu_device)


@pytest.mark.parametrize("which", [0, 1])
def test_paper_result_shapes_fp16(gpu_device, which):
    stats = check(inputs.layernorm_paper_shape(which), gpu_device)
    H.say(f"layernorm paper shape {which} stats {stats}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_no_bias(gpu_device, dtype):
    check(inputs.layernorm_case(2, 1420 + 4 * dtype, 300, 4096, dtype, bias=False), gpu_device)
    check(inputs.layernorm_case(2, 1424 + 4 * dtype, 300, 128, dtype, bias=False), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
def test_near_zero_variance_and_large_mean(gpu_device, dtype):
    """Constant rows (variance exactly zero: the output must be the bias), rows whose spread is
    tiny against their mean, rows of tiny values, a row with one outlier in first position (the
    shift the kernel uses), and large magnitudes."""
    N = 2048
    z = inputs.normal(3, 1430, 0, 8 * N).reshape(8, N)
    far = {inputs.FP32: (1000.0, 0.01), inputs.FP16: (100.0, 0.5), inputs.BF16: (100.0, 4.0)}[dtype]
    z[0] = 0.75
    z[1] = 0.0
    z[2] = far[0] + far[1] * z[2]
    z[3] *= {inputs.FP32: 1e-20, inputs.FP16: 1e-4, inputs.BF16: 1e-20}[dtype]
    z[4, 0] = {inputs.FP32: 1e6, inputs.FP16: 3e4, inputs.BF16: 1e6}[dtype]
    z[5] *= {inputs.FP32: 1e15, inputs.FP16: 1e3, inputs.BF16: 1e15}[dtype]
    z[6] = -far[0] + far[1] * z[6]
    c = inputs.layernorm_case(3, 1434, 1, N, dtype)
    case = dict(name="stability", dtype=dtype, M=8, N=N, eps=1e-5, x=inputs.to_storage(z, dtype), w=c["w"], b=c["b"])
    want = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype)
    assert np.array_equal(want[0], case["b"]) and np.array_equal(want[1], case["b"])
    check(case, gpu_device, want=want)


def test_determinism_and_row_independence(gpu_device):
    case = inputs.layernorm_case(4, 1440, 777, 5120, inputs.FP16)
    xd, wd, bd = (H.to_device(case[k], inputs.FP16, gpu_device) for k in ("x", "w", "b"))
    for m in MODES:
        H.say(f"layernorm determinism mode={mode_name(m)}")
        y = torch.empty_like(xd)
        try:
            launch(xd, wd, bd, 1e-5, m, y)
        except layernorm.LayerNormError as e:
            if e.status == layernorm.LAYERNORM_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        first = H.to_host(y, inputs.FP16).copy()
        for _ in range(2):
            launch(xd, wd, bd, 1e-5, m, y)
            torch.cuda.synchronize()
            assert np.array_equal(H.to_host(y, inputs.FP16), first)
        fresh = torch.empty_like(xd)
        launch(xd, wd, bd, 1e-5, m, fresh)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_host(fresh, inputs.FP16), first)
        if m != 0:
            for i in (0, 333, 776):
                one = H.to_host(launch(xd[i:i + 1], wd, bd, 1e-5, m, None), inputs.FP16)
                assert np.array_equal(one[0], first[i])


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1023, 1023), (33, 4097), (129, 1537), (1, 1), (7, 1), (2, 3), (1, 8),
                                 (5, 12), (3, 40001), (1, 8192)])
def test_edge_dims(gpu_device, M, N, dtype):
    check(inputs.layernorm_case(5, 1450 + 4 * dtype, M, N, dtype), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [128, 4096, 1023])
def test_in_place_and_empty(gpu_device, dtype, N):
    case = inputs.layernorm_case(5, 1460 + 4 * dtype, 97, N, dtype)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    wd, bd = H.to_device(case["w"], dtype, gpu_device), H.to_device(case["b"], dtype, gpu_device)
    bias64 = scale_of(case, mean, rstd)
    for m in MODES:
        xd = H.to_device(case["x"], dtype, gpu_device)
        H.say(f"layernorm in place N={N} mode={mode_name(m)}")
        try:
            launch(xd, wd, bd, 1e-5, m, xd)
        except layernorm.LayerNormError as e:
            if e.status == layernorm.LAYERNORM_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        compare.check_layernorm_parity(H.to_host(xd, dtype), want, bias64, dtype, f"in place {mode_name(m)}")
    empty = torch.empty((0, N), dtype=H.torch_dtype(dtype), device=gpu_device)
    assert tuple(layernorm.layernorm_fwd(empty, wd, bd, 1e-5).shape) == (0, N)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [2048, 1001, 5])
def test_misaligned_base_pointers(gpu_device, dtype, N):
    """x, w, b and y each off a 16-byte boundary by a different number of elements: the
    automatic path takes the element-aligned kernel, stays inside the buffers and matches the
    oracle; so does the element-wise kernel; the kernels that need 16-byte rows refuse."""
    M = 41
    case = inputs.layernorm_case(5, 1470 + 4 * dtype, M, N, dtype, mean=0.4)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    scale = scale_of(case, mean, rstd)
    td = H.torch_dtype(dtype)
    xbuf = torch.zeros(M * N + 8, dtype=td, device=gpu_device)
    wbuf = torch.zeros(N + 8, dtype=td, device=gpu_device)
    bbuf = torch.zeros(N + 8, dtype=td, device=gpu_device)
    xd, wd, bd = xbuf[1:1 + M * N].view(M, N), wbuf[3:3 + N], bbuf[2:2 + N]
    xd.copy_(H.to_device(case["x"], dtype, gpu_device))
    wd.copy_(H.to_device(case["w"], dtype, gpu_device))
    bd.copy_(H.to_device(case["b"], dtype, gpu_device))
    for mode in (0, layernorm.LAYERNORM_VARIANT_UNALIGNED, layernorm.LAYERNORM_VARIANT_GENERIC):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1)
        H.say(f"layernorm misaligned bases N={N} mode={mode_name(mode)}")
        layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=1)
        compare.check_layernorm_parity(H.to_host(y, dtype), want, scale, dtype, f"misaligned bases {mode_name(mode)}")
    _, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1)
    for v in (layernorm.LAYERNORM_VARIANT_WAVE, layernorm.LAYERNORM_VARIANT_BLOCK, layernorm.LAYERNORM_VARIANT_SUBWAVE):
        with pytest.raises(layernorm.LayerNormError) as e:
            layernorm.layernorm_fwd_variant(xd, wd, bd, 1e-5, v, y)
        assert e.value.status == layernorm.LAYERNORM_ERR_UNSUPPORTED


# The resident kernel (rows of at most 24 elements per thread, 256..1024 threads) walks rows
# blockIdx.x, blockIdx.x + gridDim.x, ... with two register copies of a row taking turns: row
# counts below, at and just past one and two rounds of its grid (256 or 512 workgroups on
# MI355X), odd and even numbers of rounds, full and ragged last chunks, with and without bias,
# and in place.
RESIDENT_SHAPES = [(inputs.FP16, 4096, 256), (inputs.FP16, 5120, 256), (inputs.BF16, 8192, 512),
                   (inputs.BF16, 8200, 512), (inputs.FP16, 16384, 1024), (inputs.FP32, 4096, 256),
                   (inputs.FP32, 6148, 512), (inputs.FP32, 12288, 1024)]


@pytest.mark.parametrize("dtype,N,threads", RESIDENT_SHAPES)
def test_resident_workgroups(gpu_device, dtype, N, threads):
    grid = 512 if threads == 256 else 256
    for k, M in enumerate((1, grid - 1, grid, grid + 1, 2 * grid, 2 * grid + 3, 3 * grid + grid // 2)):
        case = inputs.layernorm_case(6, 1480 + 4 * dtype, M, N, dtype, mean=-0.2, std=1.3, bias=(k % 3 != 1))
        check(case, gpu_device, modes=(0, ("threads", threads)))
    case = inputs.layernorm_case(6, 1496 + 4 * dtype, 2 * grid + 1, N, dtype)
    want, mean, rstd = oracle.layernorm_oracle(case["x"], case["w"], case["b"], 1e-5, dtype, stats=True)
    xd, wd, bd = (H.to_device(case[k], dtype, gpu_device) for k in ("x", "w", "b"))
    H.say(f"layernorm resident in place N={N} threads={threads}")
    layernorm.layernorm_fwd_tuned(xd, wd, bd, 1e-5, threads, xd)
    torch.cuda.synchronize()
    compare.check_layernorm_parity(H.to_host(xd, dtype), want, scale_of(case, mean, rstd), dtype, "resident in place")


def test_binding_rejects_mismatched_tensors(gpu_device):
    x = torch.zeros((4, 64), dtype=torch.float16, device=gpu_device)
    w = torch.ones(64, dtype=torch.float16, device=gpu_device)
    with pytest.raises(ValueError):
        layernorm.layernorm_fwd(x, w[:32], None, 1e-5)
    with pytest.raises(ValueError):
        layernorm.layernorm_fwd(x, w, w[:32], 1e-5)
    with pytest.raises(ValueError):
        layernorm.layernorm_fwd(x, w.float(), None, 1e-5)
    with pytest.raises(ValueError):
        layernorm.layernorm_fwd(x.cpu(), w, None, 1e-5)
    with pytest.raises(layernorm.LayerNormError):
        layernorm.layernorm_fwd(x, w, None, -1.0)
