"""GPU parity tests of row softmax against its CPU oracle, through the C ABI: the paper's five
stages (Section 4) in compact form.  Its stability probe for softmax is rows of large
identical values; masked (-inf) entries, wide dynamic range and NaN/inf rows are added."""
import sys

import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import inputs, softmax

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
THREADS = (8, 16, 32, 64, 256, 512, 1024)
MODES = (0, 1, 2, 3, 4, 5, 6, 7) + tuple(("threads", g) for g in THREADS)


def mode_name(m):
    return f"threads{m[1]}" if isinstance(m, tuple) else softmax.VARIANT_NAMES[m]


def launch(xd, mode, y):
    if isinstance(mode, tuple):
        return softmax.softmax_fwd_tuned(xd, mode[1], y)
    return softmax.softmax_fwd_variant(xd, mode, y)


def run_mode(xd, dtype, mode, what):
    M, N = xd.shape
    whole, y = H.alloc_guarded(M, N, dtype, xd.device)
    H.say(f"{what}: {inputs.DTYPE_NAMES[dtype]} {M}x{N} mode={mode_name(mode)}")
    try:
        launch(xd, mode, y)
    except softmax.SoftmaxError as e:
        if e.status == softmax.SOFTMAX_ERR_UNSUPPORTED and mode != 0:
            return None
        raise
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype), f"{what}: wrote outside y"
    return H.to_host(y, dtype)


def check(case, device, modes=MODES, want=None):
    dtype = case["dtype"]
    if want is None:
        want = oracle.softmax_oracle(case["x"], dtype)
    xd = H.to_device(case["x"], dtype, device)
    stats, ran = {}, 0
    for m in modes:
        got = run_mode(xd, dtype, m, case["name"])
        if got is None:
            continue
        ran += 1
        stats[mode_name(m)] = compare.check_softmax_parity(got, want, dtype, f"{case['name']} [{mode_name(m)}]")
    assert ran >= 2
    return stats


# stage 1: smoke
@pytest.mark.parametrize("dtype", DTYPES)
def test_smoke_128x128(gpu_device, dtype):
    check(inputs.softmax_case(0, 1100 + dtype, 128, 128, dtype), gpu_device)


# stage 2: shape sweep
SWEEP = [("tiny", 70, 8), ("head_64", 1031, 64), ("ctx_128", 4099, 128), ("ctx_200", 333, 200),
         ("ctx_512", 515, 512), ("ragged_1000", 301, 1000), ("ctx_2048", 517, 2048),
         ("standard_4096", 1024, 4096), ("hidden_5120", 259, 5120), ("wide_8192", 259, 8192),
         ("vocab_32000", 67, 32000), ("limit_16bit", 9, 65536), ("past_limit", 5, 65544),
         ("vocab_128256", 7, 128256), ("vocab_151936", 5, 151936), ("long_odd_262145", 3, 262145),
         ("tall", 8192, 1024)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("name,M,N", SWEEP, ids=[s[0] for s in SWEEP])
def test_shape_sweep(gpu_device, name, M, N, dtype):
    check(inputs.softmax_case(1, 1110 + dtype, M, N, dtype, 2.0), gpu_device)


@pytest.mark.parametrize("n", [4096, 8192])
def test_paper_result_shapes_fp16(gpu_device, n):
    stats = check(inputs.softmax_paper_shape(n), gpu_device)
    H.say(f"softmax {n}^2 stats {stats}")


# stage 3: stability
@pytest.mark.parametrize("dtype", DTYPES)
def test_rows_of_large_identical_values(gpu_device, dtype):
    big = {inputs.FP32: 3.0e38, inputs.FP16: 60000.0, inputs.BF16: 3.0e38}[dtype]
    N = 4096
    z = np.zeros((6, N))
    z[0] = big
    z[1] = -big
    z[2] = 88.0
    z[3] = big
    z[3, 17] = -big
    z[4] = -big
    z[4, 100] = big
    z[5, ::2] = big
    case = dict(name="large_identical", dtype=dtype, M=6, N=N, x=inputs.to_storage(z, dtype))
    want = oracle.softmax_oracle(case["x"], dtype)
    assert oracle.decode(want[0], dtype)[0] == 1.0 / N
    check(case, gpu_device, want=want)


@pytest.mark.parametrize("dtype", DTYPES)
def test_wide_dynamic_range_and_subnormal_outputs(gpu_device, dtype):
    N = 2048
    z = inputs.normal(3, 1120, 0, 6 * N).reshape(6, N)
    spread = {inputs.FP32: 30.0, inputs.FP16: 6.0, inputs.BF16: 28.0}[dtype]
    z *= spread
    z[4] = np.linspace(0.0, -{inputs.FP32: 104.0, inputs.FP16: 18.0, inputs.BF16: 93.0}[dtype], N)
    z[5] = z[4][::-1]
    case = dict(name="wide_range", dtype=dtype, M=6, N=N, x=inputs.to_storage(z, dtype))
    want = oracle.softmax_oracle(case["x"], dtype)
    if dtype == inputs.FP32:
        w = np.abs(want)
        assert np.any((w > 0) & (w < compare.FLT_MIN)), "must produce subnormal outputs"
    else:
        mag = want & 0x7FFF
        assert np.any((mag > 0) & (mag < (0x0400 if dtype == inputs.FP16 else 0x0080)))
    check(case, gpu_device, want=want)


@pytest.mark.parametrize("dtype", DTYPES)
def test_causal_mask_rows(gpu_device, dtype):
    """Row i keeps entries 0..i and has -inf beyond: the attention-score pattern."""
    N = 512
    z = inputs.normal(3, 1130, 0, N * N).reshape(N, N) * 3.0
    z[np.triu_indices(N, 1)] = -np.inf
    case = dict(name="causal", dtype=dtype, M=N, N=N, x=inputs.to_storage(z, dtype))
    want = oracle.softmax_oracle(case["x"], dtype)
    assert np.all(oracle.decode(want, dtype)[np.triu_indices(N, 1)] == 0.0)
    check(case, gpu_device, want=want)


def test_nan_inf_rows(gpu_device):
    N = 1024
    x = inputs.normal_matrix(3, 1140, 5, N, inputs.FP32)
    x[1, 7] = np.nan
    x[2, 9] = np.inf
    x[3, :] = -np.inf
    x[4, 3] = -np.inf
    want = oracle.softmax_oracle(x, inputs.FP32)
    assert np.isnan(want[1]).all() and np.isnan(want[2]).all() and np.isnan(want[3]).all()
    assert not np.isnan(want[0]).any() and want[4, 3] == 0.0
    check(dict(name="nan_inf", dtype=inputs.FP32, M=5, N=N, x=x), gpu_device, want=want)


# stage 4: determinism
def test_determinism_and_row_independence(gpu_device):
    case = inputs.softmax_case(4, 1150, 777, 4096, inputs.FP16, 2.0)
    xd = H.to_device(case["x"], inputs.FP16, gpu_device)
    for m in MODES:
        H.say(f"softmax determinism mode={mode_name(m)}")
        y = torch.empty_like(xd)
        try:
            launch(xd, m, y)
        except softmax.SoftmaxError as e:
            if e.status == softmax.SOFTMAX_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        first = H.to_host(y, inputs.FP16).copy()
        for _ in range(2):
            launch(xd, m, y)
            torch.cuda.synchronize()
            assert np.array_equal(H.to_host(y, inputs.FP16), first)
        fresh = torch.empty_like(xd)
        launch(xd, m, fresh)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_host(fresh, inputs.FP16), first)
        if m != 0:
            for i in (0, 333, 776):
                one = H.to_host(launch(xd[i:i + 1], m, None), inputs.FP16)
                assert np.array_equal(one[0], first[i])


# stage 5: edge cases
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1023, 1023), (33, 4097), (129, 1537), (1, 1), (7, 1), (2, 3), (1, 8),
                                 (5, 12), (3, 40001), (1, 8192)])
def test_edge_dims(gpu_device, M, N, dtype):
    check(inputs.softmax_case(5, 1160 + dtype, M, N, dtype, 1.5), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [128, 4096, 1023])
def test_in_place_and_empty(gpu_device, dtype, N):
    case = inputs.softmax_case(5, 1170 + dtype, 97, N, dtype)
    want = oracle.softmax_oracle(case["x"], dtype)
    for m in MODES:
        xd = H.to_device(case["x"], dtype, gpu_device)
        H.say(f"softmax in place N={N} mode={mode_name(m)}")
        try:
            launch(xd, m, xd)
        except softmax.SoftmaxError as e:
            if e.status == softmax.SOFTMAX_ERR_UNSUPPORTED:
                continue
            raise
        torch.cuda.synchronize()
        compare.check_softmax_parity(H.to_host(xd, dtype), want, dtype, f"in place {mode_name(m)}")
    empty = torch.empty((0, N), dtype=H.torch_dtype(dtype), device=gpu_device)
    assert tuple(softmax.softmax_fwd(empty).shape) == (0, N)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [2048, 1001, 5])
def test_misaligned_base_pointers(gpu_device, dtype, N):
    """Bases one and three elements off a 16-byte boundary: the automatic path takes the
    element-aligned kernel, stays inside the buffers and matches the oracle; so does the
    element-wise kernel; the kernels that need 16-byte rows refuse."""
    M = 41
    case = inputs.softmax_case(5, 1180 + dtype, M, N, dtype, 2.0)
    want = oracle.softmax_oracle(case["x"], dtype)
    xbuf = torch.zeros(M * N + 8, dtype=H.torch_dtype(dtype), device=gpu_device)
    xd = xbuf[1:1 + M * N].view(M, N)
    xd.copy_(H.to_device(case["x"], dtype, gpu_device))
    for mode in (0, softmax.SOFTMAX_VARIANT_UNALIGNED, softmax.SOFTMAX_VARIANT_GENERIC):
        whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=3)
        H.say(f"softmax misaligned bases N={N} mode={mode_name(mode)}")
        softmax.softmax_fwd_variant(xd, mode, y)
        torch.cuda.synchronize()
        assert H.guards_intact(whole, M, N, dtype, offset_elems=3)
        compare.check_softmax_parity(H.to_host(y, dtype), want, dtype, f"misaligned bases {mode_name(mode)}")
    # y at the same offset from a 16-byte boundary as x: the kernel cuts every row at the
    # boundaries the two share
    whole, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=1)
    softmax.softmax_fwd_variant(xd, softmax.SOFTMAX_VARIANT_UNALIGNED, y)
    torch.cuda.synchronize()
    assert H.guards_intact(whole, M, N, dtype, offset_elems=1)
    compare.check_softmax_parity(H.to_host(y, dtype), want, dtype, "misaligned bases, same offset")
    _, y = H.alloc_guarded(M, N, dtype, gpu_device, offset_elems=3)
    for v in (softmax.SOFTMAX_VARIANT_WAVE, softmax.SOFTMAX_VARIANT_BLOCK, softmax.SOFTMAX_VARIANT_SUBWAVE):
        with pytest.raises(softmax.SoftmaxError) as e:
            softmax.softmax_fwd_variant(xd, v, y)
        assert e.value.status == softmax.SOFTMAX_ERR_UNSUPPORTED


def test_binding_rejects_mismatched_tensors(gpu_device):
    x = torch.zeros((4, 64), dtype=torch.float16, device=gpu_device)
    with pytest.raises(ValueError):
        softmax.softmax_fwd(x, torch.zeros((4, 32), dtype=torch.float16, device=gpu_device))
    with pytest.raises(ValueError):
        softmax.softmax_fwd(x.t())
    with pytest.raises(ValueError):
        softmax.softmax_fwd(x.cpu())
    with pytest.raises(TypeError):
        softmax.softmax_fwd(x.double())
