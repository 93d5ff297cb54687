"""GPU parity tests of row cross-entropy against its CPU oracle, through the C ABI: the paper's
five stages (Section 4) in compact form.  Stability probes: rows of large identical values,
dominant logits (loss near 0), masked (-inf) classes, wide dynamic range, NaN/inf rows."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import crossentropy as ce
from paper_2603_21331_amd import inputs

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
MODES = (0, 2, 8, 16, 32, 64, 128, 256, 320, 512, 1024)  # threads per row; 0 = automatic; 8, 16 and 32
                                                          # (lane groups) only take short aligned rows,
                                                          # 2 (rows through LDS) at most 1024 classes
GUARD = 16
SENTINEL = -12345.0


def guarded(M, device):
    whole = torch.full((M + 2 * GUARD,), SENTINEL, dtype=torch.float32, device=device)
    return whole, whole[GUARD:GUARD + M]


def intact(whole, M):
    return bool((whole[:GUARD] == SENTINEL).all().item() and (whole[GUARD + M:] == SENTINEL).all().item())


def run_mode(xd, td, mode, what, with_lse=True):
    M, N = xd.shape
    lw, loss = guarded(M, xd.device)
    sw, lse = guarded(M, xd.device) if with_lse else (None, None)
    H.say(f"{what}: {M}x{N} {xd.dtype} threads={mode} lse={with_lse}")
    try:
        ce.crossentropy_fwd_tuned(xd, td, mode, loss, lse)
    except ce.CrossEntropyError as e:
        if e.status == ce.CROSSENTROPY_ERR_UNSUPPORTED and 0 < mode < 64:
            return None, None
        raise
    torch.cuda.synchronize()
    assert intact(lw, M), f"{what}: wrote outside loss"
    if with_lse:
        assert intact(sw, M), f"{what}: wrote outside lse"
    return loss.cpu().numpy(), (lse.cpu().numpy() if with_lse else None)


def check(case, device, modes=MODES, want=None):
    dtype = case["dtype"]
    t = np.asarray(case["target"], dtype=np.int64)
    if want is None:
        want = oracle.crossentropy_oracle(case["x"], t, dtype, with_lse=True)
    want_loss, want_lse = want
    ignored = (t < 0) | (t >= case["N"])
    xd = H.to_device(case["x"], dtype, device)
    td = torch.from_numpy(t).to(device)
    stats = {}
    for m in modes:
        loss, lse = run_mode(xd, td, m, case["name"])
        if loss is None:
            continue
        stats[m] = compare.check_crossentropy_parity(loss, want_loss, f"{case['name']} loss [threads {m}]",
                                                     exact_zero=ignored)
        compare.check_crossentropy_parity(lse, want_lse, f"{case['name']} lse [threads {m}]")
    # the loss alone (lse == NULL) must be the same bits
    loss_only, _ = run_mode(xd, td, 0, case["name"], with_lse=False)
    both, _ = run_mode(xd, td, 0, case["name"])
    assert np.array_equal(loss_only.view(np.uint32), both.view(np.uint32))
    return stats


# stage 1: smoke
@pytest.mark.parametrize("dtype", DTYPES)
def test_smoke_128x128(gpu_device, dtype):
    check(inputs.crossentropy_case(0, 1600 + 4 * dtype, 128, 128, dtype), gpu_device)


# stage 2: shape sweep
SWEEP = [("tiny", 70, 8), ("head_64", 1031, 64), ("ragged_200", 333, 200), ("ctx_512", 515, 512),
         ("ragged_1000", 301, 1000), ("one_wave_limit", 517, 2048), ("past_one_wave", 130, 2056),
         ("standard_4096", 1024, 4096), ("wide_8192", 259, 8192), ("vocab_32000", 67, 32000),
         ("vocab_50257", 33, 50257), ("vocab_65536", 9, 65536), ("vocab_128256", 7, 128256),
         ("batch_remainder_3", 6, 28672 + 8), ("past_256_threads", 5, 131080), ("long_300001", 3, 300001), ("tall", 8192, 1024)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("name,M,N", SWEEP, ids=[s[0] for s in SWEEP])
def test_shape_sweep(gpu_device, name, M, N, dtype):
    check(inputs.crossentropy_case(1, 1620 + 4 * dtype, M, N, dtype, 2.0, ignore_every=7), gpu_device)


def test_paper_result_shape_fp16_4096x32000(gpu_device):
    stats = check(inputs.crossentropy_paper_shape(0), gpu_device, modes=(0, 1024))
    H.say(f"cross-entropy 4096x32000 stats {stats}")


def test_benchmark_shape_fp16_8192x32000(gpu_device):
    """The shape bench.py --op crossentropy times, in its launch configuration (automatic)."""
    stats = check(inputs.crossentropy_paper_shape(1), gpu_device, modes=(0,))
    H.say(f"cross-entropy 8192x32000 stats {stats}")


# stage 3: stability
@pytest.mark.parametrize("N", [4099, 512])
@pytest.mark.parametrize("dtype", DTYPES)
def test_rows_of_large_identical_values(gpu_device, dtype, N):
    big = {inputs.FP32: 3.0e38, inputs.FP16: 60000.0, inputs.BF16: 3.0e38}[dtype]
    z = np.zeros((6, N))
    z[0] = big
    z[1] = -big
    z[2] = 88.0
    z[3] = big
    z[3, 17] = -big
    z[4] = -big
    z[4, 100] = big
    z[5, ::2] = big
    t = np.array([0, N - 1, 5, 17, 100, 1], dtype=np.int64)
    x = inputs.to_storage(z, dtype)
    want = oracle.crossentropy_oracle(x, t, dtype, with_lse=True)
    assert abs(float(want[0][0]) - np.log(N)) < 1e-6 and want[0][4] == 0.0
    check(dict(name="large_identical", dtype=dtype, M=6, N=N, x=x, target=t), gpu_device, want=want)


@pytest.mark.parametrize("dtype", DTYPES)
def test_dominant_logit_and_wide_range(gpu_device, dtype):
    """Losses from ~1e-7 (target dominates) to hundreds (target far below the maximum)."""
    N = 3000
    z = inputs.normal(3, 1640, 0, 8 * N).reshape(8, N)
    spread = {inputs.FP32: 30.0, inputs.FP16: 6.0, inputs.BF16: 28.0}[dtype]
    z[:4] *= spread
    z[4, 11] = 16.0
    z[5, 12] = 30.0
    z[6, 13] = 200.0
    z[7] = np.linspace(0.0, -300.0, N)
    t = np.array([0, 1, 2, 3, 11, 12, 13, N - 1], dtype=np.int64)
    x = inputs.to_storage(z, dtype)
    want = oracle.crossentropy_oracle(x, t, dtype, with_lse=True)
    assert 0.0 <= want[0][5] < 1e-6 and want[0][7] > 250.0
    check(dict(name="dominant_wide", dtype=dtype, M=8, N=N, x=x, target=t), gpu_device, want=want)


@pytest.mark.parametrize("dtype", DTYPES)
def test_masked_classes(gpu_device, dtype):
    """Row i keeps classes 0..i (the rest -inf); targets inside and, on odd rows, on a masked class."""
    N = 520
    z = inputs.normal(3, 1650, 0, N * N).reshape(N, N) * 3.0
    t = np.arange(N, dtype=np.int64) // 2
    t[1::2] = N - 1
    t[N - 1] = N - 1
    x = inputs.to_storage(z, dtype)
    # -inf written as bits: the fp16 conversion of the input module clamps to the finite range
    x[np.triu_indices(N, 1)] = {inputs.FP32: np.float32(-np.inf), inputs.FP16: 0xFC00, inputs.BF16: 0xFF80}[dtype]
    want = oracle.crossentropy_oracle(x, t, dtype, with_lse=True)
    assert want[0][0] == 0.0 and np.isinf(want[0][1]) and np.isfinite(want[0][N - 1])
    check(dict(name="masked", dtype=dtype, M=N, N=N, x=x, target=t), gpu_device, want=want)


def test_nan_inf_rows(gpu_device):
    N = 1024
    x = inputs.normal_matrix(3, 1660, 6, N, inputs.FP32)
    x[1, 7] = np.nan
    x[2, 9] = np.inf
    x[3, :] = -np.inf
    x[4, 3] = -np.inf
    x[5, 1000] = np.nan
    t = np.array([0, 1, 2, 3, 3, -1], dtype=np.int64)
    want = oracle.crossentropy_oracle(x, t, inputs.FP32, with_lse=True)
    assert np.isnan(want[0][1:4]).all() and want[0][4] == np.inf and want[0][5] == 0.0
    assert np.isnan(want[1][1:4]).all() and np.isnan(want[1][5]) and np.isfinite(want[1][4])
    check(dict(name="nan_inf", dtype=inputs.FP32, M=6, N=N, x=x, target=t), gpu_device, want=want)


@pytest.mark.parametrize("dtype", [inputs.FP16, inputs.BF16])
def test_targets_outside_the_classes_are_ignored(gpu_device, dtype):
    case = inputs.crossentropy_case(3, 1670, 40, 777, dtype)
    case["target"][:8] = [-100, -1, 777, 778, 1 << 40, -(1 << 62), 0, 776]
    check(case, gpu_device)


# stage 4: determinism
@pytest.mark.parametrize("N", [5000, 1000, 96, 24])
def test_determinism_and_row_independence(gpu_device, N):
    case = inputs.crossentropy_case(4, 1680, 777, N, inputs.FP16, 2.0)
    xd = H.to_device(case["x"], inputs.FP16, gpu_device)
    td = torch.from_numpy(case["target"]).to(gpu_device)
    ran = 0
    for m in MODES:
        H.say(f"cross-entropy determinism N={N} threads={m}")
        loss = torch.empty(777, dtype=torch.float32, device=gpu_device)
        try:
            ce.crossentropy_fwd_tuned(xd, td, m, loss)
        except ce.CrossEntropyError as e:
            if e.status == ce.CROSSENTROPY_ERR_UNSUPPORTED and 0 < m < 64:
                continue
            raise
        ran += 1
        torch.cuda.synchronize()
        first = loss.cpu().numpy().view(np.uint32).copy()
        for _ in range(2):
            ce.crossentropy_fwd_tuned(xd, td, m, loss)
            torch.cuda.synchronize()
            assert np.array_equal(loss.cpu().numpy().view(np.uint32), first)
        fresh = ce.crossentropy_fwd_tuned(xd, td, m)
        torch.cuda.synchronize()
        assert np.array_equal(fresh.cpu().numpy().view(np.uint32), first)
        for i in (0, 333, 776):
            one = ce.crossentropy_fwd_tuned(xd[i:i + 1], td[i:i + 1], m)
            assert one.cpu().numpy().view(np.uint32)[0] == first[i]
    assert ran == {5000: 7, 1000: 10, 96: 11, 24: 11}[N]


# stage 5: edge cases
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1023, 1023), (33, 4097), (129, 1537), (1, 1), (7, 1), (2, 3), (1, 8),
                                 (5, 12), (3, 40001), (1, 8192)])
def test_edge_dims(gpu_device, M, N, dtype):
    check(inputs.crossentropy_case(5, 1700 + 4 * dtype, M, N, dtype, 1.5), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
def test_base_pointer_aligned_to_one_element_only(gpu_device, dtype):
    M, N = 37, 1001
    case = inputs.crossentropy_case(5, 1720 + 4 * dtype, M, N, dtype)
    flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    xd = H.to_device(flat, dtype, gpu_device)[1:].view(M, N)
    td = torch.from_numpy(case["target"]).to(gpu_device)
    want = oracle.crossentropy_oracle(case["x"], case["target"], dtype)
    for m in MODES:
        loss, _ = run_mode(xd, td, m, "offset base")
        if m in (8, 16, 32):
            assert loss is None, "lane groups must refuse a base that is not 16-byte aligned"
            continue
        compare.check_crossentropy_parity(loss, want, f"offset base [threads {m}]")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [8, 16, 100, 128, 256, 264, 512, 1000, 1024, 2048])
def test_few_classes_lane_groups(gpu_device, N, dtype):
    """Rows short enough for 8, 16 or 32 lanes per row (classifier heads of 10 to 2000 classes),
    with a row count that leaves the last wavefront partly past M; every lane-group size that
    takes the shape, the automatic choice and one workgroup per row all agree with the oracle."""
    M = 1027
    case = inputs.crossentropy_case(5, 1760 + 4 * dtype, M, N, dtype, 2.0, ignore_every=11)
    stats = check(case, gpu_device, modes=(0, 2, 8, 16, 32, 64))
    assert (2 in stats) == (N <= 1024)
    nvec = N * inputs.DTYPE_BYTES[dtype] // 16
    took = sorted(m for m in stats if m in (8, 16, 32))
    assert took == [l for l in (8, 16, 32) if N * inputs.DTYPE_BYTES[dtype] % 16 == 0 and nvec <= 8 * l]


def test_more_rows_than_the_grid_limit(gpu_device):
    """M above 2^20 workgroups: the kernel walks the remaining rows in a grid-stride loop."""
    M, N = (1 << 20) + 77, 8
    case = inputs.crossentropy_case(5, 1740, M, N, inputs.BF16, 2.0, ignore_every=1000)
    check(case, gpu_device, modes=(0, 256))


def test_empty_batch_and_binding_checks(gpu_device):
    x = torch.zeros((0, 64), dtype=torch.float16, device=gpu_device)
    t = torch.zeros((0,), dtype=torch.int64, device=gpu_device)
    assert tuple(ce.crossentropy_fwd(x, t).shape) == (0,)
    x = torch.zeros((4, 64), dtype=torch.float16, device=gpu_device)
    t = torch.zeros((4,), dtype=torch.int64, device=gpu_device)
    with pytest.raises(ValueError):
        ce.crossentropy_fwd(x, t[:3])
    with pytest.raises(ValueError):
        ce.crossentropy_fwd(x, t.int())
    with pytest.raises(ValueError):
        ce.crossentropy_fwd(x, t, torch.zeros(4, dtype=torch.float16, device=gpu_device))
    with pytest.raises(ValueError):
        ce.crossentropy_fwd(x.t(), t)
    with pytest.raises(ValueError):
        ce.crossentropy_fwd(x.cpu(), t)
    with pytest.raises(TypeError):
        ce.crossentropy_fwd(x.double(), t)
    with pytest.raises(ce.CrossEntropyError):
        ce.crossentropy_fwd_tuned(x, t, 96)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [1, 2, 3, 5, 10, 17, 31, 33, 63, 64])
def test_handful_of_classes(gpu_device, N, dtype):
    """Rows shorter than a lane group (a 10-way classifier): through LDS with one to four lanes
    per row, any alignment;
    a base pointer one element off, masked classes, ignored targets and a row count that ends
    inside a wavefront."""
    M = 2051
    case = inputs.crossentropy_case(5, 1800 + 4 * dtype, M, N, dtype, 3.0, ignore_every=13)
    stats = check(case, gpu_device, modes=(0, 2, 64))
    assert 2 in stats
    flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    if N > 1:
        neg_inf = {inputs.FP32: np.float32(-np.inf), inputs.FP16: 0xFC00, inputs.BF16: 0xFF80}[dtype]
        case["x"][::3, N // 2] = neg_inf
        flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    xd = H.to_device(flat, dtype, gpu_device)[1:].view(M, N)
    td = torch.from_numpy(case["target"]).to(gpu_device)
    want = oracle.crossentropy_oracle(case["x"], case["target"], dtype)
    t = case["target"]
    for m in (0, 2):
        loss, _ = run_mode(xd, td, m, "handful, offset base")
        compare.check_crossentropy_parity(loss, want, f"handful offset base [threads {m}]",
                                          exact_zero=(t < 0) | (t >= N))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [65, 77, 100, 127, 129, 197, 255, 257, 300, 333, 511, 512, 513, 1001, 1024])
def test_up_to_1024_classes_through_lds(gpu_device, N, dtype):
    """Rows that are not whole aligned vectors, several per workgroup through LDS: two full
    tiles and a partial one, masked classes, ignored targets, and a base pointer one element
    off; the automatic path must choose this kernel for the odd lengths."""
    rows_per_tile = 16384 // (N * inputs.DTYPE_BYTES[dtype])
    M = 2 * rows_per_tile + 5
    case = inputs.crossentropy_case(5, 1840 + 4 * dtype, M, N, dtype, 3.0, ignore_every=13)
    neg_inf = {inputs.FP32: np.float32(-np.inf), inputs.FP16: 0xFC00, inputs.BF16: 0xFF80}[dtype]
    case["x"][::3, N // 2] = neg_inf
    stats = check(case, gpu_device, modes=(0, 2, 64))
    assert 2 in stats
    if N * inputs.DTYPE_BYTES[dtype] % 16:
        assert ce.crossentropy_auto_threads_per_row(N, dtype) == 2
    flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    xd = H.to_device(flat, dtype, gpu_device)[1:].view(M, N)
    td = torch.from_numpy(case["target"]).to(gpu_device)
    want = oracle.crossentropy_oracle(case["x"], case["target"], dtype)
    t = case["target"]
    for m in (0, 2):
        loss, _ = run_mode(xd, td, m, "through LDS, offset base")
        compare.check_crossentropy_parity(loss, want, f"through LDS, offset base [threads {m}]",
                                          exact_zero=(t < 0) | (t >= N))


def test_through_lds_more_tiles_than_the_grid(gpu_device):
    """The grid stops at 8192 workgroups: 8 rows of 2 KiB per tile, 65536 + 13 rows."""
    M, N = 8192 * 8 + 13, 511
    case = inputs.crossentropy_case(5, 1860, M, N, inputs.FP32, 2.0, ignore_every=1000)
    check(case, gpu_device, modes=(2,))
