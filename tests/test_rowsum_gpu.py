"""GPU parity tests of the row sum against its CPU oracle, through the C ABI: the paper's five
stages (Section 4) in compact form.  Stability probes: cancelling rows, a large mean with a
small spread, wide dynamic range, fp16 subnormals, NaN/inf rows."""
import numpy as np
import pytest
import torch

import compare
import gpu_harness as H
import oracle
from paper_2603_21331_amd import inputs
from paper_2603_21331_amd import rowsum as rs

pytestmark = pytest.mark.gpu

DTYPES = [inputs.FP32, inputs.FP16, inputs.BF16]
BLOCK_MODES = (0, 64, 128, 256, 320, 512, 1024)  # threads per row; 0 = automatic
GUARD = 16
SENTINEL = -12345.0


def guarded(M, device):
    whole = torch.full((M + 2 * GUARD,), SENTINEL, dtype=torch.float32, device=device)
    return whole, whole[GUARD:GUARD + M]


def intact(whole, M):
    return bool((whole[:GUARD] == SENTINEL).all().item() and (whole[GUARD + M:] == SENTINEL).all().item())


def modes_for(N, dtype, aligned=True):
    """Every thread count the ABI accepts for this shape."""
    vec = 4 if dtype == inputs.FP32 else 8
    modes = list(BLOCK_MODES)
    if aligned and N % vec == 0:
        modes += [g for g in (8, 16, 32) if N // vec <= 8 * g]
    if N <= 1024:
        modes.append(2)          # runs of rows through LDS
    return modes


def run_mode(xd, mode, what):
    M, N = xd.shape
    yw, y = guarded(M, xd.device)
    H.say(f"{what}: {M}x{N} {xd.dtype} threads={mode}")
    rs.rowsum_fwd_tuned(xd, mode, y)
    torch.cuda.synchronize()
    assert intact(yw, M), f"{what}: wrote outside y"
    return y.cpu().numpy()


def check(case, device, modes=None, want=None):
    dtype, N = case["dtype"], case["N"]
    if want is None:
        want = oracle.rowsum_oracle(case["x"], dtype, with_abs=True)
    want_y, want_abs = want
    xd = H.to_device(case["x"], dtype, device)
    stats = {}
    for m in (modes_for(N, dtype) if modes is None else modes):
        y = run_mode(xd, m, case["name"])
        stats[m] = compare.check_rowsum_parity(y, want_y, want_abs, N, f"{case['name']} [threads {m}]")
    return stats


# stage 1: smoke
@pytest.mark.parametrize("dtype", DTYPES)
def test_smoke_128x128(gpu_device, dtype):
    check(inputs.rowsum_case(0, 1800 + 4 * dtype, 128, 128, dtype), gpu_device)


# stage 2: shape sweep
SWEEP = [("tiny", 70, 8), ("head_64", 1031, 64), ("ragged_200", 333, 200), ("ctx_512", 515, 512),
         ("past_subwave", 301, 520), ("ragged_1000", 301, 1000), ("one_wave", 517, 2048),
         ("past_one_batch", 130, 2056), ("standard_4096", 1024, 4096), ("wide_8192", 259, 8192),
         ("n_32000", 67, 32000), ("n_50257", 33, 50257), ("n_65536", 9, 65536),
         ("batch_remainder_3", 6, 28672 + 8), ("past_1024_threads", 5, 131080), ("long_300001", 3, 300001),
         ("tall", 8192, 1024), ("tall_short", 65539, 64)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("name,M,N", SWEEP, ids=[s[0] for s in SWEEP])
def test_shape_sweep(gpu_device, name, M, N, dtype):
    check(inputs.rowsum_case(1, 1820 + 4 * dtype, M, N, dtype, 0.25, 2.0), gpu_device)


@pytest.mark.parametrize("which", [0, 1])
def test_paper_result_shapes_fp16(gpu_device, which):
    stats = check(inputs.rowsum_paper_shape(which), gpu_device, modes=(0, 256))
    H.say(f"row sum paper shape {which} stats {stats}")


# stage 3: stability
@pytest.mark.parametrize("dtype", DTYPES)
def test_cancelling_rows_and_large_means(gpu_device, dtype):
    N = 4100
    z = inputs.normal(3, 1840, 0, 8 * N).reshape(8, N)
    z[0] = np.where(np.arange(N) % 2 == 0, 1000.0, -1000.0)            # cancels to exactly 0
    z[1] = 1000.0 + 0.01 * z[1]                                          # large mean, small spread
    z[2] = z[2] * 10.0 ** (-6.0 + 9.0 * inputs.uniform(3, 1841, 0, N))   # wide range of magnitudes
    z[3] = 0.0
    z[4, :] = 0.0
    z[4, 2049] = -7.0                                                    # a single entry
    z[5] = np.abs(z[5])                                                  # one sign: no cancellation
    z[6] = z[6] * 1e-6                                                   # fp16: subnormal inputs
    z[7, ::2] = -z[7, 1::2]                                              # pairs that cancel exactly
    x = inputs.to_storage(z, dtype)
    want = oracle.rowsum_oracle(x, dtype, with_abs=True)
    assert want[0][0] == 0.0 and want[0][3] == 0.0 and want[0][4] == -7.0 and want[0][7] == 0.0
    check(dict(name="cancelling", dtype=dtype, M=8, N=N, x=x), gpu_device, want=want)


def test_nan_inf_rows(gpu_device):
    N = 1024
    x = inputs.normal_matrix(3, 1860, 7, N, inputs.FP32)
    x[1, 7] = np.nan
    x[2, 9] = np.inf
    x[3, 11] = -np.inf
    x[4, 3], x[4, 900] = np.inf, -np.inf
    x[5, :] = np.inf
    x[6, 1023] = np.nan
    want = oracle.rowsum_oracle(x, inputs.FP32, with_abs=True)
    assert np.isnan(want[0][[1, 4, 6]]).all() and want[0][2] == np.inf and want[0][3] == -np.inf
    assert want[0][5] == np.inf
    check(dict(name="nan_inf", dtype=inputs.FP32, M=7, N=N, x=x), gpu_device, want=want)


@pytest.mark.parametrize("dtype", [inputs.FP16, inputs.BF16])
def test_results_keep_fp32_digits(gpu_device, dtype):
    """Row sums of 16-bit data that are not 16-bit numbers: exact in fp32 for these inputs."""
    N = 1032
    x = inputs.to_storage(np.full((5, N), 1.0 + 2.0 ** -7), dtype)
    xd = H.to_device(x, dtype, gpu_device)
    for m in modes_for(N, dtype):
        y = run_mode(xd, m, "fp32 digits")
        assert np.all(y == np.float32(N * (1.0 + 2.0 ** -7))), m


# stage 4: determinism
def test_determinism_and_row_independence(gpu_device):
    case = inputs.rowsum_case(4, 1880, 777, 5000, inputs.FP16, 0.0, 2.0)
    xd = H.to_device(case["x"], inputs.FP16, gpu_device)
    for m in BLOCK_MODES:
        H.say(f"row sum determinism threads={m}")
        y = torch.empty(777, dtype=torch.float32, device=gpu_device)
        rs.rowsum_fwd_tuned(xd, m, y)
        torch.cuda.synchronize()
        first = y.cpu().numpy().view(np.uint32).copy()
        for _ in range(2):
            rs.rowsum_fwd_tuned(xd, m, y)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy().view(np.uint32), first)
        fresh = rs.rowsum_fwd_tuned(xd, m)
        torch.cuda.synchronize()
        assert np.array_equal(fresh.cpu().numpy().view(np.uint32), first)
        for i in (0, 336, 776):        # rows whose start has the same 16-byte alignment as row 0's
            one = rs.rowsum_fwd_tuned(xd[i:i + 1], m)
            assert one.cpu().numpy().view(np.uint32)[0] == first[i]


def test_determinism_short_rows(gpu_device):
    case = inputs.rowsum_case(4, 1884, 1001, 256, inputs.BF16)
    xd = H.to_device(case["x"], inputs.BF16, gpu_device)
    for m in (0, 8, 16, 32, 64):
        first = rs.rowsum_fwd_tuned(xd, m).cpu().numpy().view(np.uint32).copy()
        for _ in range(2):
            assert np.array_equal(rs.rowsum_fwd_tuned(xd, m).cpu().numpy().view(np.uint32), first)
        assert rs.rowsum_fwd_tuned(xd[500:501], m).cpu().numpy().view(np.uint32)[0] == first[500]


# stage 5: edge cases
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("M,N", [(1023, 1023), (33, 4097), (129, 1537), (1, 1), (7, 1), (2, 3), (1, 8),
                                 (5, 12), (3, 40001), (1, 8192), (63, 16), (65, 32), (3, 256)])
def test_edge_dims(gpu_device, M, N, dtype):
    check(inputs.rowsum_case(5, 1900 + 4 * dtype, M, N, dtype, -0.5, 1.5), gpu_device)


@pytest.mark.parametrize("dtype", DTYPES)
def test_base_pointer_aligned_to_one_element_only(gpu_device, dtype):
    M, N = 37, 1000
    case = inputs.rowsum_case(5, 1920 + 4 * dtype, M, N, dtype)
    flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    xd = H.to_device(flat, dtype, gpu_device)[1:].view(M, N)
    want_y, want_abs = oracle.rowsum_oracle(case["x"], dtype, with_abs=True)
    for m in BLOCK_MODES:
        y = run_mode(xd, m, "offset base")
        compare.check_rowsum_parity(y, want_y, want_abs, N, f"offset base [threads {m}]")
    with pytest.raises(rs.RowSumError):
        rs.rowsum_fwd_tuned(xd, 32)


def test_more_rows_than_the_grid_limit(gpu_device):
    """M above 2^20 workgroups: the kernels walk the remaining rows in a grid-stride loop."""
    M, N = (1 << 20) + 77, 8
    check(inputs.rowsum_case(5, 1940, M, N, inputs.BF16, 0.0, 2.0), gpu_device, modes=(0, 64))
    M, N = 16 * (1 << 20) + 5, 8
    check(inputs.rowsum_case(5, 1944, M, N, inputs.FP16), gpu_device, modes=(0,))


def test_empty_batch_and_binding_checks(gpu_device):
    x = torch.zeros((0, 64), dtype=torch.float16, device=gpu_device)
    assert tuple(rs.rowsum_fwd(x).shape) == (0,)
    x = torch.zeros((4, 64), dtype=torch.float16, device=gpu_device)
    with pytest.raises(ValueError):
        rs.rowsum_fwd(x, torch.zeros(3, dtype=torch.float32, device=gpu_device))
    with pytest.raises(ValueError):
        rs.rowsum_fwd(x, torch.zeros(4, dtype=torch.float16, device=gpu_device))
    with pytest.raises(ValueError):
        rs.rowsum_fwd(x.t())
    with pytest.raises(ValueError):
        rs.rowsum_fwd(x.cpu())
    with pytest.raises(TypeError):
        rs.rowsum_fwd(x.double())
    with pytest.raises(rs.RowSumError):
        rs.rowsum_fwd_tuned(x, 96)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [1, 2, 3, 5, 10, 17, 31, 33, 63, 64, 65, 77, 100, 127, 129, 197, 255, 257, 300, 511, 512, 513, 1001, 1024])
def test_short_rows_any_alignment(gpu_device, N, dtype):
    """Rows of 1 to 1024 elements: runs of rows through LDS (two full tiles and a partial one), lane groups where the rows are whole aligned vectors, one workgroup
    per row; then the same with the base pointer one element off a 16-byte boundary, where the
    automatic path must still take the short-row kernels."""
    rows_per_tile = 16384 // (N * inputs.DTYPE_BYTES[dtype])
    M = 2 * rows_per_tile + 5 if rows_per_tile < 3000 else 4099
    case = inputs.rowsum_case(5, 1900 + 4 * dtype, M, N, dtype, mean=0.25, std=2.0)
    stats = check(case, gpu_device)
    assert 2 in stats
    want_y, want_abs = oracle.rowsum_oracle(case["x"], dtype, with_abs=True)
    flat = np.concatenate([np.zeros(1, dtype=case["x"].dtype), case["x"].reshape(-1)])
    xd = H.to_device(flat, dtype, gpu_device)[1:].view(M, N)
    for m in (0, 2, 64):
        y = run_mode(xd, m, "short rows, offset base")
        compare.check_rowsum_parity(y, want_y, want_abs, N, f"short rows, offset base [threads {m}]")
    for m in (8, 16, 32):
        with pytest.raises(rs.RowSumError):
            rs.rowsum_fwd_tuned(xd, m)


def test_through_lds_more_tiles_than_the_grid(gpu_device):
    """The grid stops at 8192 workgroups: 8 rows of 2 KiB per tile, 65536 + 13 rows."""
    M, N = 8192 * 8 + 13, 511
    case = inputs.rowsum_case(5, 1920, M, N, inputs.FP32)
    check(case, gpu_device, modes=(2,))
