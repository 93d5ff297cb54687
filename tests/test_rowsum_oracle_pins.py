"""Pins for the row-sum CPU oracle.

The paper prints no worked example for its "reduce" kernel (it names it in its "Supported
kernel types" table, "hierarchical warp shuffle", and reports 8192 x 8192 and 16384 x 4096
in its Section 7.1 results), so the oracle is pinned by exact rational arithmetic with one
exact rounding to fp32, an exactly rounded library sum (math.fsum), closed forms, IEEE
corner cases and invariants.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import BF16, FP16, FP32
from paper_2603_21331_amd import inputs

import exact

DTYPES = [FP32, FP16, BF16]


def storage(values, dtype):
    return inputs.to_storage(np.asarray(values, dtype=np.float64), dtype)


def f32_bits(y):
    return np.asarray(y, dtype=np.float32).view(np.uint32)


def exact_sum_bits(x_bits_row, dtype):
    """One row in exact rational arithmetic, one rounding to fp32."""
    total = sum((exact.fraction_of_bits(int(b), dtype) for b in x_bits_row), Fraction(0))
    return exact.round_to_bits(total, FP32)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(3, 1), (3, 2), (4, 7), (3, 33), (2, 130), (2, 1000), (1, 5000)])
@pytest.mark.parametrize("mean,std", [(0.0, 1.0), (3.0, 0.25), (-0.01, 40.0)])
def test_small_inputs_against_exact_arithmetic(dtype, shape, mean, std):
    M, N = shape
    x = inputs.normal_matrix(61, 1600 + dtype, M, N, dtype, mean, std)
    got = f32_bits(oracle.rowsum_oracle(x, dtype))
    xb = exact.to_int_bits(x, dtype)
    for i in range(M):
        assert int(got[i]) == exact_sum_bits(xb[i], dtype), (i, shape)


def test_half_precision_sums_are_exact_before_the_rounding():
    """Every fp16 value is a multiple of 2^-24 below 2^16, so a sum of up to 2^13 of them fits
    in 53 bits: the fp64 total is the exact total and the result is correctly rounded, even
    for the widest spread of magnitudes the format allows."""
    M, N = 6, 4096
    z = inputs.normal(62, 1610, 0, M * N).reshape(M, N)
    scale = 10.0 ** (-7.0 + 11.5 * inputs.uniform(62, 1611, 0, M * N).reshape(M, N))
    x = storage(z * scale, FP16)
    got = f32_bits(oracle.rowsum_oracle(x, FP16))
    for i in range(M):
        assert int(got[i]) == exact_sum_bits(exact.to_int_bits(x[i], FP16), FP16)


@pytest.mark.parametrize("dtype", DTYPES)
def test_against_the_exactly_rounded_library_sum(dtype):
    """math.fsum returns the exact sum rounded once to fp64; rounding that to fp32 differs from
    one direct rounding only within 2^-53 of an fp32 tie."""
    x = inputs.normal_matrix(63, 1620 + dtype, 40, 777, dtype, 0.5, 2.0)
    got = oracle.rowsum_oracle(x, dtype)
    wide = inputs.storage_to_f64(x, dtype)
    want = np.array([np.float32(math.fsum(row)) for row in wide], dtype=np.float32)
    assert np.array_equal(f32_bits(got), f32_bits(want))
    # and numpy's pairwise fp64 sum agrees to fp64 accuracy
    assert np.allclose(got.astype(np.float64), wide.sum(axis=1), rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [1, 2, 3, 64, 1000, 4096])
def test_constant_rows(dtype, N):
    for c in (0.0, 1.0, -2.5, 0.125, 96.0):
        x = storage(np.full((2, N), c), dtype)
        got = oracle.rowsum_oracle(x, dtype)
        assert np.all(got == np.float32(c * N)), (c, N)        # c * N is exact for these values


def test_hand_worked_rows():
    # 1 + 2 + ... + N = N (N + 1) / 2; alternating signs; a single entry; a cancellation that
    # an fp32 running total loses and an fp64 one keeps
    for N in (1, 2, 10, 100, 2000):
        row = np.arange(1, N + 1, dtype=np.float32)[None, :]
        assert oracle.rowsum_oracle(row, FP32)[0] == N * (N + 1) / 2
    alt = np.array([[7.5, -7.5] * 50, [7.5, -7.5] * 49 + [7.5, 1.0]], dtype=np.float32)
    assert list(oracle.rowsum_oracle(alt, FP32)) == [0.0, 8.5]
    one_hot = np.zeros((3, 17), dtype=np.float32)
    one_hot[0, 0], one_hot[1, 16], one_hot[2, 5] = 3.0, -4.0, 0.75
    assert list(oracle.rowsum_oracle(one_hot, FP32)) == [3.0, -4.0, 0.75]
    cancel = np.array([[1.0e8, 1.0, -1.0e8], [1.0, 1.0e8, -1.0e8], [3.0e7, 0.5, -3.0e7]], dtype=np.float32)
    assert list(oracle.rowsum_oracle(cancel, FP32)) == [1.0, 1.0, 0.5]
    # 2^24 + 1 + 1: an fp32 accumulator stays at 2^24; the exact total 2^24 + 2 is representable
    creep = np.array([[16777216.0, 1.0, 1.0]], dtype=np.float32)
    assert oracle.rowsum_oracle(creep, FP32)[0] == 16777218.0


def test_single_rounding_to_nearest_even():
    # exact totals halfway between two fp32 neighbours: 2^24 + 1 -> 2^24 (even), 2^24 + 3 -> 2^24 + 4
    x = np.array([[16777216.0, 1.0, 0.0], [16777216.0, 2.0, 1.0], [16777216.0, 1.0, 0.25],
                  [-16777216.0, -1.0, 0.0], [-16777216.0, -2.0, -1.0]], dtype=np.float32)
    assert list(oracle.rowsum_oracle(x, FP32)) == [16777216.0, 16777220.0, 16777218.0, -16777216.0, -16777220.0]


def test_the_output_is_fp32_for_every_storage_type():
    # 257 * 1.00390625 is not a bf16 or fp16 number; the result must keep its fp32 digits
    for dtype in (FP16, BF16):
        x = storage(np.full((1, 257), 1.0 + 2.0 ** -7), dtype)
        y = oracle.rowsum_oracle(x, dtype)
        assert y.dtype == np.float32 and y[0] == np.float32(257 * (1.0 + 2.0 ** -7))


def test_subnormals_and_format_limits():
    tiny16 = np.array([[1, 1, 1, 0x8001, 0x03FF]], dtype=np.uint16)         # fp16 subnormals, in bits
    assert oracle.rowsum_oracle(tiny16, FP16)[0] == np.float32((2 + 1023) * 2.0 ** -24)
    big16 = np.array([[0x7BFF] * 3], dtype=np.uint16)                        # 3 * 65504
    assert oracle.rowsum_oracle(big16, FP16)[0] == 196512.0
    tinyb = np.array([[0x0001, 0x0001, 0x8001, 0x0080]], dtype=np.uint16)    # bf16 subnormals + min normal
    assert oracle.rowsum_oracle(tinyb, BF16)[0] == np.float32(2.0 ** -133 + 2.0 ** -126)
    tiny32 = np.array([[1.0e-45, 1.0e-45, 1.0e-45]], dtype=np.float32)       # 3 * 2^-149
    assert oracle.rowsum_oracle(tiny32, FP32)[0] == np.float32(3 * 2.0 ** -149)
    big32 = np.array([[3.0e38, 3.0e38], [3.0e38, -3.0e38], [-3.0e38, -3.0e38]], dtype=np.float32)
    y = oracle.rowsum_oracle(big32, FP32)
    assert y[0] == np.inf and y[1] == 0.0 and y[2] == -np.inf                # overflow of the result only


def test_infinities_and_nan():
    inf, nan = np.inf, np.nan
    x = np.array([[1.0, inf, 2.0], [1.0, -inf, 2.0], [inf, -inf, 2.0], [1.0, nan, 2.0], [inf, inf, 1.0]],
                 dtype=np.float32)
    y = oracle.rowsum_oracle(x, FP32)
    assert y[0] == inf and y[1] == -inf and np.isnan(y[2]) and np.isnan(y[3]) and y[4] == inf
    h = np.array([[0x7C00, 0x3C00], [0xFC00, 0x7C00], [0x7E00, 0x3C00]], dtype=np.uint16)
    yh = oracle.rowsum_oracle(h, FP16)
    assert yh[0] == inf and np.isnan(yh[1]) and np.isnan(yh[2])


@pytest.mark.parametrize("dtype", DTYPES)
def test_sum_of_magnitudes_output(dtype):
    x = inputs.normal_matrix(64, 1630 + dtype, 7, 300, dtype, 0.2, 3.0)
    y, a = oracle.rowsum_oracle(x, dtype, with_abs=True)
    wide = inputs.storage_to_f64(x, dtype)
    assert a.dtype == np.float64
    assert np.allclose(a, np.abs(wide).sum(axis=1), rtol=1e-13, atol=0)
    assert np.all(a >= np.abs(y.astype(np.float64)) * (1 - 1e-6))
    pos = storage(np.abs(wide), dtype)
    assert np.allclose(oracle.rowsum_oracle(pos, dtype).astype(np.float64), a, rtol=1e-7)


@pytest.mark.parametrize("dtype", DTYPES)
def test_symmetries(dtype):
    M, N = 9, 77
    x = inputs.normal_matrix(65, 1640 + dtype, M, N, dtype)
    y = oracle.rowsum_oracle(x, dtype)
    wide = inputs.storage_to_f64(x, dtype)
    # negation and power-of-two scaling are exact
    assert np.array_equal(oracle.rowsum_oracle(storage(-wide, dtype), dtype), -y)
    assert np.array_equal(oracle.rowsum_oracle(storage(4.0 * wide, dtype), dtype), np.float32(4.0) * y)
    # rows are independent, in any order and under any thread count
    perm = np.argsort(inputs.uniform(1, 2, 0, M))
    assert np.array_equal(oracle.rowsum_oracle(x[perm], dtype), y[perm])
    for i in (0, 4, 8):
        assert oracle.rowsum_oracle(x[i:i + 1], dtype)[0] == y[i]
    for nt in (1, 2, 3, 8):
        assert np.array_equal(oracle.rowsum_oracle(x, dtype, nthreads=nt), y)
    # column order changes the fp64 total by rounding noise only
    cp = np.argsort(inputs.uniform(1, 3, 0, N))
    yc = oracle.rowsum_oracle(np.ascontiguousarray(x[:, cp]), dtype)
    assert np.allclose(yc, y, rtol=1e-6, atol=1e-6)
    # additivity over a split of the columns (fp64 totals of the halves, rounded afterwards)
    left = oracle.rowsum_oracle(np.ascontiguousarray(x[:, :30]), dtype).astype(np.float64)
    right = oracle.rowsum_oracle(np.ascontiguousarray(x[:, 30:]), dtype).astype(np.float64)
    assert np.allclose(left + right, y, rtol=1e-6, atol=1e-5)


def test_rows_are_read_row_major():
    x = np.arange(12, dtype=np.float32).reshape(3, 4)            # rows 0..3, 4..7, 8..11
    assert list(oracle.rowsum_oracle(x, FP32)) == [6.0, 22.0, 38.0]
    assert list(oracle.rowsum_oracle(np.ascontiguousarray(x.T), FP32)) == [12.0, 15.0, 18.0, 21.0]


def test_oracle_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.rowsum_oracle(np.zeros(4, dtype=np.float32), FP32)
    with pytest.raises(TypeError):
        oracle.rowsum_oracle(np.zeros((2, 4), dtype=np.float32), BF16)
    with pytest.raises(ValueError):
        oracle.rowsum_oracle(np.zeros((2, 0), dtype=np.float32), FP32)
    assert oracle.rowsum_oracle(np.zeros((0, 4), dtype=np.float32), FP32).shape == (0,)


def test_bytes_model_reproduces_the_papers_throughput_column():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_reduce_throughput.txt")
    with open(path) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 2
    for M, N, us, gbps in rows:
        M, N, us, gbps = int(M), int(N), float(us), float(gbps)
        mine = inputs.rowsum_bytes(M, N, FP16) / (us * 1e-6) / 1e9
        assert abs(mine - gbps) / gbps < 1.5e-3, (M, N, mine, gbps)
        assert abs(2 * mine - gbps) / gbps > 0.5                 # a read plus an equal write: far off
    case = inputs.rowsum_paper_shape(1)
    assert case["x"].shape == (16384, 4096) and case["dtype"] == FP16


def test_comparator_rejects_what_it_should():
    import compare
    o = np.float32([10.0, 0.0, np.inf, -3.0])
    a = np.float64([100.0, 0.0, np.inf, 50.0])
    compare.check_rowsum_parity(np.float32([10.00001, 0.0, np.inf, -3.000001]), o, a, 1000)
    for g in ([10.01, 0.0, np.inf, -3.0], [10.0, 1e-3, np.inf, -3.0], [10.0, 0.0, 1.0, -3.0],
              [np.nan, 0.0, np.inf, -3.0], [10.0, 0.0, np.inf, 3.0]):
        with pytest.raises(AssertionError):
            compare.check_rowsum_parity(np.float32(g), o, a, 1000)
