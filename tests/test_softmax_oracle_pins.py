"""Pins for the softmax CPU oracle.

The paper prints no worked softmax example (it names the kernel in its "Supported kernel
types" table, its Section 7.1 results and its Section 4 stability probe, "rows of large
identical values"), so the oracle is pinned by an arbitrary-precision reference (mpmath at
60 digits, rounded by this repository's exact rational rounding), closed forms, IEEE corner
cases and invariants of the definition.
"""
import math
from fractions import Fraction

import mpmath
import numpy as np
import pytest

import oracle
from oracle import BF16, FP16, FP32
from paper_2603_21331_amd import inputs

import exact
import compare

DTYPES = [FP32, FP16, BF16]
mpmath.mp.dps = 60


def storage(values, dtype):
    return inputs.to_storage(np.asarray(values, dtype=np.float64), dtype)


def bits_of(a, dtype):
    return exact.to_int_bits(a, dtype)


def mp_softmax_bits(x_bits_row, dtype):
    """One row through mpmath: exact inputs, 60-digit exp and sum, one exact rounding."""
    xs = [exact.fraction_of_bits(int(b), dtype) for b in x_bits_row]
    m = max(xs)
    es = [mpmath.exp(mpmath.mpf((v - m).numerator) / mpmath.mpf((v - m).denominator)) for v in xs]
    s = mpmath.fsum(es)
    out = []
    for e in es:
        q = e / s
        man, exp = int(q.man), int(q.exp)
        fr = Fraction(man) * (Fraction(2) ** exp)
        if q._mpf_[0]:
            fr = -fr
        out.append(exact.round_to_bits(fr, dtype))
    return out


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(1, 1), (3, 2), (4, 7), (3, 33), (2, 130)])
@pytest.mark.parametrize("scale", [1.0, 8.0, 0.01])
def test_small_inputs_against_arbitrary_precision(dtype, shape, scale):
    M, N = shape
    z = inputs.normal(31, 1000 + dtype, 0, M * N).reshape(M, N) * scale
    x = storage(z, dtype)
    got = bits_of(oracle.softmax_oracle(x, dtype), dtype)
    xb = bits_of(x, dtype)
    for i in range(M):
        assert list(got[i]) == mp_softmax_bits(xb[i], dtype)


@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_outputs_near_a_rounding_tie_are_rounded_once(dtype):
    """numpy only LOCATES outputs within an fp32 half-ulp of a 16-bit rounding tie in a
    million-element input (where rounding twice would land one ulp off); the 60-digit
    reference decides the right bits for the rows that hold them."""
    M, N = 1 << 16, 16
    x = inputs.normal_matrix(35, 1040 + dtype, M, N, dtype)
    got = bits_of(oracle.softmax_oracle(x, dtype), dtype)
    xd = inputs.storage_to_f64(x, dtype)
    e = np.exp(xd - xd.max(axis=1, keepdims=True))
    v = e / e.sum(axis=1, keepdims=True)
    p, emin = exact.FORMATS[dtype][0], exact.FORMATS[dtype][1]
    ex = np.maximum(np.floor(np.log2(v)), emin)
    frac = np.mod(v / np.exp2(ex - (p - 1)), 1.0)
    near = (np.abs(frac - 0.5) < 2.0 ** -(24 - p)) & (frac != 0.5)
    rows = np.unique(np.nonzero(near)[0])
    assert len(rows) >= 5, "the input must contain elements in the double-rounding window"
    xb = bits_of(x, dtype)
    for i in rows[:40]:
        assert list(got[i]) == mp_softmax_bits(xb[i], dtype)


@pytest.mark.parametrize("dtype", DTYPES)
def test_wide_dynamic_range_and_subnormal_outputs(dtype):
    """Differences large enough that some outputs are subnormal or round to zero."""
    rows = {
        FP32: [[0.0, -100.0, -95.0, -103.5, -104.0, -110.0, 3.0], [50.0, -50.0, 49.5, -37.0]],
        FP16: [[0.0, -10.0, -15.0, -16.5, -17.0, -17.5, -20.0, 1.0], [11.0, -6.0, 10.5, 0.0]],
        BF16: [[0.0, -88.0, -90.0, -92.0, -93.0, -95.0, 2.0], [40.0, -50.0, 39.5, -30.0]],
    }[dtype]
    for r in rows:
        x = storage([r], dtype)
        got = bits_of(oracle.softmax_oracle(x, dtype), dtype)[0]
        want = mp_softmax_bits(bits_of(x, dtype)[0], dtype)
        assert list(got) == want
    p, emin = exact.FORMATS[dtype][0], exact.FORMATS[dtype][1]
    x = storage([rows[0]], dtype)
    y = bits_of(oracle.softmax_oracle(x, dtype), dtype)[0]
    mant_bits = p - 1
    mag = y & ((1 << (mant_bits + exact.FORMATS[dtype][3])) - 1)
    assert np.any((mag > 0) & (mag < (1 << mant_bits))), "the row must produce a subnormal output"


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [1, 2, 3, 7, 64, 1000])
def test_constant_rows_give_one_over_n(dtype, N):
    """Includes the paper's stability probe: rows of large identical values."""
    big = {FP32: 3.0e38, FP16: 60000.0, BF16: 3.0e38}[dtype]
    want = exact.round_to_bits(Fraction(1, N), dtype)
    for c in (0.0, -7.25, 1.0, big, -big):
        x = storage(np.full((2, N), c), dtype)
        got = bits_of(oracle.softmax_oracle(x, dtype), dtype)
        assert np.all(got == want), (c, N)


@pytest.mark.parametrize("dtype", DTYPES)
def test_dominant_entry_gives_exact_one_hot(dtype):
    """One entry more than 745 above the rest: every other exp underflows fp64 itself."""
    hi = {FP32: 1000.0, FP16: 1000.0, BF16: 1000.0}[dtype]
    z = np.full((1, 9), -200.0)
    z[0, 4] = hi
    y = oracle.decode(oracle.softmax_oracle(storage(z, dtype), dtype), dtype)[0]
    assert y[4] == 1.0 and np.all(np.delete(y, 4) == 0.0)


def test_two_entry_row_is_the_logistic_function():
    for a, b in ((0.0, 0.0), (1.0, 0.0), (0.5, -2.25), (-3.0, 4.0)):
        y = oracle.softmax_oracle(np.array([[a, b]], dtype=np.float32), FP32)[0].astype(np.float64)
        assert abs(y[0] - 1.0 / (1.0 + math.exp(b - a))) < 1e-7
        assert abs(y[1] - 1.0 / (1.0 + math.exp(a - b))) < 1e-7


def test_shift_invariance_is_bit_exact_when_the_shift_is_exact():
    """softmax(x + c) = softmax(x); with integer-valued fp32 inputs x + c is exact, the
    differences x - max are the same numbers, so the bits must not move."""
    k = np.round(inputs.normal(32, 1010, 0, 5 * 40).reshape(5, 40) * 6.0)
    x = k.astype(np.float32)
    y0 = oracle.softmax_oracle(x, FP32)
    for c in (1000.0, -4096.0, 0.0):
        assert np.array_equal(oracle.softmax_oracle((k + c).astype(np.float32), FP32), y0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_rows_sum_to_one_and_order_is_preserved(dtype):
    x = inputs.normal_matrix(33, 1020 + dtype, 16, 777, dtype, 0.0, 2.0)
    y = oracle.decode(oracle.softmax_oracle(x, dtype), dtype)
    xd = inputs.storage_to_f64(x, dtype)
    ulp = 2.0 ** -(exact.FORMATS[dtype][0] - 1)
    assert np.all(np.abs(y.sum(axis=1) - 1.0) < 777 * ulp * y.max(axis=1) + 1e-12)
    assert np.all(y >= 0.0) and np.all(y <= 1.0)
    for i in range(16):
        order = np.argsort(xd[i], kind="stable")
        assert np.all(np.diff(y[i][order]) >= 0.0)
    # ratios: y_j / y_k = exp(x_j - x_k), checked on the two largest entries of each row
    for i in range(16):
        j, k = np.argsort(xd[i])[-1], np.argsort(xd[i])[-2]
        assert abs(y[i, j] / y[i, k] - math.exp(xd[i, j] - xd[i, k])) < 8 * ulp * math.exp(xd[i, j] - xd[i, k])


def test_infinities_and_nan():
    ninf, nan = -np.inf, np.nan
    x = np.array([[0.0, ninf, 1.0, ninf], [ninf, ninf, ninf, ninf], [0.0, nan, 1.0, 2.0],
                  [0.0, np.inf, 1.0, 2.0], [5.0, ninf, ninf, ninf]], dtype=np.float32)
    y = oracle.softmax_oracle(x, FP32)
    sub = oracle.softmax_oracle(np.array([[0.0, 1.0]], dtype=np.float32), FP32)[0]
    assert y[0, 1] == 0.0 and y[0, 3] == 0.0
    assert np.array_equal(y[0, [0, 2]], sub)          # -inf entries drop out of the row exactly
    assert np.all(np.isnan(y[1])) and np.all(np.isnan(y[2])) and np.all(np.isnan(y[3]))
    assert np.array_equal(y[4], np.array([1.0, 0.0, 0.0, 0.0], dtype=np.float32))


@pytest.mark.parametrize("dtype", DTYPES)
def test_symmetries(dtype):
    x = inputs.normal_matrix(34, 1030 + dtype, 9, 77, dtype)
    y = oracle.softmax_oracle(x, dtype)
    perm = np.argsort(inputs.uniform(1, 2, 0, 9))
    assert np.array_equal(oracle.softmax_oracle(x[perm], dtype), y[perm])
    for i in (0, 4, 8):
        assert np.array_equal(oracle.softmax_oracle(x[i:i + 1], dtype)[0], y[i])
    for nt in (1, 2, 3, 8):
        assert np.array_equal(oracle.softmax_oracle(x, dtype, nthreads=nt), y)
    cp = np.argsort(inputs.uniform(1, 3, 0, 77))
    yc = oracle.softmax_oracle(np.ascontiguousarray(x[:, cp]), dtype)
    if dtype == FP32:
        assert compare.max_rel_err_fp32(yc, y[:, cp]) < 1e-6
    else:
        assert compare.ulp_distance(yc, y[:, cp], dtype).max() <= 1


def test_reduction_runs_along_rows_not_columns():
    x = np.zeros((3, 4), dtype=np.float32)
    x[0] = [0, 0, 0, 0]
    x[1] = [10, 0, 0, 0]
    x[2] = [0, 0, 0, 10]
    y = oracle.softmax_oracle(x, FP32)
    assert np.allclose(y.sum(axis=1), 1.0, atol=1e-6)
    assert y[1, 0] > 0.99 and y[2, 3] > 0.99 and np.all(y[0] == 0.25)


def test_oracle_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.softmax_oracle(np.zeros((2, 0), dtype=np.float32), FP32)
    with pytest.raises(TypeError):
        oracle.softmax_oracle(np.zeros((2, 4), dtype=np.float32), BF16)
    with pytest.raises(ValueError):
        oracle.softmax_oracle(np.zeros(4, dtype=np.float32), FP32)
    assert oracle.softmax_oracle(np.zeros((0, 4), dtype=np.float32), FP32).shape == (0, 4)
