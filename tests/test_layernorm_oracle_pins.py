"""Pins for the LayerNorm CPU oracle.

The paper prints no worked LayerNorm example (it names the kernel in its "Supported kernel
types" table, "Welford single-pass", and in its Section 7.1 results), so the oracle is pinned
by exact rational arithmetic on small inputs, closed forms, invariants of the definition and
numpy's own moments.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import BF16, FP16, FP32
from paper_2603_21331_amd import inputs

import exact
import compare

DTYPES = [FP32, FP16, BF16]


def storage(values, dtype):
    return inputs.to_storage(np.asarray(values, dtype=np.float64), dtype)


def bits_of(a, dtype):
    return exact.to_int_bits(a, dtype)


def exact_layernorm_bits(x_bits, w_bits, b_bits, eps32, dtype):
    """Exact moments, 300-bit square root, one exact rounding."""
    eps = Fraction(float(np.float32(eps32)))
    x_bits = np.asarray(x_bits)
    M, N = x_bits.shape
    W = [exact.fraction_of_bits(int(v), dtype) for v in w_bits]
    B = [exact.fraction_of_bits(int(v), dtype) for v in b_bits] if b_bits is not None else [Fraction(0)] * N
    out = np.zeros((M, N), dtype=np.uint32)
    for i in range(M):
        X = [exact.fraction_of_bits(int(v), dtype) for v in x_bits[i]]
        mu = sum(X) / N
        var = sum((v - mu) ** 2 for v in X) / N
        root = exact.sqrt_fraction(var + eps)
        for j in range(N):
            out[i, j] = exact.round_to_bits((X[j] - mu) * W[j] / root + B[j], dtype)
    return out


def case(seed, stream, M, N, dtype, bias=True, mean=0.0, std=1.0):
    return dict(x=inputs.normal_matrix(seed, stream, M, N, dtype, mean, std),
                w=inputs.normal_matrix(seed, stream + 1, 1, N, dtype, 1.0, 0.1)[0],
                b=inputs.normal_matrix(seed, stream + 2, 1, N, dtype, 0.0, 0.1)[0] if bias else None)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(2, 2), (3, 7), (4, 33), (2, 130)])
@pytest.mark.parametrize("eps", [1e-5, 1e-6])
@pytest.mark.parametrize("bias", [True, False])
def test_small_inputs_against_exact_rational_arithmetic(dtype, shape, eps, bias):
    M, N = shape
    c = case(41, 1200 + 4 * dtype, M, N, dtype, bias, mean=0.5, std=2.0)
    got = bits_of(oracle.layernorm_oracle(c["x"], c["w"], c["b"], eps, dtype), dtype)
    want = exact_layernorm_bits(bits_of(c["x"], dtype), bits_of(c["w"], dtype),
                                None if c["b"] is None else bits_of(c["b"], dtype), eps, dtype)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_outputs_near_a_rounding_tie_are_rounded_once(dtype):
    M, N, eps = 1 << 16, 16, 1e-5
    c = case(42, 1220 + 4 * dtype, M, N, dtype)
    got = bits_of(oracle.layernorm_oracle(c["x"], c["w"], c["b"], eps, dtype), dtype)
    xd, wd, bd = (inputs.storage_to_f64(c[k], dtype) for k in ("x", "w", "b"))
    v = np.abs((xd - xd.mean(1, keepdims=True)) / np.sqrt(xd.var(1, keepdims=True) + float(np.float32(eps))) * wd + bd)
    p, emin = exact.FORMATS[dtype][0], exact.FORMATS[dtype][1]
    e = np.maximum(np.floor(np.log2(np.where(v > 0, v, 1.0))), emin)
    frac = np.mod(v / np.exp2(e - (p - 1)), 1.0)
    near = (np.abs(frac - 0.5) < 2.0 ** -(24 - p)) & (frac != 0.5) & (v > 0)
    rows = np.unique(np.nonzero(near)[0])
    assert len(rows) >= 5
    rows = rows[:30]
    want = exact_layernorm_bits(bits_of(c["x"], dtype)[rows], bits_of(c["w"], dtype), bits_of(c["b"], dtype), eps, dtype)
    assert np.array_equal(got[rows], want)


@pytest.mark.parametrize("dtype", DTYPES)
def test_constant_row_gives_the_bias(dtype):
    """x == c: every centred value is exactly zero, so y = b (and 0 without a bias)."""
    for cval in (0.0, 3.5, -200.0):
        for N in (1, 5, 64, 257):
            x = storage(np.full((2, N), cval), dtype)
            c = case(43, 1240, 1, N, dtype)
            y = oracle.layernorm_oracle(x, c["w"], c["b"], 1e-5, dtype)
            assert np.array_equal(oracle.decode(y, dtype), np.broadcast_to(oracle.decode(c["b"], dtype), (2, N)))
            y0 = oracle.layernorm_oracle(x, c["w"], None, 1e-5, dtype)
            assert np.all(oracle.decode(y0, dtype) == 0.0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_two_valued_row_closed_form(dtype):
    """Half the row +a, half -a: mean 0, variance a^2, y = +-a w / sqrt(a^2 + eps) + b."""
    N, a, eps = 64, 1.5, 1e-5
    s = np.where(np.arange(N) % 2 == 0, 1.0, -1.0)
    x = storage((a * s)[None, :], dtype)
    c = case(44, 1250, 1, N, dtype)
    got = bits_of(oracle.layernorm_oracle(x, c["w"], c["b"], eps, dtype), dtype)[0]
    root = exact.sqrt_fraction(Fraction(a) ** 2 + Fraction(float(np.float32(eps))))
    for j in range(N):
        wq = exact.fraction_of_bits(int(bits_of(c["w"], dtype)[j]), dtype)
        bq = exact.fraction_of_bits(int(bits_of(c["b"], dtype)[j]), dtype)
        assert int(got[j]) == exact.round_to_bits(Fraction(a) * int(s[j]) * wq / root + bq, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
def test_exact_ties_round_to_even(dtype):
    """x = +-1 alternating, eps = 0: y = +-w + b exactly.  With b half an ulp of w the sum is an
    exact tie: w with an even significand stays, w with an odd one moves up to the even neighbour."""
    p = exact.FORMATS[dtype][0]
    ulp = 2.0 ** -(p - 1)
    N = 4
    x = storage([[1.0, -1.0, 1.0, -1.0]], dtype)
    w = storage([1.0, 1.0, 1.0 + ulp, 1.0 + ulp], dtype)
    b = storage([ulp / 2, ulp / 2, ulp / 2, ulp / 2], dtype)
    y = oracle.decode(oracle.layernorm_oracle(x, w, b, 0.0, dtype), dtype)[0]
    assert y[0] == 1.0                       # 1 + ulp/2 -> even neighbour 1
    assert y[1] == -1.0 + ulp / 2            # exactly representable (finer spacing below 1)
    assert y[2] == 1.0 + 2 * ulp             # 1 + ulp + ulp/2 -> even neighbour 1 + 2 ulp
    assert N == 4


def test_hand_worked_example():
    # x = [1, 2, 3, 4]: mean 2.5, centred [-1.5, -0.5, 0.5, 1.5], variance 1.25
    x = np.array([[1, 2, 3, 4]], dtype=np.float32)
    y = oracle.layernorm_oracle(x, np.ones(4, dtype=np.float32), np.zeros(4, dtype=np.float32), 0.0, FP32)[0]
    want = (np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25)).astype(np.float32)
    assert np.array_equal(y, want)


def test_statistics_against_numpy_moments():
    for dtype in DTYPES:
        c = case(45, 1260 + 4 * dtype, 16, 1000, dtype, mean=3.0, std=0.3)
        _, mu, rstd = oracle.layernorm_oracle(c["x"], c["w"], c["b"], 1e-5, dtype, stats=True)
        xd = inputs.storage_to_f64(c["x"], dtype)
        assert np.allclose(mu, xd.mean(axis=1), rtol=1e-13, atol=1e-15)
        eps = float(np.float32(1e-5))
        assert np.allclose(rstd, 1.0 / np.sqrt(xd.var(axis=1) + eps), rtol=1e-12)
        # the nearest wrong readings are far outside that band
        assert not np.allclose(rstd, 1.0 / np.sqrt(xd.var(axis=1, ddof=1) + eps), rtol=1e-5)
        assert not np.allclose(rstd, 1.0 / np.sqrt((xd * xd).mean(axis=1) + eps), rtol=1e-3)
        assert not np.allclose(rstd, 1.0 / (np.sqrt(xd.var(axis=1)) + eps), rtol=1e-6)


def test_normalised_rows_have_zero_mean_and_unit_variance():
    c = case(46, 1270, 32, 512, FP32, mean=-4.0, std=3.0)
    y = oracle.layernorm_oracle(c["x"], c["w"], c["b"], 1e-12, FP32).astype(np.float64)
    z = (y - c["b"].astype(np.float64)) / c["w"].astype(np.float64)
    assert np.all(np.abs(z.mean(axis=1)) < 1e-6)
    assert np.all(np.abs(z.var(axis=1) - 1.0) < 1e-5)


@pytest.mark.parametrize("dtype", DTYPES)
def test_shift_and_scale_invariance(dtype):
    """eps = 0: LN(2^k x) = LN(x) bit for bit; LN(x + c) = LN(x) when x + c is exact."""
    k = np.round(inputs.normal(47, 1280, 0, 6 * 40).reshape(6, 40) * 4.0)
    c = case(47, 1284, 1, 40, dtype)
    x = storage(k, dtype)
    y0 = oracle.layernorm_oracle(x, c["w"], c["b"], 0.0, dtype)
    assert np.array_equal(oracle.layernorm_oracle(storage(k * 4.0, dtype), c["w"], c["b"], 0.0, dtype), y0)
    assert np.array_equal(oracle.layernorm_oracle(storage(k + 64.0, dtype), c["w"], c["b"], 0.0, dtype), y0)
    yn = oracle.layernorm_oracle(storage(-k, dtype), c["w"], None, 0.0, dtype)
    yp = oracle.layernorm_oracle(x, c["w"], None, 0.0, dtype)
    assert np.array_equal(oracle.decode(yn, dtype), -oracle.decode(yp, dtype))


@pytest.mark.parametrize("dtype", DTYPES)
def test_symmetries(dtype):
    c = case(48, 1290 + 4 * dtype, 9, 77, dtype)
    y = oracle.layernorm_oracle(c["x"], c["w"], c["b"], 1e-5, dtype)
    perm = np.argsort(inputs.uniform(1, 2, 0, 9))
    assert np.array_equal(oracle.layernorm_oracle(c["x"][perm], c["w"], c["b"], 1e-5, dtype), y[perm])
    for i in (0, 4, 8):
        assert np.array_equal(oracle.layernorm_oracle(c["x"][i:i + 1], c["w"], c["b"], 1e-5, dtype)[0], y[i])
    for nt in (1, 2, 3, 8):
        assert np.array_equal(oracle.layernorm_oracle(c["x"], c["w"], c["b"], 1e-5, dtype, nthreads=nt), y)
    cp = np.argsort(inputs.uniform(1, 3, 0, 77))
    yc = oracle.layernorm_oracle(np.ascontiguousarray(c["x"][:, cp]), c["w"][cp], c["b"][cp], 1e-5, dtype)
    if dtype == FP32:
        assert np.allclose(yc, y[:, cp], rtol=1e-5, atol=1e-6)
    else:
        assert compare.ulp_distance(yc, y[:, cp], dtype).max() <= 1


def test_weight_and_bias_are_indexed_by_column():
    N = 8
    c = case(49, 1300, N, N, FP32)
    w = np.zeros(N, dtype=np.float32)
    w[3] = 2.0
    b = np.arange(N, dtype=np.float32)
    y = oracle.layernorm_oracle(c["x"], w, b, 1e-5, FP32)
    others = [0, 1, 2, 4, 5, 6, 7]
    assert np.array_equal(y[:, others], np.broadcast_to(b[others], (N, 7)))
    assert np.all(y[:, 3] != 3.0)


def test_large_mean_small_spread_is_handled():
    """Mean 1000, spread 0.01: a one-pass E[x^2] - E[x]^2 in low precision would cancel badly;
    the oracle's centred second pass must agree with exact arithmetic."""
    c = case(50, 1310, 3, 50, FP32, mean=1000.0, std=0.01)
    got = bits_of(oracle.layernorm_oracle(c["x"], c["w"], c["b"], 1e-5, FP32), FP32)
    want = exact_layernorm_bits(bits_of(c["x"], FP32), bits_of(c["w"], FP32), bits_of(c["b"], FP32), 1e-5, FP32)
    assert np.array_equal(got, want)


def test_oracle_rejects_bad_arguments():
    x = np.zeros((2, 4), dtype=np.float32)
    w = np.ones(4, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.layernorm_oracle(x, w, None, -1.0, FP32)
    with pytest.raises(ValueError):
        oracle.layernorm_oracle(x, np.ones(5, dtype=np.float32), None, 1e-5, FP32)
    with pytest.raises(ValueError):
        oracle.layernorm_oracle(x, w, np.ones(3, dtype=np.float32), 1e-5, FP32)
    with pytest.raises(TypeError):
        oracle.layernorm_oracle(x, w, None, 1e-5, BF16)
    assert oracle.layernorm_oracle(np.zeros((0, 4), dtype=np.float32), w, None, 1e-5, FP32).shape == (0, 4)
