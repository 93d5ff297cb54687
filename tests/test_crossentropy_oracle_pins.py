"""Pins for the cross-entropy CPU oracle.

The paper prints no worked example (it names the kernel "cross_ent" in its "Supported kernel
types" table, "online log-sum-exp, fused NLL", and in its Section 7.1 results), so the oracle is
pinned by a 60-digit mpmath reference with correct rounding to fp32, closed forms, IEEE corner
cases, invariants, and the independent softmax oracle (loss = -log softmax[target]).
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

DTYPES = [FP32, FP16, BF16]
mpmath.mp.dps = 60


def storage(values, dtype):
    return inputs.to_storage(np.asarray(values, dtype=np.float64), dtype)


def mp_loss_bits(x_bits_row, t, dtype):
    """One row through mpmath: exact inputs, 60-digit lse, one exact rounding to fp32."""
    xs = [exact.fraction_of_bits(int(b), dtype) for b in x_bits_row]
    mp = [mpmath.mpf(v.numerator) / mpmath.mpf(v.denominator) for v in xs]
    m = max(mp)
    q = m + mpmath.log(mpmath.fsum(mpmath.exp(v - m) for v in mp)) - mp[t]
    if q == 0:
        return 0
    fr = Fraction(int(q.man)) * Fraction(2) ** int(q.exp)
    if q < 0:
        fr = -fr
    return exact.round_to_bits(fr, FP32)


def loss_bits(loss):
    return np.asarray(loss, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(3, 2), (4, 7), (3, 33), (2, 130), (2, 1000)])
@pytest.mark.parametrize("scale", [1.0, 6.0, 0.05])
def test_small_inputs_against_arbitrary_precision(dtype, shape, scale):
    M, N = shape
    x = storage(inputs.normal(51, 1500 + dtype, 0, M * N).reshape(M, N) * scale, dtype)
    t = (inputs.raw_u64(51, 1510, 0, M) % np.uint64(N)).astype(np.int64)
    got = loss_bits(oracle.crossentropy_oracle(x, t, dtype))
    xb = exact.to_int_bits(x, dtype)
    for i in range(M):
        assert int(got[i]) == mp_loss_bits(xb[i], int(t[i]), dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("N", [1, 2, 3, 7, 64, 1000, 32000])
def test_constant_rows_give_log_n(dtype, N):
    big = {FP32: 3.0e38, FP16: 60000.0, BF16: 3.0e38}[dtype]
    want = np.float32(math.log(N))
    for c in (0.0, -7.25, big, -big):
        x = storage(np.full((2, N), c), dtype)
        got = oracle.crossentropy_oracle(x, np.array([0, N - 1]), dtype)
        assert np.all(np.abs(got.astype(np.float64) - math.log(N)) <= abs(float(want)) * 2.0 ** -23), (c, N)


def test_two_class_row_is_the_logistic_loss():
    for a, b in ((0.0, 0.0), (1.0, 0.0), (0.5, -2.25), (-3.0, 4.0), (30.0, -30.0)):
        l = oracle.crossentropy_oracle(np.array([[a, b], [a, b]], dtype=np.float32), np.array([0, 1]), FP32)
        assert abs(l[0] - math.log1p(math.exp(b - a))) <= 1e-7 * max(1.0, l[0])
        assert abs(l[1] - math.log1p(math.exp(a - b))) <= 1e-7 * max(1.0, l[1])


def test_dominant_logit():
    z = np.full((2, 9), -200.0)
    z[:, 4] = 1000.0
    l = oracle.crossentropy_oracle(z.astype(np.float32), np.array([4, 0]), FP32)
    assert l[0] == 0.0 and l[1] == 1200.0


@pytest.mark.parametrize("dtype", DTYPES)
def test_against_the_softmax_oracle(dtype):
    """loss = -log softmax(x)[target]; the softmax oracle is a separate file with its own code."""
    x = inputs.normal_matrix(52, 1520 + dtype, 32, 500, dtype, 0.0, 2.0)
    t = (inputs.raw_u64(52, 1530, 0, 32) % np.uint64(500)).astype(np.int64)
    loss = oracle.crossentropy_oracle(x, t, dtype).astype(np.float64)
    p = oracle.softmax_oracle(inputs.storage_to_f64(x, dtype).astype(np.float32), FP32).astype(np.float64)
    want = -np.log(p[np.arange(32), t])
    assert np.allclose(loss, want, rtol=2e-6, atol=1e-6)


def test_shift_invariance_and_lse_shift():
    k = np.round(inputs.normal(53, 1540, 0, 5 * 40).reshape(5, 40) * 6.0)
    t = np.array([0, 7, 39, 20, 3])
    l0, lse0 = oracle.crossentropy_oracle(k.astype(np.float32), t, FP32, with_lse=True)
    for c in (1000.0, -4096.0):
        l1, lse1 = oracle.crossentropy_oracle((k + c).astype(np.float32), t, FP32, with_lse=True)
        assert np.allclose(lse1, lse0 + c, rtol=0, atol=1e-9)
        assert np.allclose(l1, l0, rtol=1e-6, atol=1e-6)
    assert np.all(l0 >= 0.0)


def test_target_selects_the_column_of_its_own_row():
    x = np.zeros((3, 4), dtype=np.float32)
    x[0] = [5, 0, 0, 0]
    x[1] = [0, 5, 0, 0]
    x[2] = [0, 0, 0, 5]
    lse = math.log(math.exp(5) + 3)
    l = oracle.crossentropy_oracle(x, np.array([0, 0, 3]), FP32).astype(np.float64)
    assert abs(l[0] - (lse - 5)) < 1e-6 and abs(l[1] - lse) < 1e-6 and abs(l[2] - (lse - 5)) < 1e-6


def test_ignored_rows_infinities_and_nan():
    ninf, nan = -np.inf, np.nan
    x = np.array([[0.0, ninf, 1.0, ninf], [ninf, ninf, ninf, ninf], [0.0, nan, 1.0, 2.0],
                  [0.0, np.inf, 1.0, 2.0], [0.0, 1.0, 2.0, 3.0], [0.0, 1.0, 2.0, 3.0], [0.0, ninf, 1.0, 2.0]],
                 dtype=np.float32)
    t = np.array([2, 0, 0, 0, -100, 4, 1])
    l = oracle.crossentropy_oracle(x, t, FP32)
    assert abs(l[0] - math.log1p(math.exp(-1.0))) < 1e-7      # -inf logits drop out
    assert np.isnan(l[1]) and np.isnan(l[2]) and np.isnan(l[3])
    assert l[4] == 0.0 and l[5] == 0.0                         # targets outside [0, N): ignored
    assert l[6] == np.inf                                      # target on a -inf logit


@pytest.mark.parametrize("dtype", DTYPES)
def test_symmetries(dtype):
    x = inputs.normal_matrix(54, 1550 + dtype, 9, 77, dtype)
    t = (inputs.raw_u64(54, 1560, 0, 9) % np.uint64(77)).astype(np.int64)
    l = oracle.crossentropy_oracle(x, t, dtype)
    perm = np.argsort(inputs.uniform(1, 2, 0, 9))
    assert np.array_equal(oracle.crossentropy_oracle(x[perm], t[perm], dtype), l[perm])
    for i in (0, 4, 8):
        assert oracle.crossentropy_oracle(x[i:i + 1], t[i:i + 1], dtype)[0] == l[i]
    for nt in (1, 2, 3, 8):
        assert np.array_equal(oracle.crossentropy_oracle(x, t, dtype, nthreads=nt), l)
    cp = np.argsort(inputs.uniform(1, 3, 0, 77))
    inv = np.argsort(cp)
    lc = oracle.crossentropy_oracle(np.ascontiguousarray(x[:, cp]), inv[t], dtype)
    assert np.allclose(lc, l, rtol=1e-6, atol=1e-7)


def test_oracle_rejects_bad_arguments():
    x = np.zeros((2, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.crossentropy_oracle(x, np.array([0, 1, 2]), FP32)
    with pytest.raises(TypeError):
        oracle.crossentropy_oracle(x, np.array([0, 1], dtype=np.int32), FP32)
    with pytest.raises(TypeError):
        oracle.crossentropy_oracle(x, np.array([0, 1]), BF16)
    assert oracle.crossentropy_oracle(np.zeros((0, 4), dtype=np.float32), np.zeros(0, dtype=np.int64), FP32).shape == (0,)


def test_bytes_model_reproduces_the_papers_throughput_column():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_crossentropy_throughput.txt")
    with open(path) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 2
    for M, N, us, gbps in rows:
        M, N, us, gbps = int(M), int(N), float(us), float(gbps)
        mine = inputs.crossentropy_bytes(M, N, FP16) / (us * 1e-6) / 1e9
        assert abs(mine - gbps) / gbps < 1e-3, (M, N, mine, gbps)
        other = inputs.crossentropy_bytes(M, 32768, FP16) / (us * 1e-6) / 1e9
        assert abs(other - gbps) / gbps > 2e-2
    case = inputs.crossentropy_paper_shape(0)
    assert case["x"].shape == (4096, 32000) and case["target"].min() >= 0 and case["target"].max() < 32000


def test_comparator_rejects_what_it_should():
    import compare
    compare.check_crossentropy_parity(np.float32([10.00005, 0.0, np.inf]), np.float32([10.0, 0.0, np.inf]))
    for g, o in (([10.0002], [10.0]), ([1e-4], [0.0]), ([np.nan], [1.0]), ([1.0], [np.inf]), ([np.inf], [1.0])):
        with pytest.raises(AssertionError):
            compare.check_crossentropy_parity(np.float32(g), np.float32(o))
    with pytest.raises(AssertionError):
        compare.check_crossentropy_parity(np.float32([1e-7]), np.float32([0.0]), exact_zero=np.array([True]))
