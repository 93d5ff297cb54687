"""Pins for the CPU oracle: it is checked here against things other than itself.

The paper prints no worked RMSNorm example (it names the kernel in its
"Supported kernel types" table and its Section 7.1 results), so the pins are:
exact rational arithmetic on small inputs, closed forms of special rows,
invariants of the definition, numpy's own float conversions, and a library
2-norm.  Each is chosen so that a plausible slip in the oracle (mean over N-1,
eps outside the root, a dropped element, a transposed index, a double rounding)
fails at least one test.
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
import compare

DTYPES = [FP32, FP16, BF16]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def storage(values, dtype):
    return inputs.to_storage(np.asarray(values, dtype=np.float64), dtype)


def bits_of(a, dtype):
    return exact.to_int_bits(a, dtype)


# ---------------------------------------------------------------- conversions

def test_decode_all_fp16_patterns_against_numpy():
    b = np.arange(65536, dtype=np.uint16)
    want = b.view(np.float16).astype(np.float64)
    got = oracle.decode(b, FP16)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_decode_all_bf16_patterns_against_float32_hardware():
    b = np.arange(65536, dtype=np.uint16)
    want = (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = oracle.decode(b, BF16)
    ok = ~np.isnan(want)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_decode_matches_exact_fraction(dtype):
    rng = np.random.default_rng(1)
    for b in rng.integers(0, 65536, 400):
        b = int(b)
        _, _, _, ebits = exact.FORMATS[dtype]
        mbits = exact.FORMATS[dtype][0] - 1
        if (b >> mbits) & ((1 << ebits) - 1) == (1 << ebits) - 1:
            continue
        got = oracle.decode(np.array([b], dtype=np.uint16), dtype)[0]
        assert Fraction(float(got)) == exact.fraction_of_bits(b, dtype)


@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_encode_roundtrips_every_finite_pattern(dtype):
    b = np.arange(65536, dtype=np.uint16)
    v = oracle.decode(b, dtype)
    ok = ~np.isnan(v)
    assert np.array_equal(oracle.encode(v[ok], dtype), b[ok])


def test_encode_fp16_against_numpy_single_rounding():
    rng = np.random.default_rng(2)
    v = np.concatenate([
        rng.standard_normal(50000) * 10.0 ** rng.uniform(-9, 6, 50000),
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 65520.001, 1e9, -1e9,
                  2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26, 6.1e-5]),
    ])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.encode(v, FP16), want)


def test_encode_fp32_against_hardware_conversion():
    rng = np.random.default_rng(3)
    v = np.concatenate([
        rng.standard_normal(50000) * 10.0 ** rng.uniform(-44, 38, 50000),
        np.array([0.0, -0.0, 3.4028234663852886e38, 3.4028235677973366e38, 1e39,
                  2.0 ** -149, 2.0 ** -150, 2.0 ** -150 * 1.0000001, 1.0 + 2.0 ** -24,
                  1.0 + 2.0 ** -24 + 2.0 ** -50, 1.0 + 3 * 2.0 ** -24]),
    ])
    with np.errstate(over="ignore"):
        want = v.astype(np.float32)
    got = oracle.encode(v, FP32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_encode_bf16_ties_and_double_rounding_trap():
    cases = {
        1.0 + 2.0 ** -8: 0x3F80,                      # exact tie -> even (1.0)
        1.0 + 3 * 2.0 ** -8: 0x3F82,                  # exact tie -> even (1 + 2^-6)
        1.0 + 2.0 ** -8 + 2.0 ** -30: 0x3F81,         # above the tie; fp32 first would give 0x3F80
        1.0 + 2.0 ** -8 - 2.0 ** -30: 0x3F80,
        -(1.0 + 2.0 ** -8 + 2.0 ** -30): 0xBF81,
        (2 - 2.0 ** -7) * 2.0 ** 127: 0x7F7F,          # max finite bf16
        float(np.nextafter((2 - 2.0 ** -8) * 2.0 ** 127, 0.0)): 0x7F7F,  # just under max + half ulp
        (2 - 2.0 ** -8) * 2.0 ** 127: 0x7F80,          # the halfway point rounds to even = inf
        1e39: 0x7F80,
        2.0 ** -133: 0x0001,                          # smallest subnormal
        2.0 ** -134: 0x0000,                          # tie -> even (0)
        2.0 ** -134 * 1.5: 0x0001,
        0.0: 0x0000,
    }
    v = np.array(list(cases.keys()))
    want = np.array(list(cases.values()), dtype=np.uint16)
    assert np.array_equal(oracle.encode(v, BF16), want)
    assert oracle.encode(np.array([-0.0]), BF16)[0] == 0x8000


@pytest.mark.parametrize("dtype", DTYPES)
def test_encode_against_exact_rounding(dtype):
    rng = np.random.default_rng(4 + dtype)
    lo, hi = {FP32: (-46, 39), FP16: (-9, 6), BF16: (-42, 39)}[dtype]
    v = rng.standard_normal(600) * 10.0 ** rng.uniform(lo, hi, 600)
    got = bits_of(oracle.encode(v, dtype), dtype)
    for k in range(v.size):
        assert int(got[k]) == exact.round_to_bits(Fraction(float(v[k])), dtype), float(v[k])


# ------------------------------------------------ exact arithmetic, small inputs

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(1, 1), (2, 2), (3, 7), (4, 33), (2, 130)])
@pytest.mark.parametrize("eps", [1e-6, 1e-5, 0.0])
def test_small_inputs_against_exact_rational_arithmetic(dtype, shape, eps):
    M, N = shape
    c = inputs.random_case(11, 200 + 2 * dtype, M, N, dtype, eps)
    got = bits_of(oracle.rmsnorm_oracle(c["x"], c["w"], eps, dtype), dtype)
    want = exact.rmsnorm_exact_bits(bits_of(c["x"], dtype), bits_of(c["w"], dtype), eps, dtype)
    assert np.array_equal(got, want)


def test_adversarial_magnitudes_against_exact_arithmetic():
    """Rows like the adversarial workload's: tiny scale, huge scale, a 60000 spike, zeros."""
    N = 24
    z = inputs.normal(5, 7, 0, 5 * N).reshape(5, N)
    z[0] *= 1e-4
    z[1] *= 1e4
    z[2] *= 1e-2
    z[2, 5] = -60000.0
    z[3] = 0.0
    z[4] = 0.0
    z[4, 23] = 60000.0
    x = storage(z, FP16)
    w = inputs.normal_matrix(5, 8, 1, N, FP16, 1.0, 0.1)[0]
    got = bits_of(oracle.rmsnorm_oracle(x, w, 1e-6, FP16), FP16)
    want = exact.rmsnorm_exact_bits(x, w, 1e-6, FP16)
    assert np.array_equal(got, want)
    assert np.all((got[3] & 0x7FFF) == 0)


@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_outputs_near_a_rounding_tie_are_rounded_once(dtype):
    """Outputs whose exact value lies within an fp32 half-ulp of a 16-bit rounding tie would come
    out one ulp off if the product were rounded to fp32 first.  numpy only LOCATES such
    elements in a million-element input; exact rational arithmetic then decides what the
    right bits are for the rows that hold them."""
    M, N, eps = 1 << 16, 16, 1e-6
    c = inputs.random_case(12, 260 + 2 * dtype, M, N, dtype, eps)
    got = bits_of(oracle.rmsnorm_oracle(c["x"], c["w"], eps, dtype), dtype)
    xd = inputs.storage_to_f64(c["x"], dtype)
    wd = inputs.storage_to_f64(c["w"], dtype)
    v = np.abs(xd / np.sqrt((xd * xd).mean(axis=1, keepdims=True) + float(np.float32(eps))) * wd)
    p = exact.FORMATS[dtype][0]
    emin = exact.FORMATS[dtype][1]
    with np.errstate(divide="ignore"):
        e = np.maximum(np.floor(np.log2(np.where(v > 0, v, 1.0))), emin)
    frac = np.mod(v / np.exp2(e - (p - 1)), 1.0)
    window = 2.0 ** -(24 - p)          # an fp32 half-ulp, in units of the 16-bit ulp
    near = (np.abs(frac - 0.5) < window) & (frac != 0.5) & (v > 0)
    rows = np.unique(np.nonzero(near)[0])
    assert len(rows) >= 5, "the input must contain elements in the double-rounding window"
    rows = rows[:40]
    want = exact.rmsnorm_exact_bits(bits_of(c["x"], dtype)[rows], bits_of(c["w"], dtype), eps, dtype)
    assert np.array_equal(got[rows], want)


# ------------------------------------------------------------------ closed forms

def _closed_form_bits(num: Fraction, under_root: Fraction, dtype):
    return exact.round_to_bits(num / exact.sqrt_fraction(under_root), dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("c", [0.5, -3.0, 1.0 / 3.0, 200.0, 1e-3])
def test_constant_row_closed_form(dtype, c):
    """x == c everywhere  =>  y_j = w_j * c / sqrt(c^2 + eps), whatever N is."""
    eps = 1e-5
    for N in (1, 5, 64, 257):
        x = storage(np.full((2, N), c), dtype)
        w = inputs.normal_matrix(3, 9, 1, N, dtype, 1.0, 0.1)[0]
        got = bits_of(oracle.rmsnorm_oracle(x, w, eps, dtype), dtype)
        cq = exact.fraction_of_bits(int(bits_of(x, dtype)[0, 0]), dtype)
        epsq = Fraction(float(np.float32(eps)))
        for j in range(N):
            wq = exact.fraction_of_bits(int(bits_of(w, dtype)[j]), dtype)
            want = _closed_form_bits(wq * cq, cq * cq + epsq, dtype)
            assert int(got[0, j]) == want and int(got[1, j]) == want


@pytest.mark.parametrize("dtype", DTYPES)
def test_zero_row_gives_zero(dtype):
    x = storage(np.zeros((3, 40)), dtype)
    w = inputs.normal_matrix(3, 10, 1, 40, dtype, 1.0, 0.1)[0]
    y = oracle.rmsnorm_oracle(x, w, 1e-6, dtype)
    assert np.all(oracle.decode(y, dtype) == 0.0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_one_hot_row_closed_form(dtype):
    """x = a e_k  =>  y_k = w_k a / sqrt(a^2/N + eps), all other outputs zero."""
    N, eps = 48, 1e-6
    for k, a in ((0, 2.0), (17, -60000.0 if dtype == FP16 else -3.0e4), (47, 0.125)):
        z = np.zeros((1, N))
        z[0, k] = a
        x = storage(z, dtype)
        w = inputs.normal_matrix(3, 12, 1, N, dtype, 1.0, 0.1)[0]
        got = bits_of(oracle.rmsnorm_oracle(x, w, eps, dtype), dtype)[0]
        aq = Fraction(a)
        wq = exact.fraction_of_bits(int(bits_of(w, dtype)[k]), dtype)
        want = _closed_form_bits(wq * aq, aq * aq / N + Fraction(float(np.float32(eps))), dtype)
        assert int(got[k]) == want
        others = np.delete(oracle.decode(exact.from_int_bits(got, dtype), dtype), k)
        assert np.all(others == 0.0)
    # eps -> 0: |y_k| -> sqrt(N) |w_k|
    z = np.zeros((1, 64))
    z[0, 3] = -7.0
    y = oracle.decode(oracle.rmsnorm_oracle(storage(z, FP32), storage(np.ones(64), FP32), 0.0, FP32), FP32)
    assert y[0, 3] == -8.0


@pytest.mark.parametrize("dtype", DTYPES)
def test_plus_minus_one_row_closed_form(dtype):
    """x_j in {+1,-1}  =>  y_j = x_j w_j / sqrt(1 + eps)."""
    N, eps = 96, 1e-5
    s = np.where(inputs.uniform(4, 13, 0, N) < 0.5, -1.0, 1.0)
    x = storage(s[None, :], dtype)
    w = inputs.uniform_vector(4, 14, N, dtype, 0.5, 1.5)
    got = bits_of(oracle.rmsnorm_oracle(x, w, eps, dtype), dtype)[0]
    root = 1 + Fraction(float(np.float32(eps)))
    for j in range(N):
        wq = exact.fraction_of_bits(int(bits_of(w, dtype)[j]), dtype)
        assert int(got[j]) == _closed_form_bits(wq * int(s[j]), root, dtype)


def test_hand_worked_examples():
    with open(os.path.join(GOLDEN, "hand_examples.txt")) as f:
        lines = [ln for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(lines) == 4
    for ln in lines:
        xs, ys = ln.split("|")
        x = np.array([[float(t) for t in xs.split()]], dtype=np.float32)
        want = np.array([float(t) for t in ys.split()]).astype(np.float32)
        got = oracle.rmsnorm_oracle(x, np.ones(x.shape[1], dtype=np.float32), 0.0, FP32)[0]
        assert np.array_equal(got, want), (x, got, want)


# -------------------------------------------------------------------- invariants

def test_rstd_against_library_two_norm():
    """w == 1, eps == 0: y = x sqrt(N) / ||x||_2, so r = sqrt(N) / ||x||_2."""
    for dtype in DTYPES:
        c = inputs.random_case(21, 300 + 2 * dtype, 16, 1000, dtype, 0.0)
        r = oracle.rmsnorm_oracle_rstd(c["x"], 0.0, dtype)
        xd = inputs.storage_to_f64(c["x"], dtype)
        want = math.sqrt(1000) / np.linalg.norm(xd, axis=1)
        assert np.allclose(r, want, rtol=1e-13, atol=0)


def test_rstd_against_compensated_sum_and_eps_placement():
    c = inputs.random_case(22, 310, 8, 8192, BF16, 1e-5)
    r = oracle.rmsnorm_oracle_rstd(c["x"], 1e-5, BF16)
    xd = inputs.storage_to_f64(c["x"], BF16)
    eps = float(np.float32(1e-5))
    for i in range(8):
        ms = math.fsum(v * v for v in xd[i]) / 8192
        assert abs(r[i] * math.sqrt(ms + eps) - 1.0) < 1e-13
        # the two nearest wrong readings are far outside that band
        assert abs(r[i] * (math.sqrt(ms) + eps) - 1.0) > 1e-7
        assert abs(r[i] * math.sqrt(ms * 8192 / 8191 + eps) - 1.0) > 1e-6


def test_norm_invariant():
    """mean_j (y_j / w_j)^2 = ms / (ms + eps), checked on fp32 outputs."""
    eps = 1e-2
    c = inputs.random_case(23, 320, 32, 512, FP32, eps)
    y = oracle.rmsnorm_oracle(c["x"], c["w"], eps, FP32).astype(np.float64)
    xd = c["x"].astype(np.float64)
    wd = c["w"].astype(np.float64)
    ms = (xd * xd).mean(axis=1)
    lhs = ((y / wd) ** 2).mean(axis=1)
    assert np.allclose(lhs, ms / (ms + float(np.float32(eps))), rtol=1e-6)


@pytest.mark.parametrize("dtype", DTYPES)
def test_power_of_two_scale_invariance_is_bit_exact(dtype):
    """eps = 0: scaling x by 2^k scales ms by 4^k exactly, so the output bits do not move."""
    c = inputs.random_case(24, 330 + 2 * dtype, 6, 200, dtype, 0.0)
    y0 = oracle.rmsnorm_oracle(c["x"], c["w"], 0.0, dtype)
    for k in (-3, 4):
        xs = storage(inputs.storage_to_f64(c["x"], dtype) * 2.0 ** k, dtype)
        assert np.array_equal(inputs.storage_to_f64(xs, dtype),
                              inputs.storage_to_f64(c["x"], dtype) * 2.0 ** k)
        assert np.array_equal(oracle.rmsnorm_oracle(xs, c["w"], 0.0, dtype), y0)


def test_general_scale_invariance_as_eps_vanishes():
    c = inputs.random_case(25, 340, 4, 300, FP32, 0.0)
    x64 = c["x"].astype(np.float64)
    y0 = oracle.rmsnorm_oracle(c["x"], c["w"], 1e-12, FP32)
    y1 = oracle.rmsnorm_oracle((x64 * 1000.0).astype(np.float32), c["w"], 1e-12, FP32)
    assert compare.max_rel_err_fp32(y1, y0) < 1e-6


@pytest.mark.parametrize("dtype", DTYPES)
def test_symmetries(dtype):
    c = inputs.random_case(26, 350 + 2 * dtype, 9, 77, dtype, 1e-6)
    x, w = c["x"], c["w"]
    y = oracle.rmsnorm_oracle(x, w, 1e-6, dtype)
    # negation: y(-x) = -y(x), bit for bit (flip the sign bit)
    if dtype == FP32:
        yn = oracle.rmsnorm_oracle(-x, w, 1e-6, dtype)
        assert np.array_equal(yn.view(np.uint32), y.view(np.uint32) ^ np.uint32(0x80000000))
    else:
        yn = oracle.rmsnorm_oracle(x ^ np.uint16(0x8000), w, 1e-6, dtype)
        assert np.array_equal(yn, y ^ np.uint16(0x8000))
    # row permutation permutes the outputs exactly
    perm = np.argsort(inputs.uniform(1, 2, 0, 9))
    assert np.array_equal(oracle.rmsnorm_oracle(x[perm], w, 1e-6, dtype), y[perm])
    # row independence: each row alone gives the same bits; so does any thread count
    for i in (0, 4, 8):
        assert np.array_equal(oracle.rmsnorm_oracle(x[i:i + 1], w, 1e-6, dtype)[0], y[i])
    for nt in (1, 2, 3, 8):
        assert np.array_equal(oracle.rmsnorm_oracle(x, w, 1e-6, dtype, nthreads=nt), y)
    # column permutation of x and w together permutes the outputs (up to fp64 sum order)
    cp = np.argsort(inputs.uniform(1, 3, 0, 77))
    yc = oracle.rmsnorm_oracle(np.ascontiguousarray(x[:, cp]), w[cp], 1e-6, dtype)
    if dtype == FP32:
        assert compare.max_rel_err_fp32(yc, y[:, cp]) < 1e-6
    else:
        assert compare.ulp_distance(yc, y[:, cp], dtype).max() <= 1


def test_weight_is_indexed_by_column_not_row():
    """A transposed or row-indexed weight would break this: w = e_3 selects column 3."""
    N = 8
    c = inputs.random_case(27, 360, N, N, FP32, 1e-6)
    w = np.zeros(N, dtype=np.float32)
    w[3] = 2.0
    y = oracle.rmsnorm_oracle(c["x"], w, 1e-6, FP32)
    assert np.all(y[:, [0, 1, 2, 4, 5, 6, 7]] == 0.0)
    assert np.all(y[:, 3] != 0.0)
    x64 = c["x"].astype(np.float64)
    want = 2.0 * x64[:, 3] / np.sqrt((x64 * x64).mean(axis=1) + float(np.float32(1e-6)))
    assert np.array_equal(y[:, 3], want.astype(np.float32))


def test_single_rounding_differs_from_rounding_the_normalised_value_first():
    """The product x*r*w is rounded once; rounding x*r to bf16 before the multiply is a
    different (wrong, for this task) reading, and is visibly different on real data."""
    c = inputs.config2(M=4)
    y = oracle.rmsnorm_oracle(c["x"], c["w"], c["eps"], BF16)
    xd = inputs.storage_to_f64(c["x"], BF16)
    wd = inputs.storage_to_f64(c["w"], BF16)
    r = oracle.rmsnorm_oracle_rstd(c["x"], c["eps"], BF16)
    once = oracle.encode(xd * r[:, None] * wd, BF16)
    twice = oracle.encode(oracle.decode(oracle.encode(xd * r[:, None], BF16), BF16) * wd, BF16)
    assert np.array_equal(y, once)
    assert np.count_nonzero(twice != once) > 100


# ---------------------------------------------------------------- argument checks

def test_oracle_rejects_bad_arguments():
    x = np.zeros((2, 4), dtype=np.float32)
    w = np.ones(4, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.rmsnorm_oracle(x, w, -1.0, FP32)
    with pytest.raises(ValueError):
        oracle.rmsnorm_oracle(x, w, float("nan"), FP32)
    with pytest.raises(ValueError):
        oracle.rmsnorm_oracle(x, np.ones(5, dtype=np.float32), 1e-6, FP32)
    with pytest.raises(TypeError):
        oracle.rmsnorm_oracle(x, w, 1e-6, BF16)
    assert oracle.rmsnorm_oracle(np.zeros((0, 4), dtype=np.float32), w, 1e-6, FP32).shape == (0, 4)


# ------------------------------------------------------------ measurement model

def test_bytes_model_reproduces_the_papers_throughput_column():
    with open(os.path.join(GOLDEN, "paper_rmsnorm_throughput.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for M, N, us, gbps in rows:
        M, N, us, gbps = int(M), int(N), float(us), float(gbps)
        mine = inputs.algorithmic_bytes(M, N, inputs.FP16) / (us * 1e-6) / 1e9
        # the table rounds the time to 0.1 us and the rate to 1 GB/s
        assert abs(mine - gbps) / gbps < 2e-3, (M, N, mine, gbps)
    assert inputs.algorithmic_bytes(16384, 8192, inputs.BF16) == 536887296


# ----------------------------------------------------------- comparator sanity

def test_ulp_comparator():
    a = np.array([0x3F80, 0x3F80, 0x0000, 0x8000, 0x0001, 0x7F7F], dtype=np.uint16)
    b = np.array([0x3F81, 0x3F7F, 0x8000, 0x0001, 0x8001, 0x7F80], dtype=np.uint16)
    assert list(compare.ulp_distance(a, b, BF16)) == [1, 1, 0, 1, 2, 1]
    with pytest.raises(AssertionError):
        compare.ulp_distance(np.array([0x7FC0], dtype=np.uint16), np.array([0x3F80], dtype=np.uint16), BF16)
    with pytest.raises(AssertionError):
        compare.check_parity(np.array([0x3F82], dtype=np.uint16), np.array([0x3F80], dtype=np.uint16), BF16)
    with pytest.raises(AssertionError):
        compare.check_parity(np.array([1.0 + 2e-5], dtype=np.float32), np.array([1.0], dtype=np.float32), FP32)
    compare.check_parity(np.array([1.0 + 5e-6, -0.0], dtype=np.float32), np.array([1.0, 0.0], dtype=np.float32), FP32)
