"""Comparators for GPU-vs-oracle parity (numpy only; no method arithmetic).

fp32: relative error against the oracle value, with exact zeros required where
the oracle is zero.  fp16 / bf16: distance in units in the last place, measured
on the bit patterns after mapping them to a monotone integer line on which +0
and -0 coincide.
"""
from __future__ import annotations

import numpy as np

FLT_MIN = float(np.finfo(np.float32).tiny)


def ordinal16(bits: np.ndarray) -> np.ndarray:
    """Sign-magnitude 16-bit patterns -> monotone signed integers (+0 == -0 == 0)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


def _nan_mask16(bits: np.ndarray, dtype: int) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16)
    if dtype == 1:   # fp16: exponent 0x7C00, mantissa 0x03FF
        return ((b & 0x7C00) == 0x7C00) & ((b & 0x03FF) != 0)
    return ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)


def ulp_distance(got: np.ndarray, want: np.ndarray, dtype: int) -> np.ndarray:
    """Elementwise ulp distance for 16-bit storage; NaNs must sit in the same places."""
    gn, wn = _nan_mask16(got, dtype), _nan_mask16(want, dtype)
    if not np.array_equal(gn, wn):
        raise AssertionError("NaN positions differ between result and oracle")
    d = np.abs(ordinal16(got) - ordinal16(want))
    d[gn] = 0
    return d


def max_rel_err_fp32(got: np.ndarray, want: np.ndarray) -> float:
    g = np.asarray(got, dtype=np.float32).astype(np.float64)
    o = np.asarray(want, dtype=np.float32).astype(np.float64)
    gn, on = np.isnan(g), np.isnan(o)
    if not np.array_equal(gn, on):
        raise AssertionError("NaN positions differ between result and oracle")
    zero = (o == 0.0) & ~on
    if np.any(g[zero] != 0.0):
        raise AssertionError("result is non-zero where the oracle is exactly zero")
    ok = ~on & ~zero
    if not ok.any():
        return 0.0
    return float(np.max(np.abs(g[ok] - o[ok]) / np.maximum(np.abs(o[ok]), FLT_MIN)))


# Tolerances of the benchmark spec: fp32 max rel err <= 1e-5; bf16 <= 1 ulp
# after rounding; fp16 <= 2 ulp.
TOL_FP32_REL = 1e-5
TOL_ULP = {1: 2, 2: 1}


def check_parity(got: np.ndarray, want: np.ndarray, dtype: int, what: str = "") -> dict:
    """Asserts the stated tolerance; returns the measured error statistics."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if dtype == 0:
        err = max_rel_err_fp32(got, want)
        assert err <= TOL_FP32_REL, f"{what}: fp32 max rel err {err:.3e} > {TOL_FP32_REL}"
        return {"max_rel_err": err}
    d = ulp_distance(got, want, dtype)
    worst = int(d.max()) if d.size else 0
    frac = float(np.count_nonzero(d)) / max(d.size, 1)
    assert worst <= TOL_ULP[dtype], (
        f"{what}: max ulp distance {worst} > {TOL_ULP[dtype]} "
        f"(first at flat index {int(np.argmax(d))})")
    return {"max_ulp": worst, "frac_off": frac}


# ---- row softmax ---------------------------------------------------------------------------
# Tolerances: bf16 <= 1 ulp, fp16 <= 2 ulp against the oracle after its
# single rounding; fp32 |g - o| <= 1e-5 |o| + 2 subnormal quanta (outputs below FLT_MIN have
# fewer than 24 significant bits, so a purely relative bound cannot hold there).
SOFTMAX_FP32_ABS_FLOOR = 2.0 * 2.0 ** -149


def check_softmax_parity(got: np.ndarray, want: np.ndarray, dtype: int, what: str = "") -> dict:
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if dtype == 0:
        g = got.astype(np.float64)
        o = want.astype(np.float64)
        gn, on = np.isnan(g), np.isnan(o)
        assert np.array_equal(gn, on), f"{what}: NaN positions differ"
        ok = ~on
        if not ok.any():
            return {"max_rel_err": 0.0}
        excess = np.abs(g[ok] - o[ok]) - SOFTMAX_FP32_ABS_FLOOR
        rel = np.maximum(excess, 0.0) / np.maximum(np.abs(o[ok]), FLT_MIN)
        err = float(rel.max())
        assert err <= TOL_FP32_REL, f"{what}: fp32 max rel err {err:.3e} > {TOL_FP32_REL}"
        return {"max_rel_err": err}
    d = ulp_distance(got, want, dtype)
    worst = int(d.max()) if d.size else 0
    assert worst <= TOL_ULP[dtype], (
        f"{what}: max ulp distance {worst} > {TOL_ULP[dtype]} (first at flat index {int(np.argmax(d))})")
    return {"max_ulp": worst, "frac_off": float(np.count_nonzero(d)) / max(d.size, 1)}


# ---- LayerNorm -----------------------------------------------------------------------------
# LayerNorm subtracts (the mean from x, possibly the bias against the scaled value), so any
# fp32 implementation carries an ABSOLUTE error of a few fp32 ulps of the row's scale, which
# is not small relative to an output that happens to land near zero.  An element passes if
# it meets the relative bound of the other kernels (fp32 1e-5; bf16 1 ulp; fp16 2 ulp against
# the oracle after its rounding) OR lies within 2^-20 of the element's scale
# |w_j| * max_j |z_i| + |b_j|, where z_i is the normalised row (from the oracle's fp64 mean
# and rstd).
LAYERNORM_ABS = 2.0 ** -20


def check_layernorm_parity(got, want, scale, dtype: int, what: str = "") -> dict:
    """scale: (M, N) fp64 array of |w_j| * max|z_i| + |b_j| (see layernorm_scale)."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if dtype == 0:
        g = got.astype(np.float64)
        o = want.astype(np.float64)
        assert np.array_equal(np.isnan(g), np.isnan(o)), f"{what}: NaN positions differ"
        ok = ~np.isnan(o)
        diff = np.abs(g - o)
        rel_ok = diff <= TOL_FP32_REL * np.abs(o)
        abs_ok = diff <= LAYERNORM_ABS * scale
        bad = ok & ~(rel_ok | abs_ok)
        assert not bad.any(), (f"{what}: {int(bad.sum())} fp32 elements outside both bounds; first at "
                               f"{tuple(np.argwhere(bad)[0])}: got {g[bad][0]!r} want {o[bad][0]!r}")
        worst = float((diff / np.maximum(scale, FLT_MIN))[ok].max()) if ok.any() else 0.0
        return {"max_err_over_scale": worst, "frac_abs_only": float((ok & ~rel_ok).mean())}
    from_bits = _f64_from_16
    d = ulp_distance(got, want, dtype)
    ulp_ok = d <= TOL_ULP[dtype]
    diff = np.abs(from_bits(got, dtype) - from_bits(want, dtype))
    with np.errstate(invalid="ignore"):
        abs_ok = diff <= LAYERNORM_ABS * scale
    bad = ~(ulp_ok | abs_ok)
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements outside both bounds; first at "
                           f"{tuple(np.argwhere(bad)[0])}, ulp distance {int(d[bad][0])}")
    return {"max_ulp_where_relative": int(d[ulp_ok].max()) if ulp_ok.any() else 0,
            "frac_off": float(np.count_nonzero(d)) / max(d.size, 1),
            "frac_abs_only": float((~ulp_ok).mean())}


def _f64_from_16(bits, dtype: int) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16)
    if dtype == 1:
        return b.view(np.float16).astype(np.float64)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def layernorm_scale(x_f64, w_f64, b_f64, mean, rstd) -> np.ndarray:
    zmax = (np.abs(x_f64 - mean[:, None]) * rstd[:, None]).max(axis=1)
    s = np.abs(w_f64)[None, :] * zmax[:, None]
    if b_f64 is not None:
        s = s + np.abs(b_f64)[None, :]
    return s


# ---- row cross-entropy ---------------------------------------------------------------------
# loss = log(s) - (x_t - m) in fp32.  The sum s >= 1 is an fp32 sum of N rounded exponentials
# (chains of at most ~100 additions per thread plus the fixed reduction tree, each rounding
# 2^-24 of s), so log(s), and with it the loss, carries an ABSOLUTE error of up to ~100 * 2^-24
# in the worst case (a few 1e-7 in practice) whatever the size of the loss; d_t = x_t - m and
# the final subtraction add 2^-24 relative each.  Bound: 1e-5 relative (the fp32 tolerance of
# the other kernels) plus 2^-17 absolute.  NaN and infinite results must agree exactly, and an
# ignored row must be exactly 0.
CROSSENTROPY_ABS = 2.0 ** -17


def check_crossentropy_parity(got, want, what: str = "", exact_zero=None) -> dict:
    """got: fp32 from the GPU; want: the oracle's values (fp32 losses or fp64 log-sum-exps).
    exact_zero: optional boolean mask of rows whose result must be exactly 0."""
    g = np.asarray(got).astype(np.float64)
    o = np.asarray(want).astype(np.float64)
    assert g.shape == o.shape, f"{what}: shape {g.shape} vs {o.shape}"
    assert np.array_equal(np.isnan(g), np.isnan(o)), f"{what}: NaN positions differ"
    inf = np.isinf(o)
    assert np.array_equal(g[inf], o[inf]) and not np.isinf(g[~inf & ~np.isnan(o)]).any(), \
        f"{what}: infinities differ"
    if exact_zero is not None:
        assert np.all(g[exact_zero] == 0.0), f"{what}: an ignored row is not exactly 0"
    ok = np.isfinite(o)
    if not ok.any():
        return {"max_abs_err": 0.0, "max_excess_rel": 0.0}
    diff = np.abs(g[ok] - o[ok])
    bound = TOL_FP32_REL * np.abs(o[ok]) + CROSSENTROPY_ABS
    worst = int(np.argmax(diff - bound))
    assert np.all(diff <= bound), (f"{what}: |{g[ok][worst]!r} - {o[ok][worst]!r}| = {diff[worst]:.3e} "
                                   f"> {bound[worst]:.3e}")
    return {"max_abs_err": float(diff.max()),
            "max_rel_err": float((diff / np.maximum(np.abs(o[ok]), 1.0)).max())}


# ---- row sum ---------------------------------------------------------------------------------
# An fp32 sum has no relative accuracy of its own: when the terms cancel, the result is small
# and the rounding errors are not.  Each addition rounds by at most 2^-24 of the partial sum it
# forms, which is at most the sum of magnitudes A = sum_j |x_j| of the row, and an element
# passes through at most D additions on its way to the result, so |g - exact| <= D * 2^-24 * A
# whatever the order.  The kernel's D: a thread's chain (at most N / 256 terms: 64 threads, 4
# lanes of an fp32 vector, is the coarsest split it ever uses), the fold of the chains, six
# levels across the wavefront and up to 16 wavefront partials in turn, together below
# N / 256 + 32.  The relative term covers the oracle's own rounding of its result to fp32.
ROWSUM_DEPTH_BASE = 32
ROWSUM_TERMS_PER_CHAIN = 256


def check_rowsum_parity(got, want, abs_sum, N: int, what: str = "") -> dict:
    """got: fp32 sums from the GPU; want: the oracle's fp32 sums; abs_sum: the oracle's fp64
    sums of magnitudes; N: row length."""
    g = np.asarray(got).astype(np.float64)
    o = np.asarray(want).astype(np.float64)
    a = np.asarray(abs_sum, dtype=np.float64)
    assert g.shape == o.shape == a.shape, f"{what}: shapes {g.shape} {o.shape} {a.shape}"
    assert np.array_equal(np.isnan(g), np.isnan(o)), f"{what}: NaN positions differ"
    inf = np.isinf(o)
    assert np.array_equal(g[inf], o[inf]) and not np.isinf(g[~inf & ~np.isnan(o)]).any(), \
        f"{what}: infinities differ"
    ok = np.isfinite(o)
    if not ok.any():
        return {"max_err_over_abs_sum": 0.0, "max_abs_err": 0.0}
    depth = ROWSUM_DEPTH_BASE + N / ROWSUM_TERMS_PER_CHAIN
    diff = np.abs(g[ok] - o[ok])
    bound = TOL_FP32_REL * np.abs(o[ok]) + depth * 2.0 ** -24 * a[ok]
    worst = int(np.argmax(diff - bound))
    assert np.all(diff <= bound), (f"{what}: |{g[ok][worst]!r} - {o[ok][worst]!r}| = {diff[worst]:.3e} "
                                   f"> {bound[worst]:.3e}")
    return {"max_err_over_abs_sum": float((diff / np.maximum(a[ok], FLT_MIN)).max()),
            "max_abs_err": float(diff.max())}
