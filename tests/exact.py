"""Exact-arithmetic helpers for pinning the oracle (pure Python, no oracle code).

Values are `fractions.Fraction`s; the only irrational step, the square root, is
taken with 300 fractional bits through math.isqrt, which is more than 10^80
times finer than any rounding boundary these tests can meet.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

# (significand bits incl. hidden bit, min normal exponent, max exponent, exponent field bits)
FORMATS = {0: (24, -126, 127, 8), 1: (11, -14, 15, 5), 2: (8, -126, 127, 8)}

SQRT_BITS = 300


def fraction_of_bits(bits: int, dtype: int) -> Fraction:
    """Exact value of a finite bit pattern."""
    p, emin, emax, ebits = FORMATS[dtype]
    mbits = p - 1
    mant = bits & ((1 << mbits) - 1)
    expo = (bits >> mbits) & ((1 << ebits) - 1)
    sign = -1 if (bits >> (mbits + ebits)) & 1 else 1
    assert expo != (1 << ebits) - 1, "not finite"
    if expo == 0:
        return sign * Fraction(mant) * Fraction(2) ** (emin - mbits)
    return sign * Fraction(mant + (1 << mbits)) * Fraction(2) ** (expo - emax - mbits)


def sqrt_fraction(v: Fraction) -> Fraction:
    """floor(sqrt(v) * 2^SQRT_BITS) / 2^SQRT_BITS for v >= 0."""
    n, d = v.numerator, v.denominator
    return Fraction(math.isqrt((n * d) << (2 * SQRT_BITS)), d << SQRT_BITS)


def round_to_bits(v: Fraction, dtype: int) -> int:
    """Bit pattern of v rounded to nearest, ties to even; overflow gives infinity."""
    p, emin, emax, ebits = FORMATS[dtype]
    mbits = p - 1
    sign = (1 << (mbits + ebits)) if v < 0 else 0
    a = abs(v)
    if a == 0:
        return sign
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, emin)
    ulp = Fraction(2) ** (e - mbits)
    q, rem = divmod(a, ulp)
    q = int(q)
    if rem * 2 > ulp or (rem * 2 == ulp and q % 2 == 1):
        q += 1
    if q == (1 << p):          # rounded up into the next binade
        q >>= 1
        e += 1
    if e > emax:
        return sign | (((1 << ebits) - 1) << mbits)
    if q < (1 << mbits):       # subnormal (only possible when e == emin)
        return sign | q
    return sign | ((e + emax) << mbits) | (q - (1 << mbits))


def to_int_bits(a: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array (float32 or uint16 patterns) -> python-int-friendly uint32 patterns."""
    a = np.asarray(a)
    if dtype == 0:
        return a.astype(np.float32).view(np.uint32)
    return a.astype(np.uint16).astype(np.uint32)


def from_int_bits(bits, dtype: int) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint32)
    if dtype == 0:
        return b.view(np.float32)
    return b.astype(np.uint16)


def rmsnorm_exact_bits(x_bits, w_bits, eps_float32: float, dtype: int):
    """RMSNorm of one or more rows in exact arithmetic, one final rounding.

    x_bits: (M, N) integer bit patterns, w_bits: (N,).  eps is the float the GPU
    call would receive, taken at its exact binary value.
    """
    eps = Fraction(float(np.float32(eps_float32)))
    x_bits = np.asarray(x_bits)
    M, N = x_bits.shape
    W = [fraction_of_bits(int(b), dtype) for b in w_bits]
    out = np.zeros((M, N), dtype=np.uint32)
    for i in range(M):
        X = [fraction_of_bits(int(b), dtype) for b in x_bits[i]]
        ms = sum(v * v for v in X) / N
        root = sqrt_fraction(ms + eps)
        for j in range(N):
            out[i, j] = round_to_bits(X[j] * W[j] / root, dtype)
    return out
