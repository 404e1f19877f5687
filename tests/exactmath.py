"""Exact-arithmetic helpers for the tests: correct rounding of a rational to a
binary floating-point format, and ulp distances.  Independent of both the
oracle and the HIP path."""
from fractions import Fraction

import numpy as np

FORMATS = {
    # name: (precision bits incl. hidden bit, emin of normals, emax)
    "f32": (24, -126, 127),
    "bf16": (8, -126, 127),
}


def round_fraction(x: Fraction, fmt: str):
    """Round the rational x to the nearest value of `fmt` (ties to even).
    Returns (sign, m, q) with value = (-1)^sign * m * 2^q, m < 2^p, or 'inf'."""
    p, emin, emax = FORMATS[fmt]
    sign = 1 if x < 0 else 0
    ax = -x if x < 0 else x
    if ax == 0:
        return (sign, 0, emin - (p - 1))
    # exponent of leading bit: 2^e <= ax < 2^(e+1)
    e = ax.numerator.bit_length() - ax.denominator.bit_length()
    if Fraction(2) ** e > ax:
        e -= 1
    if Fraction(2) ** (e + 1) <= ax:
        e += 1
    e = max(e, emin)
    q = e - (p - 1)                       # exponent of the last kept bit
    scaled = ax / (Fraction(2) ** q)      # exact
    m = scaled.numerator // scaled.denominator
    rem = scaled - m
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (m & 1)):
        m += 1
    if m == (1 << p):
        m >>= 1
        q += 1
    if q + (p - 1) > emax:
        return (sign, "inf", 0)
    return (sign, m, q)


def fraction_to_f32_bits(x: Fraction) -> int:
    sign, m, q = round_fraction(x, "f32")
    if m == "inf":
        return (sign << 31) | 0x7F800000
    if m == 0:
        return sign << 31
    if m < (1 << 23):                      # subnormal
        return (sign << 31) | m
    return (sign << 31) | ((q + 23 + 127) << 23) | (m - (1 << 23))


def fraction_to_bf16_bits(x: Fraction) -> int:
    sign, m, q = round_fraction(x, "bf16")
    if m == "inf":
        return (sign << 15) | 0x7F80
    if m == 0:
        return sign << 15
    if m < (1 << 7):
        return (sign << 15) | m
    return (sign << 15) | ((q + 7 + 127) << 7) | (m - (1 << 7))


def f32_from_bits(b):
    return np.array(b, dtype=np.uint32).view(np.float32)


def bf16_bits_to_fraction(h: int) -> Fraction:
    f = np.array([int(h) << 16], dtype=np.uint32).view(np.float32)[0]
    return Fraction(float(f))


def ordered_f32(a: np.ndarray) -> np.ndarray:
    """Map fp32 bit patterns to integers that are monotone in the value
    (+0 and -0 coincide)."""
    u = np.ascontiguousarray(a).view(np.uint32).astype(np.int64)
    return np.where(u & 0x80000000, -(u & 0x7FFFFFFF), u)


def ordered_bf16(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a).view(np.uint16).astype(np.int64)
    return np.where(u & 0x8000, -(u & 0x7FFF), u)


def ulp_distance(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Element-wise distance in units in the last place.  float32 arrays are
    fp32; uint16 arrays are bf16 bit patterns.  NaN matches only NaN (distance
    0), else a huge distance."""
    assert x.dtype == y.dtype and x.shape == y.shape
    if x.dtype == np.float32:
        ox, oy = ordered_f32(x), ordered_f32(y)
        nx, ny = np.isnan(x), np.isnan(y)
    elif x.dtype == np.uint16:
        ox, oy = ordered_bf16(x), ordered_bf16(y)
        nx = ((x & 0x7F80) == 0x7F80) & ((x & 0x7F) != 0)
        ny = ((y & 0x7F80) == 0x7F80) & ((y & 0x7F) != 0)
    else:
        raise TypeError(x.dtype)
    d = np.abs(ox - oy)
    d = np.where(nx & ny, 0, d)
    d = np.where(nx ^ ny, np.int64(1) << 40, d)
    return d
