"""Exact-arithmetic helpers for pinning the oracle.

Nothing here is shared with the oracle or with the GPU library: IEEE
binary32 rounding is re-derived from rationals (fractions.Fraction), so a
value computed here is "what the mathematics says", not "what some float
unit returned".
"""
from fractions import Fraction
import math

import numpy as np

_F32_MIN_EXP = -126      # exponent of the smallest normal
_F32_MANT = 23


def fraction_to_f32(fr: Fraction) -> np.float32:
    """Round a rational to the nearest binary32, ties to even (finite range)."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, _F32_MIN_EXP)                      # subnormals share the lowest exponent
    ulp = Fraction(2) ** (e - _F32_MANT)
    n = round(a / ulp)                            # Fraction.__round__: ties to even
    val = n * ulp
    if val >= Fraction(2) ** 128:
        raise OverflowError("beyond binary32 range")
    out = np.float32(float(val))                  # val is exactly representable
    assert Fraction(float(out)) == val
    return np.float32(sign) * out


def f32_fraction(x) -> Fraction:
    return Fraction(float(np.float32(x)))


def rint_half_even_f64(t: np.ndarray) -> np.ndarray:
    """Nearest integer, ties to even, written without rint/round library calls."""
    t = np.asarray(t, np.float64)
    f = np.floor(t)
    d = t - f                                     # exact for |t| < 2^52
    up = (d > 0.5) | ((d == 0.5) & (np.mod(f, 2.0) == 1.0))
    return f + up


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> exact values, from the format's definition (no casts)."""
    bits = np.asarray(bits, np.uint16).astype(np.int64)
    sign = np.where(bits >> 15, -1.0, 1.0)
    exp = (bits >> 7) & 0xFF
    man = bits & 0x7F
    normal = np.ldexp(1.0 + man / 128.0, exp - 127)
    sub = np.ldexp(man / 128.0, -126)
    val = np.where(exp == 0, sub, normal)
    val = np.where(exp == 255, np.nan, val)
    return sign * val


def all_finite_bf16_bits() -> np.ndarray:
    b = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    exp = (b >> 7) & 0xFF
    return b[exp != 255]


def bf16_rne_from_fraction(fr: Fraction) -> int:
    """Round a rational to bf16 (8 significant bits), ties to even; returns the bit pattern."""
    if fr == 0:
        return 0
    sign = 0x8000 if fr < 0 else 0
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)
    ulp = Fraction(2) ** (e - 7)
    n = round(a / ulp)
    if e == -126 and n < 128:                      # subnormal
        return sign | int(n)
    if n == 256:                                   # carried into the next binade
        n, e = 128, e + 1
    return sign | ((e + 127) << 7) | (int(n) - 128)


def unpack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Bytes -> signed 4-bit values, even element from the low nibble."""
    c = np.asarray(codes, np.uint8).astype(np.int16)
    lo = c & 0xF
    hi = (c >> 4) & 0xF
    out = np.empty(c.size * 2, np.int16)
    out[0::2] = lo
    out[1::2] = hi
    return np.where(out >= 8, out - 16, out).astype(np.int32)


def unpack_codes(codes: np.ndarray, numel: int, bits: int) -> np.ndarray:
    """Code bytes -> signed integers, from the stated layout: int8 for 8 bits; nibbles for 4;
    for 5 and 6 bits a nibble plane (numel/2 bytes) followed by the plane of high bits."""
    c = np.asarray(codes, np.uint8)
    if bits == 8:
        return c.view(np.int8).astype(np.int32)
    lo = np.empty(numel, np.int32)
    lo[0::2] = c[: numel // 2] & 0xF
    lo[1::2] = c[: numel // 2] >> 4
    if bits == 4:
        field = lo
    elif bits == 5:
        hb = c[numel // 2: numel // 2 + numel // 8]
        hi = ((hb[:, None] >> np.arange(8)) & 1).reshape(-1).astype(np.int32)
        field = lo | (hi << 4)
    elif bits == 6:
        hb = c[numel // 2: numel // 2 + numel // 4]
        hi = ((hb[:, None] >> (2 * np.arange(4))) & 3).reshape(-1).astype(np.int32)
        field = lo | (hi << 4)
    else:
        raise ValueError(bits)
    return np.where(field >= (1 << (bits - 1)), field - (1 << bits), field).astype(np.int32)


def pack_codes(q: np.ndarray, bits: int) -> np.ndarray:
    """Signed integers -> code bytes (inverse of unpack_codes), for building dequantize inputs."""
    q = np.asarray(q, np.int64).reshape(-1)
    n = q.size
    u = (q & ((1 << bits) - 1)).astype(np.uint8)
    if bits == 8:
        return u
    lo = u & 0xF
    nib = (lo[0::2] | (lo[1::2] << 4)).astype(np.uint8)
    if bits == 4:
        return nib
    hi = (u >> 4).astype(np.uint8)
    if bits == 5:
        high = (hi.reshape(-1, 8) << np.arange(8, dtype=np.uint8)).sum(axis=1).astype(np.uint8)
    else:
        high = (hi.reshape(-1, 4) << (2 * np.arange(4, dtype=np.uint8))).sum(axis=1).astype(np.uint8)
    return np.concatenate([nib, high])
