"""Storage-type conversions for the CPU oracle.

TEST INFRASTRUCTURE ONLY (see `oracle.access_pattern`).  The paper computes
over reals (its notation uses f64, Sec. 3.1); the GPU library stores int8,
int32, bfloat16 and float32, and 8-bit floats (OCP e4m3) as contraction operands.  These helpers convert between those storage
types and the int64 / float64 values the interpreter works on.  bfloat16 is
the upper 16 bits of an IEEE-754 binary32; conversion to it rounds to nearest,
ties to even.  Integers never saturate: a result outside int32 is an error.
"""

from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> the exact values as float64."""
    b = np.asarray(bits).astype(np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even (NaN stays NaN)."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(f)
    rounded = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), rounded)
    return rounded.astype(np.uint16)


def e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint8 OCP e4m3 bit patterns -> exact float64 values.

    Format (OCP 8-bit floating point specification, E4M3): sign, 4 exponent bits with bias 7,
    3 mantissa bits; exponent 0 holds the subnormals m/8 * 2^-6; there is no infinity, and only
    exponent 15 with mantissa 7 is NaN, so the largest finite value is 1.75 * 2^8 = 448."""
    b = np.asarray(bits).astype(np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = (b & 0x7).astype(np.float64)
    normal = np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64))
    subnormal = np.ldexp(m / 8.0, -6)
    v = sign * np.where(e == 0, subnormal, normal)
    return np.where((e == 15) & ((b & 0x7) == 7), np.nan, v)


def round_to_f32(x: np.ndarray) -> np.ndarray:
    """float64 -> float32 with a single rounding (nearest even)."""
    return np.asarray(x, dtype=np.float64).astype(np.float32)


def round_to_bf16_value(x: np.ndarray) -> np.ndarray:
    """float64 -> float32 -> bfloat16, returned as the float64 value of the bfloat16."""
    return bf16_bits_to_f64(f32_to_bf16_bits(round_to_f32(x)))


def to_i32_checked(x: np.ndarray) -> np.ndarray:
    """int64 -> int32, refusing values that do not fit (no saturation anywhere)."""
    x = np.asarray(x)
    if not np.issubdtype(x.dtype, np.integer):
        raise TypeError("integer result expected")
    if x.size and (x.max() > np.iinfo(np.int32).max or x.min() < np.iinfo(np.int32).min):
        raise OverflowError("result does not fit int32")
    return x.astype(np.int32)

