"""Exact decoders for the 16-bit and 8-bit input formats, and the output rounding.

Test infrastructure only (see the package docstring).

The paper fixes the element type of every GEMM to BF16 with an FP32
accumulator (section 4, experimental setup).  BF16 is the upper half of an
IEEE-754 binary32: 1 sign, 8 exponent (bias 127) and 7 fraction bits.  The
8-bit extension uses OCP FP8 E4M3 ("fn": finite + NaN only): 1 sign, 4 exponent
(bias 7), 3 fraction bits, no infinities, NaN only at S.1111.111, max 448.

Readings taken where the paper is silent:
  * output rounding fp -> bf16 is round-to-nearest, ties-to-even, NaN kept,
    subnormals not flushed; the oracle rounds its float64 result once.
"""
import numpy as np


def _bf16_decode_formula(bits):
    """uint16 bit patterns -> float64 values, exactly.

    value = (-1)^s * 2^(e-127) * (1 + f/128)   for 0 < e < 255
          = (-1)^s * 2^(-126) * (f/128)        for e == 0
          = inf / nan                          for e == 255
    """
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    s = (b >> 15) & 1
    e = (b >> 7) & 0xFF
    f = b & 0x7F
    sign = np.where(s == 1, -1.0, 1.0)
    normal = np.ldexp(1.0 + f / 128.0, (e - 127).astype(np.int64))
    sub = np.ldexp(f / 128.0, -126)
    special = np.where(f == 0, np.inf, np.nan)
    mag = np.where(e == 0, sub, np.where(e == 255, special, normal))
    return sign * mag


_BF16 = _bf16_decode_formula(np.arange(65536, dtype=np.uint32).astype(np.uint16))


def bf16_decode(bits):
    """uint16 bit patterns -> float64 values, exactly (the formula above, tabulated for all 65536 patterns)."""
    return _BF16[np.asarray(bits, dtype=np.uint16)]


def bf16_round(x):
    """float64 -> nearest bf16-representable float64 (ties to even), one rounding.

    bf16 carries 8 significant bits, so a value with binary exponent E
    (x = f * 2^E, 0.5 <= |f| < 1) is rounded to a multiple of 2^(E-8); below
    the smallest normal (2^-126) the grid spacing stays at 2^-133.  Magnitudes
    that round to 2^128 or more become infinity.
    """
    x = np.asarray(x, dtype=np.float64)
    _, E = np.frexp(x)
    quantum = np.maximum(E.astype(np.int64) - 8, -133)
    finite = np.isfinite(x)
    xs = np.where(finite, x, 0.0)
    q = np.rint(np.ldexp(xs, -quantum))           # np.rint rounds half to even
    y = np.ldexp(q, quantum)
    y = np.where(np.abs(y) >= 2.0 ** 128, np.copysign(np.inf, xs), y)
    return np.where(finite, y, x)


def bf16_encode(x):
    """float64 -> uint16 bf16 bit patterns (round-to-nearest-even)."""
    y = bf16_round(x).astype(np.float32)          # exact: bf16 values are binary32 values
    return (y.view(np.uint32) >> 16).astype(np.uint16)


def e4m3_table():
    """All 256 OCP E4M3 (finite+NaN) values as float64, indexed by the byte."""
    t = np.empty(256, dtype=np.float64)
    for b in range(256):
        s, e, m = b >> 7, (b >> 3) & 0xF, b & 7
        if e == 15 and m == 7:
            v = float("nan")
        elif e == 0:
            v = (m / 8.0) * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[b] = -v if s else v
    return t


_E4M3 = e4m3_table()


def e4m3_decode(bits):
    """uint8 bit patterns -> float64 values, exactly."""
    return _E4M3[np.asarray(bits, dtype=np.uint8)]


def decode(bits, dtype):
    """Decode an input operand: dtype is "bf16" (uint16 bits) or "fp8" (uint8 bits)."""
    if dtype == "bf16":
        return bf16_decode(bits)
    if dtype == "fp8":
        return e4m3_decode(bits)
    raise ValueError(f"unknown dtype {dtype!r}")
