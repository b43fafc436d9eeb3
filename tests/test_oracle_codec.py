"""Pins for the oracle's number formats: closed forms written with Python's exact
arithmetic, anchor values of the formats, and the library's converters."""
import struct
from fractions import Fraction

import numpy as np
import torch

from oracle import codec


def _bf16_exact(b):
    """bf16 pattern -> Fraction (or None for inf/nan), straight from the format definition."""
    s, e, f = b >> 15, (b >> 7) & 0xFF, b & 0x7F
    if e == 255:
        return None
    if e == 0:
        v = Fraction(f, 128) * Fraction(1, 2 ** 126)
    else:
        v = (1 + Fraction(f, 128)) * (Fraction(2) ** (e - 127))
    return -v if s else v


def test_bf16_decode_all_patterns_against_format_definition():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    dec = codec.bf16_decode(bits)
    for b in range(0, 65536, 7):          # every 7th pattern exactly (covers all exponents)
        ex = _bf16_exact(b)
        if ex is None:
            assert not np.isfinite(dec[b])
        else:
            assert Fraction(float(dec[b])) == ex, hex(b)
    # and all of them against binary32 reinterpretation (bf16 = top half of a float32)
    for b in range(65536):
        f32 = struct.unpack("<f", struct.pack("<I", b << 16))[0]
        if f32 != f32:
            assert dec[b] != dec[b]
        else:
            assert dec[b] == f32, hex(b)


def test_bf16_decode_matches_library():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    lib = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    dec = codec.bf16_decode(bits)
    nan = np.isnan(lib)
    assert np.array_equal(np.isnan(dec), nan)
    assert np.array_equal(dec[~nan], lib[~nan])
    assert np.array_equal(np.signbit(dec[~nan]), np.signbit(lib[~nan]))


def test_bf16_anchors():
    assert codec.bf16_decode(np.uint16(0x3F80)) == 1.0
    assert codec.bf16_decode(np.uint16(0xC000)) == -2.0
    assert codec.bf16_decode(np.uint16(0x0080)) == 2.0 ** -126
    assert codec.bf16_decode(np.uint16(0x0001)) == 2.0 ** -133
    assert codec.bf16_decode(np.uint16(0x7F7F)) == (2 - 2.0 ** -7) * 2.0 ** 127
    assert np.isinf(codec.bf16_decode(np.uint16(0x7F80)))


def test_bf16_encode_roundtrip_and_ties():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    dec = codec.bf16_decode(bits)
    ok = ~np.isnan(dec)
    assert np.array_equal(codec.bf16_encode(dec[ok]), bits[ok])
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 0x3F80 and 0x3F81
    assert codec.bf16_encode(np.float64(1 + 2.0 ** -8)) == 0x3F80
    assert codec.bf16_encode(np.float64(1 + 3 * 2.0 ** -8)) == 0x3F82
    assert codec.bf16_encode(np.float64(1 + 2.0 ** -8 + 2.0 ** -40)) == 0x3F81   # just above the tie
    assert codec.bf16_encode(np.float64(-(1 + 2.0 ** -8))) == 0xBF80
    # one rounding only: 1 + 2^-8 - 2^-30 would round up to the tie in float32 first if rounded twice
    assert codec.bf16_encode(np.float64(1 + 2.0 ** -8 - 2.0 ** -30)) == 0x3F80
    assert codec.bf16_encode(np.float64(1 + 3 * 2.0 ** -8 - 2.0 ** -30)) == 0x3F81
    # subnormal grid, overflow, carry into the next binade
    assert codec.bf16_encode(np.float64(2.0 ** -133)) == 0x0001
    assert codec.bf16_encode(np.float64(2.0 ** -134)) == 0x0000          # tie to even (0)
    assert codec.bf16_encode(np.float64(3 * 2.0 ** -134)) == 0x0002      # tie to even (2)
    assert codec.bf16_encode(np.float64(1e39)) == 0x7F80
    assert codec.bf16_encode(np.float64(-1e39)) == 0xFF80
    assert codec.bf16_encode(np.float64(2 - 2.0 ** -9)) == 0x4000        # rounds up to 2.0
    assert codec.bf16_encode(np.float64(0.0)) == 0
    assert np.isnan(codec.bf16_decode(codec.bf16_encode(np.float64("nan"))))


def test_bf16_encode_matches_library_on_float32_inputs():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-60, 60, 200000))).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(codec.bf16_encode(x.astype(np.float64)), lib)


def test_bf16_encode_monotone():
    x = np.sort(np.random.default_rng(3).standard_normal(50000))
    y = codec.bf16_decode(codec.bf16_encode(x))
    assert np.all(np.diff(y) >= 0)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)   # half an ulp of 8 significant bits


def test_e4m3_table_against_format_definition_and_library():
    t = codec.e4m3_table()
    assert t[0x38] == 1.0
    assert t[0x7E] == 448.0
    assert t[0x08] == 2.0 ** -6          # smallest normal
    assert t[0x01] == 2.0 ** -9          # smallest subnormal
    assert t[0x07] == 7 * 2.0 ** -9
    assert t[0xB8] == -1.0
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    assert np.sum(np.isnan(t)) == 2      # no infinities, only the two NaN codes
    assert np.all(np.diff(t[:0x7F]) > 0)  # positive codes are strictly increasing
    lib = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    nan = np.isnan(lib)
    assert np.array_equal(np.isnan(t), nan)
    assert np.array_equal(t[~nan], lib[~nan])
    bits = np.array([[0x38, 0x7E], [0xB8, 0x01]], dtype=np.uint8)
    assert np.array_equal(codec.e4m3_decode(bits), [[1.0, 448.0], [-1.0, 2.0 ** -9]])
