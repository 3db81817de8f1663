"""Pins for the oracle's decoders and rounders against libraries and closed forms."""
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import formats as fm
from oracle.rounding import rne_fp32, rz_fp32, to_fp32, RNE, RZ
from helpers import f32_bits, bits_f32


def _value_or_special(d):
    if d.cls == fm.NAN:
        return "nan"
    if d.cls == fm.INF:
        return "-inf" if d.sign else "inf"
    return d.value


def test_fp16_decode_all_codes_against_numpy():
    codes = np.arange(65536, dtype=np.uint16)
    vals = codes.view(np.float16).astype(np.float64)
    for c in range(65536):
        d = fm.decode(c, fm.FP16)
        v = vals[c]
        if np.isnan(v):
            assert d.cls == fm.NAN
        elif np.isinf(v):
            assert d.cls == fm.INF and d.sign == (v < 0)
        else:
            assert d.value == Fraction(float(v)), hex(c)
            assert d.sign == (c >> 15)


@pytest.mark.parametrize("fmt,tdt", [(fm.E4M3, torch.float8_e4m3fn), (fm.E5M2, torch.float8_e5m2)])
def test_fp8_decode_all_codes_against_torch(fmt, tdt):
    vals = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(tdt).to(torch.float64).numpy()
    for c in range(256):
        d = fm.decode(c, fmt)
        v = vals[c]
        if np.isnan(v):
            assert d.cls == fm.NAN
        elif np.isinf(v):
            assert d.cls == fm.INF
        else:
            assert d.value == Fraction(float(v)), hex(c)


def test_bf16_decode_all_codes_against_torch():
    codes = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    vals = codes.view(torch.bfloat16).to(torch.float64).numpy()
    for c in range(65536):
        d = fm.decode(c, fm.BF16)
        v = vals[c]
        if np.isnan(v):
            assert d.cls == fm.NAN
        elif np.isinf(v):
            assert d.cls == fm.INF
        else:
            assert d.value == Fraction(float(v)), hex(c)


def test_format_extremes():
    assert fm.decode(0x7E, fm.E4M3).value == 448           # largest finite E4M3
    assert fm.decode(0x7F, fm.E4M3).cls == fm.NAN
    assert fm.decode(0x78, fm.E4M3).value == 256           # exponent field 15 is a normal binade in E4M3
    assert fm.decode(0x7B, fm.E5M2).value == 57344
    assert fm.decode(0x7C, fm.E5M2).cls == fm.INF
    assert fm.decode(0x01, fm.E4M3).value == Fraction(1, 512)
    assert fm.decode(0x01, fm.E5M2).value == Fraction(1, 65536)


def test_unnormalised_exponent_of_zero_and_subnormal():
    # Exp = 1 - bias for exponent field 0, no hidden bit
    for fmt, e in [(fm.E4M3, -6), (fm.E5M2, -14), (fm.FP16, -14), (fm.BF16, -126), (fm.FP32, -126)]:
        z = fm.decode(0, fmt)
        assert z.cls == fm.ZERO and z.exp == e and z.sig == 0
        s = fm.decode(1, fmt)
        assert s.cls == fm.SUBNORMAL and s.exp == e and s.sig == 1


def test_fp32_decode_random_against_struct():
    rng = np.random.default_rng(1)
    for b in rng.integers(0, 1 << 32, size=5000, dtype=np.uint64):
        b = int(b)
        d = fm.decode(b, fm.FP32)
        v = bits_f32(b)
        if v != v:
            assert d.cls == fm.NAN
        elif v in (float("inf"), float("-inf")):
            assert d.cls == fm.INF
        else:
            assert d.value == Fraction(v)


def test_rne_matches_libc_on_exact_doubles():
    # a double is an exact rational; the hardware double->float conversion rounds it once (RNE)
    rng = np.random.default_rng(2)
    xs = rng.standard_normal(20000) * np.exp(rng.uniform(-100, 88, 20000))
    xs = np.concatenate([xs, rng.standard_normal(2000) * 1e-41, [0.0, 1e-46, -1e-46, 3.4028235e38, 3.4028236e38]])
    for x in xs:
        got = rne_fp32(Fraction(float(x)))
        assert got == (0 if x == 0 else f32_bits(x)), x


def test_rne_ties_and_boundaries():
    one = Fraction(1)
    ulp = Fraction(1, 1 << 23)
    assert rne_fp32(one + ulp / 2) == f32_bits(1.0)                       # tie -> even (down)
    assert rne_fp32(one + ulp + ulp / 2) == f32_bits(1.0) + 2             # tie -> even (up)
    assert rne_fp32(one + ulp / 2 + Fraction(1, 1 << 80)) == f32_bits(1.0) + 1
    assert rne_fp32(Fraction(2) - ulp / 4) == f32_bits(2.0)               # carry into next binade
    tiny = Fraction(1, 1 << 149)
    assert rne_fp32(tiny / 2) == 0                                        # tie at half the smallest subnormal -> even = 0
    assert rne_fp32(-tiny / 2) == 0x80000000                              # sign kept on a non-zero value
    assert rne_fp32(tiny / 2 + Fraction(1, 1 << 200)) == 1
    assert rne_fp32(Fraction(3, 2) * tiny) == 2
    maxf = Fraction(bits_f32(0x7F7FFFFF))
    half_ulp_max = Fraction(2) ** (127 - 24)
    assert rne_fp32(maxf + half_ulp_max - 1) == 0x7F7FFFFF
    assert rne_fp32(maxf + half_ulp_max) == 0x7F800000                    # tie -> even = 2^128 -> inf
    assert rne_fp32(-(maxf + half_ulp_max)) == 0xFF800000
    assert rne_fp32(0) == 0


def test_rz_is_truncation():
    rng = np.random.default_rng(3)
    xs = rng.standard_normal(5000) * np.exp(rng.uniform(-100, 88, 5000))
    for x in xs:
        fx = Fraction(float(x))
        b = rz_fp32(fx)
        v = Fraction(bits_f32(b))
        assert abs(v) <= abs(fx) and (b >> 31) == (x < 0)
        nxt = Fraction(bits_f32(b + 1))                                     # next magnitude up
        assert abs(nxt) > abs(fx)
    assert rz_fp32(Fraction(2) ** 200) == 0x7F7FFFFF
    assert rz_fp32(-Fraction(2) ** 128) == 0xFF7FFFFF
    assert rz_fp32(Fraction(1, 1 << 150)) == 0
    assert rz_fp32(-Fraction(1, 1 << 150)) == 0x80000000


def test_rne_within_half_ulp_rz_within_one_ulp():
    # error bounds of the output conversion: paper Sec. 6.1, Table "Sources and upper bounds"
    rng = np.random.default_rng(4)
    for _ in range(3000):
        num = int(rng.integers(1, 1 << 62))
        den = int(rng.integers(1, 1 << 62))
        x = Fraction(num, den) * Fraction(2) ** int(rng.integers(-120, 100))
        for mode, bound in ((RNE, Fraction(1, 2)), (RZ, Fraction(1))):
            b = to_fp32(x, mode)
            v = Fraction(bits_f32(b))
            e = max(((b >> 23) & 0xFF), 1) - 127
            ulp = Fraction(2) ** (e - 23)
            assert abs(v - x) <= bound * ulp
