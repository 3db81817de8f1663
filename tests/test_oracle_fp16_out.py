"""CPU tests of FP16 accumulators and outputs (paper Algorithm "T-FDPA" with F_C = FP16 and rho = RNE-FP16, Table
"Conversion functions"; Table "T-FDPA and ST-FDPA parameter selection" lists the FP16-output instructions).  Pins:
the binary16 rounder against numpy's correctly rounded float64 -> float16 conversion and against hand-picked
boundary cases; the closed form (wide F: RNE-FP16 of the exact rational); the paper's worked example of Sec. 5 carried
over to an FP16 accumulator by hand; the FP16 accumulator's own exponent range; special values with the FP16 NaN
pattern 0x7FFF of Sec. 4.2; the C form against the rational form."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, fdpa_group, emulate_mma, emulate_element, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from oracle.rounding import to_fp16, RNE, RZ
from paper_2511_10909_amd import synth


def h(x):
    return int(np.float16(x).view(np.uint16))


def test_fp16_rounder_against_numpy_and_boundaries():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, 4000), [0.0, 65504.0, 65519.99, 65520.0, 1e9, 2.0 ** -24,
                        2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -20), 2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12), 3 * 2.0 ** -25]])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    for v, w in zip(x, want):
        got = to_fp16(Fraction(float(v)), RNE)
        if v == 0:
            assert got == 0
        else:
            assert got == int(w), (v, hex(got), hex(int(w)))
    # round to zero: never away, overflow saturates at 65504
    assert to_fp16(Fraction(65519), RZ) == 0x7BFF and to_fp16(Fraction(10 ** 9), RZ) == 0x7BFF and to_fp16(Fraction(-10 ** 9), RZ) == 0xFBFF
    assert to_fp16(Fraction(65520), RNE) == 0x7C00 and to_fp16(Fraction(65519), RNE) == 0x7BFF
    assert to_fp16(Fraction(1) + Fraction(1, 2048), RNE) == 0x3C00 and to_fp16(Fraction(1) + Fraction(3, 2048), RNE) == 0x3C02   # ties to even
    assert to_fp16(Fraction(1) + Fraction(1023, 1024 * 1024), RZ) == 0x3C00
    assert to_fp16(Fraction(-1, 2 ** 25), RNE) == 0x8000 and to_fp16(Fraction(1, 2 ** 24), RNE) == 0x0001     # a tie to even zero keeps its sign


def test_wide_f_is_rne_fp16_of_the_exact_sum():
    rng = np.random.default_rng(1)
    p = ModelParams(group_len=8, frac_bits=60)
    for _ in range(300):
        a = synth.narrow_exponent_bits(rng, 8, fm.FP16, 8, 20).tolist()
        b = synth.narrow_exponent_bits(rng, 8, fm.FP16, 8, 20).tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP16, 5, 25)[0])
        exact = fm.decode(c, fm.FP16).value + sum(fm.decode(x, fm.FP16).value * fm.decode(y, fm.FP16).value for x, y in zip(a, b))
        assert fdpa_group(p, a, b, c, fm.FP16, fm.FP16, tc=fm.FP16) == to_fp16(exact, RNE)


def test_worked_example_with_fp16_accumulator():
    # Sec. 5's vector scaled to fit binary16: c = 2^11, products -2^11, -0.5, -0.25, -0.125 (exact sum -0.875).
    # Aligned at e_max = 11 with F fractional bits the small products keep what lies at or above 2^(11 - F):
    # F = 11: nothing (0.0); F = 12: -0.5; F = 13: -0.75; F = 14: all of -0.875.
    a = [h(-2.0 ** 6), h(-0.5), h(-0.25), h(-0.125)]
    b = [h(2.0 ** 5), h(1.0), h(1.0), h(1.0)]
    c = h(2.0 ** 11)
    for F, want in ((11, 0.0), (12, -0.5), (13, -0.75), (14, -0.875)):
        p = ModelParams(group_len=4, frac_bits=F, out_round=RZ)
        assert fdpa_group(p, a, b, c, fm.FP16, fm.FP16, tc=fm.FP16) == h(want), F


def test_fp16_accumulator_exponent_floor_is_minus_14():
    # c = 0 as FP16 has Exp = 1 - 15 = -14 (as FP32 it would be -126).  One product 2^-15 * 2^-15 * (1 + 2^-10)^2
    # = 2^-30 (1 + 2^-9 + 2^-20): aligned at e_max = -14 with F = 24 the unit is 2^-38, so the 2^-50 bit is cut,
    # and RNE-FP16 of 2^-30 (1 + 2^-9) is 0 either way.  With the accumulator 2^-20 (exponent -20 as FP32, but a
    # subnormal FP16 with Exp = -14) and F = 12, the product lies below the unit 2^-26 and vanishes: d = c.
    x = h(2.0 ** -15 * (1 + 2.0 ** -10))       # subnormal FP16
    p = ModelParams(group_len=1, frac_bits=12)
    c = h(2.0 ** -20)
    assert fdpa_group(p, [x], [x], c, fm.FP16, fm.FP16, tc=fm.FP16) == c
    # ... whereas a product 2^-24 (1.5), two units of 2^-26 + ..., is kept and added: 2^-20 + 2^-24 + 2^-25 -> FP16 grid 2^-24
    y, z = h(1.5 * 2.0 ** -12), h(2.0 ** -12)
    assert fdpa_group(p, [y], [z], c, fm.FP16, fm.FP16, tc=fm.FP16) == to_fp16(Fraction(2) ** -20 + Fraction(3, 2 ** 25), RNE)
    # eight products of 2^-27 each lie below that unit one by one and are all cut (d = c), although together they are
    # 2^-24, a binary16 number: with the accumulator's exponent read as -20 (its binary32 exponent) the unit would be
    # 2^-32 and the result c + 2^-24
    a8, b8 = [h(2.0 ** -13)] * 8, [h(2.0 ** -14)] * 8
    assert fdpa_group(p.with_(group_len=8), a8, b8, c, fm.FP16, fm.FP16, tc=fm.FP16) == c
    assert fdpa_group(p.with_(group_len=8, frac_bits=13), a8, b8, c, fm.FP16, fm.FP16, tc=fm.FP16) == h(2.0 ** -20 + 2.0 ** -24)
    # flush of inputs and outputs uses the binary16 threshold 2^-14
    q = ModelParams(group_len=1, frac_bits=24, ftz_in=True)
    assert fdpa_group(q, [h(1.0)], [h(1.0)], h(2.0 ** -15), fm.FP16, fm.FP16, tc=fm.FP16) == h(1.0)
    q = ModelParams(group_len=1, frac_bits=24, ftz_out=True)
    assert fdpa_group(q, [h(-2.0 ** -8)], [h(2.0 ** -8)], 0, fm.FP16, fm.FP16, tc=fm.FP16) == 0x8000
    assert fdpa_group(q.with_(ftz_out=False), [h(-2.0 ** -8)], [h(2.0 ** -8)], 0, fm.FP16, fm.FP16, tc=fm.FP16) == h(-2.0 ** -16)


def test_fp16_specials():
    p = ModelParams(group_len=2, frac_bits=24, nan_bits=0x7FFF)
    one, inf, nan = h(1.0), 0x7C00, 0x7E01
    assert fdpa_group(p, [one, one], [one, one], nan, fm.FP16, fm.FP16, tc=fm.FP16) == 0x7FFF
    assert fdpa_group(p, [inf, one], [one, one], h(3.0), fm.FP16, fm.FP16, tc=fm.FP16) == 0x7C00
    assert fdpa_group(p, [inf, one], [h(-1.0), one], inf, fm.FP16, fm.FP16, tc=fm.FP16) == 0x7FFF
    assert fdpa_group(p, [inf, one], [0, one], 0, fm.FP16, fm.FP16, tc=fm.FP16) == 0x7FFF
    assert fdpa_group(p, [one, one], [one, one], 0xFC00, fm.FP16, fm.FP16, tc=fm.FP16) == 0xFC00
    # overflow of the sum: 60000 + 2 * 4000 -> infinity under RNE, 65504 under RZ
    big = [h(4000.0), h(4000.0)]
    assert fdpa_group(p, big, [one, one], h(60000.0), fm.FP16, fm.FP16, tc=fm.FP16) == 0x7C00
    assert fdpa_group(p.with_(out_round=RZ), big, [one, one], h(60000.0), fm.FP16, fm.FP16, tc=fm.FP16) == 0x7BFF
    with pytest.raises(ValueError):
        fdpa_group(ModelParams(group_len=2, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD), [one, one], [one, one], 0, fm.FP16, fm.FP16, tc=fm.FP16)


def test_chain_rounds_to_fp16_after_every_group():
    # two groups of one product: (2048 + 1) + 1 with the intermediate rounded to binary16 (spacing 2 at 2048) gives
    # 2048 + 0 -> 2048 (tie to even) then 2048 + 1 -> 2048 again; rounded once it would be 2050
    one = h(1.0)
    p = ModelParams(group_len=1, frac_bits=24)
    assert emulate_element(p, [one, one], [one, one], h(2048.0), fm.FP16, fm.FP16, tc=fm.FP16) == h(2048.0)
    assert emulate_element(p.with_(group_len=2), [one, one], [one, one], h(2048.0), fm.FP16, fm.FP16, tc=fm.FP16) == h(2050.0)


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.E4M3, fm.E5M2), (fm.BF16, fm.FP16)])
def test_fp16_accumulator_o2_matches_oracle(ta, tb):
    rng = np.random.default_rng(400 + ta)
    for trial in range(24):
        L = int(rng.choice([1, 2, 4, 8, 0]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([11, 13, 24, 25])), c_mode=int(rng.choice([C_IN_GROUP, C_AFTER_EXACT])),
                        out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)), nan_bits=0x7FFF)
        nb, m, n, k = 2, 3, 4, 16
        if trial % 3 == 0:
            A, B = synth.random_bits(rng, (nb, m, k), ta), synth.random_bits(rng, (nb, n, k), tb)
            C = synth.random_bits(rng, (nb, m, n), fm.FP16, finite=False)
        else:
            lo, hi = {fm.FP16: (3, 20), fm.E4M3: (0, 12), fm.E5M2: (3, 20), fm.BF16: (110, 132)}[ta], {fm.FP16: (3, 20), fm.E4M3: (0, 12), fm.E5M2: (3, 20), fm.BF16: (110, 132)}[tb]
            A, B = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo), synth.narrow_exponent_bits(rng, (nb, n, k), tb, *hi)
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP16, 0, 30)
        want = emulate_mma(p, A, B, C, ta, tb, tc=fm.FP16)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb, tc=fm.FP16)
        assert np.array_equal(got, want), (trial, p, np.argwhere(got != want)[:3])
        assert want.max() <= 0xFFFF
