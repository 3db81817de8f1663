"""The exact mode of the rational oracle (c_mode = C_EXACT, Algorithm "E-FDPA"), pinned to what the paper prints, to the
definition written out with Python integers, and to the truncated models' limit."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import formats as fm
from oracle.fdpa import ModelParams, emulate_element, fdpa_group, e_fdpa, exact_width, C_EXACT, C_IN_GROUP
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from helpers import f32_bits, bits_f32, fp16_bits, bf16_bits


def test_worked_example_cdna1_rows():
    """Sec. 5, Table "divergent results": the CDNA1 instructions (E-FDPA, L = 2 for BF16 and 4 for FP16, chained) give -0.875."""
    a = [-2.0 ** 13, -0.5, -0.25, -0.125] + [0.0] * 12
    b = [2.0 ** 10, 1.0, 1.0, 1.0] + [0.0] * 12
    c = f32_bits(2.0 ** 23)
    for enc, t, L in ((fp16_bits, fm.FP16, 4), (bf16_bits, fm.BF16, 2)):
        p = ModelParams(group_len=L, c_mode=C_EXACT)
        got = emulate_element(p, [enc(x) for x in a], [enc(x) for x in b], c, t, t)
        assert bits_f32(got) == -0.875
    # one exact group of all sixteen: the same, since no intermediate rounding loses anything here
    assert bits_f32(emulate_element(ModelParams(group_len=0, c_mode=C_EXACT), [fp16_bits(x) for x in a], [fp16_bits(x) for x in b], c, fm.FP16, fm.FP16)) == -0.875


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.FP32, fm.FP32), (fm.TF32, fm.TF32)])
def test_one_group_is_the_correctly_rounded_integer_sum(ta, tb):
    """The definition with plain Python integers: every term an integer multiple of 2^-400, summed as integers, rounded
    once by the hardware double -> float conversion where the sum is a double, else by the oracle's own rounder."""
    rng = np.random.default_rng(5 + ta)
    fa, fb = fm.FORMATS[ta], fm.FORMATS[tb]
    for trial in range(300):
        L = int(rng.choice([1, 2, 4, 8, 16]))
        a = synth.random_bits(rng, (L,), ta).tolist()
        b = synth.random_bits(rng, (L,), tb).tolist()
        c = int(synth.narrow_exponent_bits(rng, (1,), fm.FP32, 60, 200)[0]) if trial % 3 else int(synth.random_bits(rng, (1,), fm.FP32)[0])
        total = 0                                          # units of 2^-400
        for x, y in zip(a, b):
            dx, dy = fm.decode(x, ta), fm.decode(y, tb)
            total += (-1) ** (dx.sign ^ dy.sign) * dx.sig * dy.sig << (dx.exp + dy.exp - dx.mbits - dy.mbits + 400)
        dc = fm.decode(c, fm.FP32)
        total += (-1) ** dc.sign * dc.sig << (dc.exp - 23 + 400)
        got = fdpa_group(ModelParams(c_mode=C_EXACT), a, b, c, ta, tb)
        assert got == e_fdpa(a, b, c, ta, tb)
        exact = Fraction(total, 1 << 400)
        if exact == Fraction(float(exact)) and abs(float(exact)) < 3e38:
            want = f32_bits(float(exact))
            if float(exact) == 0.0:
                want = 0
            assert got == want, (trial, a, b, c)


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.E5M2, fm.E4M3)])
def test_exact_mode_is_the_limit_of_the_truncated_model(ta, tb):
    """With F at least the distance from e_max to the lowest set bit of any term, T-FDPA cuts nothing and must agree."""
    rng = np.random.default_rng(17 + ta)
    for trial in range(200):
        L = int(rng.choice([2, 4, 8]))
        a = synth.random_bits(rng, (2 * L,), ta).tolist()
        b = synth.random_bits(rng, (2 * L,), tb).tolist()
        c = int(synth.narrow_exponent_bits(rng, (1,), fm.FP32, 100, 150)[0])
        F = max(exact_width(a[:L], b[:L], c, ta, tb), 1)
        one = fdpa_group(ModelParams(c_mode=C_EXACT), a[:L], b[:L], c, ta, tb)
        assert one == fdpa_group(ModelParams(frac_bits=F, c_mode=C_IN_GROUP), a[:L], b[:L], c, ta, tb)
        # chained: every group rounds once
        two = emulate_element(ModelParams(group_len=L, c_mode=C_EXACT), a, b, c, ta, tb)
        assert two == fdpa_group(ModelParams(c_mode=C_EXACT), a[L:], b[L:], one, ta, tb)


def test_exact_mode_switches_and_specials():
    p = ModelParams(c_mode=C_EXACT, nan_bits=0x7FFFFFFF)
    inf, nan, one, zero = 0x7C00, 0x7E00, 0x3C00, 0
    assert fdpa_group(p, [inf, one], [one, one], 0, fm.FP16, fm.FP16) == 0x7F800000
    assert fdpa_group(p, [inf, one], [zero, one], 0, fm.FP16, fm.FP16) == 0x7FFFFFFF          # inf * 0
    assert fdpa_group(p, [inf, one], [one, one], 0xFF800000, fm.FP16, fm.FP16) == 0x7FFFFFFF   # +inf and -inf
    assert fdpa_group(p, [nan, one], [one, one], 0, fm.FP16, fm.FP16) == 0x7FFFFFFF
    # cancellation to an exact zero: +0.0; RZ against RNE on a tie; output flush
    assert fdpa_group(p, [one, 0xBC00], [one, one], 0x80000000, fm.FP16, fm.FP16) == 0
    tie_c = f32_bits(2.0 ** 24)                                                            # 2^24 + 1: halfway between two floats
    assert fdpa_group(p, [one], [one], tie_c, fm.FP16, fm.FP16) == f32_bits(2.0 ** 24)        # ties to even
    assert fdpa_group(p, [0x4200], [one], tie_c, fm.FP16, fm.FP16) == f32_bits(2.0 ** 24 + 4)  # 2^24 + 3 -> up
    assert fdpa_group(p.with_(out_round=RZ), [0x4200], [one], tie_c, fm.FP16, fm.FP16) == f32_bits(2.0 ** 24 + 2)
    tiny = fdpa_group(p, [1], [1], 0, fm.FP16, fm.FP16)                                        # 2^-48: a normal binary32
    assert bits_f32(tiny) == 2.0 ** -48
    assert fdpa_group(p.with_(ftz_out=True), [1], [1], 1, fm.FP16, fm.FP16) == f32_bits(2.0 ** -48)
    assert fdpa_group(p.with_(ftz_out=True), [0], [0], 1, fm.FP16, fm.FP16) == 0               # a subnormal result is flushed
    assert fdpa_group(p.with_(ftz_in=True), [1], [one], 0, fm.FP16, fm.FP16) == 0              # a subnormal operand is flushed
