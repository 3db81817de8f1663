"""CPU tests of the FP6 (E2M3, E3M2) and FP4 (E2M1) operand types (Require line of paper Algorithms "T-FDPA" and
"ST-FDPA": F_A, F_B in {..., FP8, FP6, FP4}; element formats of the OCP microscaling specification).  Pins: the
published value sets of the three formats; brute force over every operand pair against exact rational arithmetic;
the unnormalised exponent of FP4 / FP6 subnormals (hand-derived truncation case); C form = rational form."""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, fdpa_group, emulate_mma, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from oracle.rounding import to_fp32, RNE, RZ
from helpers import f32_bits, bits_f32
from paper_2511_10909_amd import synth

NEW = (fm.E2M3, fm.E3M2, fm.E2M1)


def test_value_sets():
    # E2M1: the eight magnitudes of the specification, sign in bit 3
    mags = [fm.decode(c, fm.E2M1).value for c in range(8)]
    assert mags == [0, Fraction(1, 2), 1, Fraction(3, 2), 2, 3, 4, 6]
    assert [fm.decode(8 + c, fm.E2M1).value for c in range(8)] == [-x for x in mags]
    assert all(fm.decode(c, fm.E2M1).finite for c in range(16))
    # E2M3: 64 codes, largest 7.5, smallest subnormal 0.125, smallest normal 1.0; E3M2: largest 28, smallest subnormal
    # 0.0625, smallest normal 0.25; neither has an infinity or a NaN
    assert fm.decode(0b011111, fm.E2M3).value == Fraction(15, 2) and fm.decode(0b000001, fm.E2M3).value == Fraction(1, 8)
    assert fm.decode(0b001000, fm.E2M3).value == 1 and fm.decode(0b111111, fm.E2M3).value == Fraction(-15, 2)
    assert fm.decode(0b011111, fm.E3M2).value == 28 and fm.decode(0b000001, fm.E3M2).value == Fraction(1, 16)
    assert fm.decode(0b000100, fm.E3M2).value == Fraction(1, 4) and fm.decode(0b100100, fm.E3M2).value == Fraction(-1, 4)
    for t, n in ((fm.E2M3, 64), (fm.E3M2, 64)):
        vals = [fm.decode(c, t) for c in range(n)]
        assert all(v.finite for v in vals)
        pos = [v.value for v in vals[:n // 2]]
        assert pos == sorted(pos) and len(set(pos)) == n // 2                 # monotone in the code, all distinct
    # bits above the code are ignored
    assert fm.decode(0xF0 | 0b0101, fm.E2M1).value == fm.decode(0b0101, fm.E2M1).value
    # unnormalised exponents: codes with exponent field 0 have Exp = 1 - bias and no hidden bit
    assert fm.decode(0b0001, fm.E2M1).exp == 0 and fm.decode(0b0001, fm.E2M1).sig == 1      # 0.5 = 0.1b * 2^0
    assert fm.decode(0b000011, fm.E3M2).exp == -2 and fm.decode(0b000011, fm.E3M2).sig == 3


@pytest.mark.parametrize("ta,tb", [(fm.E2M1, fm.E2M1), (fm.E2M3, fm.E3M2), (fm.E2M1, fm.E4M3), (fm.E5M2, fm.E2M3)])
def test_every_operand_pair_against_exact_arithmetic(ta, tb):
    # k = 1, F wide enough to keep every bit: d = RNE-FP32(a b + c) with the product and the sum exact
    p = ModelParams(group_len=1, frac_bits=90)
    na, nb_ = 1 << fm.FORMATS[ta].width, 1 << fm.FORMATS[tb].width
    for c in (0.0, 1.0, -0.3333333432674408, 3.0e-5):
        cb = f32_bits(c)
        for x, y in product(range(na), range(nb_)):
            dx, dy = fm.decode(x, ta), fm.decode(y, tb)
            if not (dx.finite and dy.finite):
                continue
            want = to_fp32(dx.value * dy.value + Fraction(float(np.float32(c))), RNE)
            assert fdpa_group(p, [x], [y], cb, ta, tb) == want, (x, y, c)


def test_subnormal_fp4_keeps_its_unnormalised_exponent():
    # FP4: 0.5 is the subnormal 0.1b * 2^0, so 0.5 * 0.5 has e_k = 0 + 0 and significand product 0.01b.  Next to
    # 6 * 6 = 36 = 10.01b * 2^(2+2), e_max = 4; with F = 5 the unit is 2^-1: the 0.25 is cut (36.0); with F = 6 it is
    # kept (36.25).  Were the operand normalised (Exp = -1), nothing would change here, but a zero operand shows it:
    # 0 * 6 has e_k = 0 + 2, so alone with c = 2^-10 (e_c = -10) it sets e_max = 2 and F = 11 cuts c to nothing.
    half, six, zero = 0b0001, 0b0111, 0
    p = ModelParams(group_len=2, frac_bits=5, out_round=RZ)
    assert bits_f32(fdpa_group(p, [six, half], [six, half], 0, fm.E2M1, fm.E2M1)) == 36.0
    assert bits_f32(fdpa_group(p.with_(frac_bits=6), [six, half], [six, half], 0, fm.E2M1, fm.E2M1)) == 36.25
    q = ModelParams(group_len=1, frac_bits=11, out_round=RZ)
    assert fdpa_group(q, [zero], [six], f32_bits(2.0 ** -10), fm.E2M1, fm.E2M1) == 0
    assert bits_f32(fdpa_group(q.with_(frac_bits=12), [zero], [six], f32_bits(2.0 ** -10), fm.E2M1, fm.E2M1)) == 2.0 ** -10


@pytest.mark.parametrize("ta,tb", [(fm.E2M1, fm.E2M1), (fm.E2M3, fm.E2M3), (fm.E3M2, fm.E2M1), (fm.E4M3, fm.E2M1), (fm.E3M2, fm.E5M2)])
def test_o2_matches_oracle_on_fp6_fp4(ta, tb):
    rng = np.random.default_rng(70 + 9 * ta + tb)
    for trial in range(16):
        L = int(rng.choice([2, 4, 8, 16, 32]))
        mode = int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([6, 13, 25])), c_mode=mode, out_round=int(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)))
        if mode == C_AFTER_RD:
            p = p.with_(frac_bits2=31, split=int(rng.integers(0, 4 if (L or k) % 4 == 0 else 3)), f2_at_leading_bit=bool(rng.integers(0, 2)))
        nb, m, n, k = 2, 3, 3, 32
        A = rng.integers(0, 1 << fm.FORMATS[ta].width, size=(nb, m, k)).astype(np.uint8)
        B = rng.integers(0, 1 << fm.FORMATS[tb].width, size=(nb, n, k)).astype(np.uint8)
        if ta == fm.E4M3 or ta == fm.E5M2:
            A = synth.random_bits(rng, (nb, m, k), ta)
        if tb == fm.E4M3 or tb == fm.E5M2:
            B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 110, 135)
        SA = rng.integers(100, 150, size=(nb, m, 1)).astype(np.uint8)
        SB = rng.integers(100, 150, size=(nb, n, 1)).astype(np.uint8)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (trial, p)
        want = emulate_mma(p, A, B, C, ta, tb, SA, SB, 32)
        got, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, 32, ta, tb)
        assert np.array_equal(got, want), (trial, p)


def test_tf32_operands_ignore_the_low_13_bits():
    # TF32 (Require lines of Algorithms "T-FDPA" and "TR-FDPA"): a binary32 word of which the sign, the 8 exponent bits
    # and the top 10 mantissa bits count.  Values with 11 significant bits behave like FP16 values of the same
    # significand; the low 13 bits change nothing; specials are those of binary32.
    rng = np.random.default_rng(12)
    p = ModelParams(group_len=4, frac_bits=24, out_round=RZ)
    for _ in range(200):
        x = synth.narrow_exponent_bits(rng, 8, fm.FP16, 5, 25)
        xf = x.astype(np.uint16).view(np.float16).astype(np.float32).view(np.uint32)          # the same values as binary32 words
        a16, b16, a32, b32 = x[:4].tolist(), x[4:].tolist(), xf[:4].tolist(), xf[4:].tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 110, 140)[0])
        want = fdpa_group(p, a16, b16, c, fm.FP16, fm.FP16)
        assert fdpa_group(p, a32, b32, c, fm.TF32, fm.TF32) == want
        noisy = [int(v) | int(rng.integers(0, 1 << 13)) for v in a32]
        assert fdpa_group(p, noisy, b32, c, fm.TF32, fm.TF32) == want
    assert fm.decode(0x7F800000, fm.TF32).cls == fm.INF and fm.decode(0x7F802000, fm.TF32).cls == fm.NAN
    assert fm.decode(0x7F801FFF, fm.TF32).cls == fm.INF                 # a NaN payload only in the ignored bits reads as infinity
    assert fm.decode(0x00002000, fm.TF32).cls == fm.SUBNORMAL and fm.decode(0x00001FFF, fm.TF32).cls == fm.ZERO
    # C form = rational form
    for trial in range(10):
        q = ModelParams(group_len=int(rng.choice([2, 4, 8])), frac_bits=int(rng.choice([13, 24, 25])), out_round=int(rng.integers(0, 2)),
                        c_mode=int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD])))
        if q.c_mode == C_AFTER_RD:
            q = q.with_(frac_bits2=31)
        A = synth.random_bits(rng, (2, 3, 16), fm.FP32, finite=(trial % 2 == 0))
        B = synth.random_bits(rng, (2, 3, 16), fm.FP32)
        if trial % 3:
            A = synth.narrow_exponent_bits(rng, (2, 3, 16), fm.FP32, 100, 150)
            B = synth.narrow_exponent_bits(rng, (2, 3, 16), fm.FP32, 100, 150)
        C = synth.narrow_exponent_bits(rng, (2, 3, 3), fm.FP32, 80, 170)
        want = emulate_mma(q, A, B, C, fm.TF32, fm.TF32)
        got, _ = o2lib.emulate_mma(q, A, B, C, fm.TF32, fm.TF32)
        assert np.array_equal(got, want), (trial, q)
