"""CPU tests of block-scaled operation (paper Algorithm "ST-FDPA": T-FDPA whose products also take
Exp(alpha) + Exp(beta) of their block's E8M0 scale factors).  The paper prints no worked value for it, so the pins are
what the definition fixes: unit scales change nothing; a power-of-two scale commutes with exact arithmetic (closed
form: the correctly rounded exact result on the scaled operands); scales move e_max and hence what is truncated;
NaN scales; and the C form equals the rational form."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_mma, emulate_element, fdpa_group, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, SPLIT_HALVES
from oracle.rounding import rne_fp32
from helpers import f32_bits, bits_f32
from paper_2511_10909_amd import synth


def e4m3(x):
    import torch
    return int(torch.tensor([x], dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8)[0])


def test_unit_scales_change_nothing():
    rng = np.random.default_rng(1)
    A = synth.random_bits(rng, (2, 3, 64), fm.E4M3)
    B = synth.random_bits(rng, (2, 4, 64), fm.E5M2)
    C = synth.narrow_exponent_bits(rng, (2, 3, 4), fm.FP32, 100, 150)
    ones_a, ones_b = np.full((2, 3, 2), 127, dtype=np.uint8), np.full((2, 4, 2), 127, dtype=np.uint8)
    for p in (ModelParams(group_len=32, frac_bits=25), ModelParams(group_len=16, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD),
              ModelParams(group_len=8, frac_bits=24, c_mode=C_AFTER_EXACT)):
        assert np.array_equal(emulate_mma(p, A, B, C, fm.E4M3, fm.E5M2, ones_a, ones_b, 32), emulate_mma(p, A, B, C, fm.E4M3, fm.E5M2))


def test_scales_are_exact_powers_of_two_in_the_wide_limit():
    # with F wide nothing is truncated: d = RNE-FP32(c + sum 2^(sa + sb - 254) a_k b_k), block by block
    rng = np.random.default_rng(2)
    p = ModelParams(group_len=32, frac_bits=700)
    for _ in range(60):
        a = synth.random_bits(rng, 64, fm.E4M3).tolist()
        b = synth.random_bits(rng, 64, fm.E4M3).tolist()
        a = [x if (x & 0x7F) != 0x7F else 0x30 for x in a]
        b = [x if (x & 0x7F) != 0x7F else 0x30 for x in b]
        sa, sb = rng.integers(100, 150, size=2).tolist(), rng.integers(100, 150, size=2).tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 90, 170)[0])
        d = c
        for g in range(2):
            v = fm.decode(d, fm.FP32).value
            for k in range(32 * g, 32 * g + 32):
                v += fm.decode(a[k], fm.E4M3).value * fm.decode(b[k], fm.E4M3).value * Fraction(2) ** (sa[g] + sb[g] - 254)
            d = rne_fp32(v) if v != 0 else 0
        assert emulate_element(p, a, b, c, fm.E4M3, fm.E4M3, sa, sb, 32) == d


def test_scales_enter_e_max():
    # two blocks of one product each (block = 1 for the sake of the example), F = 8: 1*1 scaled by 2^0 and
    # (1 + 2^-2)*1 scaled by 2^-8.  e_max = 0: the second term 2^-8 + 2^-10 keeps 2^-8 only
    p = ModelParams(group_len=2, frac_bits=8)
    a, b = [e4m3(1.0), e4m3(1.25)], [e4m3(1.0), e4m3(1.0)]
    d = emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [127, 119], [127, 127], 1)
    assert bits_f32(d) == 1.0 + 2.0 ** -8
    # the other way round the first product is the small one: e_max = 8, 1 * 2^0 is kept exactly
    d = emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [127, 135], [127, 127], 1)
    assert bits_f32(d) == 1.0 + 1.25 * 2.0 ** 8
    # scales of both operands add
    d = emulate_element(ModelParams(group_len=1, frac_bits=24), [e4m3(1.5)], [e4m3(1.0)], 0, fm.E4M3, fm.E4M3, [130], [120], 1)
    assert bits_f32(d) == 1.5 * 2.0 ** -4


def test_nan_scale_and_range():
    p = ModelParams(group_len=2, frac_bits=24, nan_bits=0x7FFFFFFF)
    a, b = [e4m3(1.0), e4m3(1.0)], [e4m3(1.0), e4m3(1.0)]
    assert emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [0xFF], [127], 2) == 0x7FFFFFFF
    assert emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [127], [0xFF], 2) == 0x7FFFFFFF
    # extreme scales: 2^127 * 2^127 overflows the output conversion (RNE: infinity); 2^-127 * 2^-127 underflows to +0
    assert emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [254], [254], 2) == 0x7F800000
    assert emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [0], [0], 2) == 0
    with pytest.raises(ValueError):
        emulate_element(p, a, b, 0, fm.E4M3, fm.E4M3, [127, 127], [127], 2)


@pytest.mark.parametrize("ta,tb", [(fm.E4M3, fm.E4M3), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16)])
def test_o2_equals_rational_form_with_scales(ta, tb):
    rng = np.random.default_rng(60 + ta + tb)
    for trial in range(14):
        block = int(rng.choice([8, 16, 32]))
        k = block * int(rng.integers(1, 4))
        L = int(rng.choice([x for x in (2, 4, 8, 16, 32, 0) if x == 0 or k % x == 0]))
        mode = int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([8, 13, 24, 25, 30])), c_mode=mode, out_round=int(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)))
        if mode == C_AFTER_RD:
            p = p.with_(frac_bits2=31, split=int(rng.integers(0, 4 if (L or k) % 4 == 0 else 3)) if (L or k) % 2 == 0 else 0, f2_at_leading_bit=bool(rng.integers(0, 2)),
                        acc_special_truncation=bool(rng.integers(0, 2)), sum_drop_distance=int(rng.choice([0, 28])))
        nb, m, n = 2, 3, 4
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 60, 200)
        SA = rng.integers(90, 165, size=(nb, m, k // block)).astype(np.uint8)
        SB = rng.integers(90, 165, size=(nb, n, k // block)).astype(np.uint8)
        if trial % 5 == 0:
            SA[0, 0, 0] = 0xFF
            SB[1, 1, 0] = 0
            SA[1, 2, 0] = 254
        want = emulate_mma(p, A, B, C, ta, tb, SA, SB, block)
        got, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, block, ta, tb)
        assert np.array_equal(got, want), (p, block, np.argwhere(got != want)[:3])


# ---- wide_products: no infinity from a single product of magnitude >= 2^128 ---------------------------------

def _bf16(x):
    b = np.float32(x).view(np.uint32)
    assert b & 0xFFFF == 0
    return int(b >> 16)


def test_wide_products_cancel_instead_of_nan():
    # 2^100 * 2^30 - 2^100 * 2^30 + c: with the overflow rule of Sec. 4.2 both products are infinities of opposite
    # sign (NaN); with wide products they cancel exactly, and what is left is the accumulator rounded down to F bits
    # below E = 130: nothing of c = 1.5, all of c = 2^120
    p = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, nan_bits=0xFFC00000)
    a = [_bf16(2.0 ** 100), _bf16(-2.0 ** 100)] + [0] * 6
    b = [_bf16(2.0 ** 30), _bf16(2.0 ** 30)] + [0] * 6
    c = int(np.float32(1.5).view(np.uint32))
    assert fdpa_group(p, a, b, c, fm.BF16, fm.BF16) == 0xFFC00000
    assert fdpa_group(p.with_(wide_products=True), a, b, c, fm.BF16, fm.BF16) == 0
    big = int(np.float32(2.0 ** 120).view(np.uint32))
    assert fdpa_group(p, a, b, big, fm.BF16, fm.BF16) == 0xFFC00000
    assert fdpa_group(p.with_(wide_products=True), a, b, big, fm.BF16, fm.BF16) == big
    # a single wide product overflows only through the conversion: RNE gives infinity, RZ the largest finite value
    a[1] = 0
    assert fdpa_group(p.with_(wide_products=True), a, b, c, fm.BF16, fm.BF16) == 0x7F800000
    assert fdpa_group(p.with_(wide_products=True, out_round=1), a, b, c, fm.BF16, fm.BF16) == 0x7F7FFFFF
    # 2^130 - 2^130 (1 - 2^-7) = 2^123: finite
    a[1] = _bf16(-2.0 ** 100 * (1 - 2.0 ** -7))
    assert fdpa_group(p.with_(wide_products=True), a, b, 0, fm.BF16, fm.BF16) == int(np.float32(2.0 ** 123).view(np.uint32))
    # with scales: 1.5 * 2^(200) - 1.5 * 2^(200) + 0 = 0
    a8 = [0x3C, 0xBC] + [0] * 6
    b8 = [0x38, 0x38] + [0] * 6
    assert fdpa_group(p.with_(wide_products=True), a8, b8, 0, fm.E4M3, fm.E4M3, scale_exp=[200] * 8) == 0
    assert fdpa_group(p, a8, b8, 0, fm.E4M3, fm.E4M3, scale_exp=[200] * 8) == 0xFFC00000


def test_wide_products_o2_matches_oracle():
    rng = np.random.default_rng(77)
    for trial in range(40):
        ta, tb = [(fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.BF16, fm.FP16)][trial % 3]
        L = int(rng.choice([2, 4, 8]))
        k = 16
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([13, 24])), frac_bits2=31, c_mode=C_AFTER_RD, wide_products=True,
                        split=int(rng.integers(0, 4 if (L or k) % 4 == 0 else 3)), skip_zero_terms=bool(rng.integers(0, 2)), out_round=int(rng.integers(0, 2)),
                        f2_at_leading_bit=bool(rng.integers(0, 2)), acc_special_truncation=bool(rng.integers(0, 2)))
        nb, m, n = 2, 3, 3
        if ta == fm.BF16:
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 180, 254)
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 180 if tb == fm.BF16 else 1, 254 if tb == fm.BF16 else 30)
        else:
            A = synth.random_bits(rng, (nb, m, k), ta)
            B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 200, 254)
        SA = rng.integers(150, 255, size=(nb, m, k // 8)).astype(np.uint8)
        SB = rng.integers(150, 255, size=(nb, n, k // 8)).astype(np.uint8)
        want = emulate_mma(p, A, B, C, ta, tb, SA, SB, 8)
        got, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, 8, ta, tb)
        assert np.array_equal(got, want), (trial, p)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (trial, p)


# ---- f2_at_leading_bit in the subnormal range: the rounding position stops at 2^(-126 - F2) --------------------

def test_leading_bit_rounding_stops_at_smallest_normal_exponent():
    p = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, f2_at_leading_bit=True, skip_zero_terms=True)
    a = [e4m3(1.0), e4m3(1.0)] + [0] * 6
    b = [e4m3(1.0), e4m3(1.0)] + [0] * 6
    # 2^-150 + 2^-158: half a last place of the subnormal grid and a little more.  Below the leading bit 31 bits would
    # keep the little more (result 2^-149); the rounding position 2^-157 does not, and the tie goes to even (zero).
    # (Without the leading-bit rule the position is 2^(E - 31) with E = -126, the zero accumulator's exponent: the same.)
    se = [-150, -158] + [0] * 6
    assert fdpa_group(p, a, b, 0, fm.E4M3, fm.E4M3, scale_exp=se) == 0
    assert fdpa_group(p.with_(f2_at_leading_bit=False), a, b, 0, fm.E4M3, fm.E4M3, scale_exp=se) == 0
    # 2^-150 + 2^-157 is kept: above the tie
    assert fdpa_group(p, a, b, 0, fm.E4M3, fm.E4M3, scale_exp=[-150, -157] + [0] * 6) == 1
    # negative: -(3 2^-150) + 2^-158 = -1.5 ulp + a little: rounded down to -1.5 ulp first, tie to even: -2 ulp
    a[0] = e4m3(-1.5)
    assert fdpa_group(p, a, b, 0, fm.E4M3, fm.E4M3, scale_exp=[-149, -158] + [0] * 6) == 0x80000002
    assert fdpa_group(p.with_(f2_at_leading_bit=False), a, b, 0, fm.E4M3, fm.E4M3, scale_exp=[-149, -158] + [0] * 6) == 0x80000002
    # a zero accumulator takes part with the exponent -126: a product sum 28 or more binary places below it is dropped
    q = p.with_(sum_drop_distance=28)
    a16, b16 = [e4m3(1.25)] * 8, [e4m3(1.0)] * 8
    assert fdpa_group(q, a16, b16, 0, fm.E4M3, fm.E4M3, scale_exp=[-153] * 8) == 1        # 10 * 2^-153 = 0.625 of 2^-149
    assert fdpa_group(q, a16, b16, 0, fm.E4M3, fm.E4M3, scale_exp=[-154] * 8) == 0
    assert fdpa_group(p, a16, b16, 0, fm.E4M3, fm.E4M3, scale_exp=[-154] * 8) == 0        # 0.3125: rounds to zero anyway
    a16, b16 = [e4m3(1.75)] * 8, [e4m3(1.5)] * 8                                         # 21 * 2^-154 = 0.65625 of 2^-149
    assert fdpa_group(p, a16, b16, 0, fm.E4M3, fm.E4M3, scale_exp=[-154] * 8) == 1
    assert fdpa_group(q, a16, b16, 0, fm.E4M3, fm.E4M3, scale_exp=[-154] * 8) == 0
    # results of 2^-126 and more are untouched by the floor
    assert fdpa_group(p, a, b, 0, fm.E4M3, fm.E4M3, scale_exp=[-100, -135] + [0] * 6) == \
        fdpa_group(p.with_(f2_at_leading_bit=False, frac_bits2=40), a, b, 0, fm.E4M3, fm.E4M3, scale_exp=[-100, -135] + [0] * 6)


def test_tiny_range_o2_matches_oracle():
    rng = np.random.default_rng(91)
    for trial in range(30):
        ta, tb = [(fm.E4M3, fm.E4M3), (fm.E5M2, fm.E4M3), (fm.BF16, fm.BF16)][trial % 3]
        L = int(rng.choice([2, 8, 16]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([13, 24])), frac_bits2=31, c_mode=C_AFTER_RD,
                        wide_products=True, split=int(rng.integers(0, 4 if L % 4 == 0 else 3)), skip_zero_terms=bool(rng.integers(0, 2)),
                        f2_at_leading_bit=True, frac_bits_acc=24, frac_bits_merge=24 if trial % 2 else 0, zero_result_positive=bool(rng.integers(0, 2)))
        if p.frac_bits_merge and p.split == 0:
            p = p.with_(frac_bits_merge=0)
        nb, m, n, k = 2, 3, 3, 32
        if ta == fm.BF16:
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 40, 70)
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 40, 70)
        else:
            A = synth.random_bits(rng, (nb, m, k), ta)
            B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 0, 3) if trial % 2 else np.zeros((nb, m, n), dtype=np.uint32)
        SA = rng.integers(40, 70, size=(nb, m, k // 16)).astype(np.uint8)
        SB = rng.integers(40, 70, size=(nb, n, k // 16)).astype(np.uint8)
        if ta == fm.BF16:
            SA[:] = 127
            SB[:] = 127
        want = emulate_mma(p, A, B, C, ta, tb, SA, SB, 16)
        got, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, 16, ta, tb)
        assert np.array_equal(got, want), (trial, p)
        assert np.count_nonzero(want & 0x7FFFFFFF) > want.size // 8 or ta == fm.BF16
