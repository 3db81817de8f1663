"""CPU tests of the oracle's TR-FDPA and GTR-FDPA operations (paper Sec. 4.1.3, Algorithms
"TR-FDPA" and "GTR-FDPA"; overflow rule of Sec. 4.2; parameters of Table "TR-FDPA and GTR-FDPA
parameter selection": F = 24, F2 = 31, RNE-FP32, L_max = 8 for 16-bit and 16 for 8-bit inputs).

The paper's printed values for these operations (Table of d_00, CDNA3 rows) are checked with the
other rows of that table in test_oracle_model.py / test_oracle_o2.py.  That example exercises the
round-down of the even/odd merge only, so the other roundings are pinned here by cases whose results
are worked out by hand from the algorithms' steps (derivations beside each case), by the closed form
the operations reduce to when nothing is lost, and by order relations that hold for any input.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import (ModelParams, fdpa_group, emulate_mma, e_fdpa,
                         C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD)
from oracle.rounding import RNE, RZ
from oracle.stats import ordered_key
from helpers import f32_bits, bits_f32, fp16_bits, bf16_bits
from paper_2511_10909_amd import synth

TR = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
GTR = ModelParams(group_len=16, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD_EVEN_ODD)
WIDE = 700


def _pad(vals, L, enc=fp16_bits):
    return [enc(v) for v in vals] + [enc(0.0)] * (L - len(vals))


def _run(p, a, b, c, L=8, enc=fp16_bits, t=fm.FP16):
    return fdpa_group(p, _pad(a, L, enc), _pad(b, L, enc), f32_bits(c), t, t)


# ------------------------------------------------------------------ hand-derived cases
def test_accumulator_is_rounded_down_to_F_bits():
    # one product 1*1: T = 1 at e_max = 0.  c = -2^-30: E = 0, s_c' = RD_24(-2^-30) = -2^-24,
    # S = 1 - 2^-24, which binary32 holds exactly (0x3F7FFFFF).  Truncation toward zero would give 1.0.
    assert _run(TR, [1.0], [1.0], -2.0 ** -30) == 0x3F7FFFFF
    # a positive accumulator of the same size is rounded down to 0
    assert _run(TR, [1.0], [1.0], 2.0 ** -30) == 0x3F800000
    # so small a negative accumulator never vanishes, however far below the sum it lies
    assert _run(TR, [1.0], [1.0], -2.0 ** -126) == 0x3F7FFFFF


def test_special_truncation_of_the_accumulator():
    # the same case in GTR-FDPA: e_c = -30 < E - F - 1 = -25, so the accumulator's term is dropped
    assert _run(GTR, [1.0], [1.0], -2.0 ** -30, L=16) == 0x3F800000
    # e_c = -25 is the last exponent that is kept: RD_24(-2^-25) = -2^-24
    assert _run(GTR, [1.0], [1.0], -2.0 ** -25, L=16) == 0x3F7FFFFF
    assert _run(GTR, [1.0], [1.0], -2.0 ** -26, L=16) == 0x3F800000
    # TR-FDPA has no such rule
    assert _run(TR, [1.0], [1.0], -2.0 ** -26) == 0x3F7FFFFF


def test_product_sum_is_rounded_down_to_F2_bits():
    # products -64*1 and 2^-10*1: e_max = 6, T = -(1 - 2^-16).  c = 2^30 (1 + 2^-23): E = 30,
    # T 2^-24 = -(2^-24 - 2^-40), RD_31 -> -2^-24; S = 1 + 2^-23 - 2^-24 = 1 + 2^-24: a tie, to even: 2^30.
    # Without the rounding (or with truncation toward zero) S > 1 + 2^-24 and the result is the next float up.
    c = bits_f32(0x4E800001)
    assert _run(TR, [-64.0, 2.0 ** -10], [1.0, 1.0], c) == 0x4E800000
    assert _run(GTR, [-64.0, 2.0 ** -10], [1.0, 1.0], c, L=16) == 0x4E800000
    assert _run(TR.with_(c_mode=C_AFTER_EXACT), [-64.0, 2.0 ** -10], [1.0, 1.0], c) == 0x4E800001
    # F2 = 40 keeps the sum exact here
    assert _run(TR.with_(frac_bits2=40), [-64.0, 2.0 ** -10], [1.0, 1.0], c) == 0x4E800001


def test_even_odd_merge_rounds_down():
    # even products: 2^13 * 2^10 = 2^23 (e_even = 23, T_even = 1); odd products: -0.25 (e_odd = -2, T_odd = -1).
    # merge at e_max = 23: RD_24(-2^-25) = -2^-24, T = 1 - 2^-24, d = 2^23 - 0.5 (exactly a binary32 number)
    assert bits_f32(_run(GTR, [2.0 ** 13, -0.25], [2.0 ** 10, 1.0], 0.0, L=16)) == 2.0 ** 23 - 0.5
    # a positive small odd sum is rounded down to nothing
    assert bits_f32(_run(GTR, [2.0 ** 13, 0.25], [2.0 ** 10, 1.0], 0.0, L=16)) == 2.0 ** 23
    # the same two products in one fused group (TR-FDPA) are truncated toward zero at e_max instead
    assert bits_f32(_run(TR, [2.0 ** 13, -0.25], [2.0 ** 10, 1.0], 0.0)) == 2.0 ** 23
    # both in the even group (indices 0 and 2): truncated toward zero as well
    assert bits_f32(_run(GTR, [2.0 ** 13, 0.0, -0.25], [2.0 ** 10, 0.0, 1.0], 0.0, L=16)) == 2.0 ** 23


def test_groups_use_their_own_maximum_exponent():
    # odd group: 2^-12 and 2^-13 * (1 + 2^-10) ... kept to 24 bits below e_odd, not below e_even.
    # even: 2^12 (e = 12); odd: 2^-12 (e = -12).  T_odd = 1 at e_odd; merged at 12: 2^-24 survives exactly.
    d = _run(GTR, [2.0 ** 12, 2.0 ** -12], [1.0, 1.0], -(2.0 ** 12), L=16)
    assert bits_f32(d) == 2.0 ** -12
    # one place lower and the round-down takes it away
    d = _run(GTR, [2.0 ** 12, 2.0 ** -13], [1.0, 1.0], -(2.0 ** 12), L=16)
    assert d == 0


def test_product_overflow_is_an_infinity():
    p = TR.with_(group_len=2)
    big = bf16_bits(2.0 ** 64)
    # 2^64 * 2^64 = 2^128: the product itself overflows although the sum 2^128 - 2^127 would be finite
    a, b = [big, bf16_bits(-(2.0 ** 63))], [big, big]
    assert fdpa_group(p, a, b, 0, fm.BF16, fm.BF16) == 0x7F800000
    assert fdpa_group(p.with_(c_mode=C_IN_GROUP), a, b, 0, fm.BF16, fm.BF16) == f32_bits(2.0 ** 127)
    assert fdpa_group(p, [big, big], [bf16_bits(-(2.0 ** 64)), big], 0, fm.BF16, fm.BF16) == p.nan_bits
    assert fdpa_group(p, [bf16_bits(-(2.0 ** 64)), 0], [big, 0], 0, fm.BF16, fm.BF16) == 0xFF800000
    # just below the limit nothing overflows: (2^64 - 2^56)^2 < 2^128
    near = bf16_bits(2.0 ** 64 - 2.0 ** 56)
    d = fdpa_group(p, [near, 0], [near, 0], 0, fm.BF16, fm.BF16)
    assert d == f32_bits((2.0 ** 64 - 2.0 ** 56) ** 2)
    # a subnormal-times-large product whose unnormalised exponent sum is high but whose value is small
    assert fdpa_group(p, [0x0001, 0], [bf16_bits(2.0 ** 127), 0], 0, fm.BF16, fm.BF16) == f32_bits(2.0 ** -6)
    # GTR-FDPA on FP8 can never overflow (|a b| <= 57344^2 < 2^32)
    assert fdpa_group(GTR, [0x7B] * 16, [0x7B] * 16, 0, fm.E5M2, fm.E5M2) == f32_bits(16 * 57344.0 ** 2)


# ------------------------------------------------------------------ closed forms and order relations
@pytest.mark.parametrize("mode", [C_AFTER_RD, C_AFTER_RD_EVEN_ODD])
def test_wide_F_is_the_correctly_rounded_exact_result(mode):
    # with F and F2 wide enough no alignment loses a bit and both operations reduce to E-FDPA
    rng = np.random.default_rng(31 + mode)
    p = ModelParams(frac_bits=WIDE, frac_bits2=WIDE, c_mode=mode)
    for t in (fm.FP16, fm.E5M2, fm.E4M3):
        for _ in range(80):
            a = synth.random_bits(rng, 8, t).tolist()
            b = synth.random_bits(rng, 8, t).tolist()
            c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 90, 160)[0])
            if mode == C_AFTER_RD_EVEN_ODD:
                # the special truncation is part of the operation at any F; keep the accumulator above its threshold
                c = (c & 0x807FFFFF) | (140 << 23)
            assert fdpa_group(p, a, b, c, t, t) == e_fdpa(a, b, c, t, t)


@pytest.mark.parametrize("mode,L,t", [(C_AFTER_RD, 8, fm.FP16), (C_AFTER_RD, 8, fm.BF16),
                                      (C_AFTER_RD_EVEN_ODD, 16, fm.E5M2), (C_AFTER_RD_EVEN_ODD, 16, fm.E4M3)])
def test_round_down_brackets(mode, L, t):
    """Every rounding after the truncated product sums is downward and rho is monotonic, so
         d(a, b, c) <= d_no_RD(a, b, c) <= -d(-a, b, -c),
    where d_no_RD adds the same truncated sums and c exactly (for TR-FDPA that is c_mode C_AFTER_EXACT;
    for GTR-FDPA it is built here from the two group sums)."""
    rng = np.random.default_rng(77 + mode + t)
    p = ModelParams(group_len=L, frac_bits=24, frac_bits2=31, c_mode=mode)
    sign_in = 0x8000 if t in (fm.FP16, fm.BF16) else 0x80
    strict_lo = strict_hi = 0
    for trial in range(300):
        a = synth.narrow_exponent_bits(rng, L, t, 10, 20).tolist() if t != fm.E4M3 else synth.random_bits(rng, L, t).tolist()
        b = synth.narrow_exponent_bits(rng, L, t, 10, 20).tolist() if t != fm.E4M3 else synth.random_bits(rng, L, t).tolist()
        if t == fm.BF16:
            a = synth.narrow_exponent_bits(rng, L, t, 120, 135).tolist()
            b = synth.narrow_exponent_bits(rng, L, t, 120, 135).tolist()
        if t == fm.E4M3:
            a = [x if (x & 0x7F) != 0x7F else 0x38 for x in a]      # no NaN codes
            b = [x if (x & 0x7F) != 0x7F else 0x38 for x in b]
        base = 127 + (0 if t == fm.BF16 else (-10 if t != fm.E4M3 else 0))
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, base - 30, base + 12)[0])
        d = fdpa_group(p, a, b, c, t, t)
        d_mirror = fdpa_group(p, [x ^ sign_in for x in a], b, c ^ 0x80000000, t, t) ^ 0x80000000
        if mode == C_AFTER_RD:
            mid = fdpa_group(p.with_(c_mode=C_AFTER_EXACT), a, b, c, t, t)
            lo, m_, hi = (int(ordered_key(x)) for x in (d, mid, d_mirror))
            assert lo <= m_ <= hi, (trial, hex(d), hex(mid), hex(d_mirror))
        else:
            lo, hi = int(ordered_key(d)), int(ordered_key(d_mirror))
            assert lo <= hi
        strict_lo += lo < hi
    assert strict_lo > 10          # the bracket is not trivially tight: the rounding direction does matter


def test_loss_is_bounded_and_one_sided():
    # S 2^E lies below T 2^e_max + c by less than 2^(E - F2) + 2^(E - F)   (TR-FDPA, before rho)
    rng = np.random.default_rng(5)
    p = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
    q = p.with_(c_mode=C_AFTER_EXACT)
    for _ in range(200):
        a = synth.narrow_exponent_bits(rng, 8, fm.FP16, 8, 22).tolist()
        b = synth.narrow_exponent_bits(rng, 8, fm.FP16, 8, 22).tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 100, 150)[0])
        d, ref = fdpa_group(p, a, b, c, fm.FP16, fm.FP16), fdpa_group(q, a, b, c, fm.FP16, fm.FP16)
        x, y = Fraction(bits_f32(d)), Fraction(bits_f32(ref))
        da = [fm.decode(v, fm.FP16) for v in a]
        db = [fm.decode(v, fm.FP16) for v in b]
        E = max(max(u.exp + v.exp for u, v in zip(da, db)), fm.decode(c, fm.FP32).exp)
        ulp = Fraction(2) ** (max(E + 5, -126) - 23)       # |S| < 2^5 * 2^E: generous bound on one output ulp
        assert x <= y
        assert y - x <= Fraction(2) ** (E - 31) + Fraction(2) ** (E - 24) + 2 * ulp


def test_bias_toward_minus_infinity():
    """Sec. 6 (numerical bias): with A, B ~ 1000 N(0,1) in FP16, C ~ N(0,1) and K = 8 the error of the TR-FDPA
    result against the real value leans negative, while the same operation without the RD steps is centred."""
    rng = np.random.default_rng(2024)
    n = 40000
    A = (1000.0 * rng.standard_normal((n, 1, 8))).astype(np.float16).view(np.uint16)
    B = (1000.0 * rng.standard_normal((n, 1, 8))).astype(np.float16).view(np.uint16)
    Cf = rng.standard_normal((n, 1, 1)).astype(np.float32)
    C = Cf.view(np.uint32)
    real = (A.view(np.float16).astype(np.float64) * B.view(np.float16).astype(np.float64)).sum(axis=2)[:, :, None] + Cf
    d_rd = o2lib.emulate_mma(TR, A, B, C, fm.FP16, fm.FP16)[0].view(np.float32).astype(np.float64)
    d_ex = o2lib.emulate_mma(TR.with_(c_mode=C_AFTER_EXACT), A, B, C, fm.FP16, fm.FP16)[0].view(np.float32).astype(np.float64)
    delta_rd, delta_ex = (d_rd - real).ravel(), (d_ex - real).ravel()
    se = delta_ex.std() / np.sqrt(n)
    assert delta_rd.mean() < -6 * se
    assert abs(delta_ex.mean()) < 4 * se
    assert (delta_rd <= delta_ex).all() and (delta_rd < delta_ex).mean() > 0.05


# ------------------------------------------------------------------ the C form agrees with the rational form
@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2),
                                   (fm.E4M3, fm.E4M3), (fm.FP16, fm.BF16)])
def test_o2_equals_rational_oracle_tr_gtr(ta, tb):
    rng = np.random.default_rng(300 + 8 * ta + tb)
    for trial in range(16):
        mode = C_AFTER_RD if trial % 2 else C_AFTER_RD_EVEN_ODD
        L = int(rng.choice([2, 4, 8, 16, 0]))
        k = int(rng.choice([8, 16, 32])) if L == 0 else L * int(rng.integers(1, 4))
        F = int(rng.choice([0, 3, 13, 23, 24, 25, 31, 40]))
        F2 = min(int(rng.choice([0, 24, 31, 31, 31, 36, 48])), F + 40)     # the C form's stated limit
        p = ModelParams(group_len=L, frac_bits=F, frac_bits2=F2, c_mode=mode, out_round=int(rng.integers(0, 2)),
                        ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        nan_bits=0x7FFFFFFF if trial % 3 == 0 else 0x7FC00000)
        nb, m, n = 2, 3, 4
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        lo, hi = ((90, 165) if trial % 4 < 2 else (1, 254))
        if ta == fm.BF16 and tb == fm.BF16 and trial % 4 < 2:
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 100, 150)
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 100, 150)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, lo, hi)
        if trial % 5 == 0:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.02)
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.02)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.05)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (p, np.argwhere(got != want)[:3])


def test_o2_accumulator_exponent_sweep():
    # the accumulator's exponent swept across every alignment distance, both signs, extreme significands
    for mode, L in ((C_AFTER_RD, 2), (C_AFTER_RD_EVEN_ODD, 2)):
        p = ModelParams(group_len=L, frac_bits=24, frac_bits2=31, c_mode=mode)
        A = np.array([[[fp16_bits(1.5), fp16_bits(-2.0 ** -8 * 1.0009765625)]]], dtype=np.uint16)
        B = np.array([[[fp16_bits(1.25), fp16_bits(1.0)]]], dtype=np.uint16)
        for ec in range(127 - 70, 127 + 45):
            for csig in (0, 1, 0x7FFFFF, 0x400000, 0x2AAAAA):
                for sgn in (0, 1):
                    C = np.array([[[(sgn << 31) | (ec << 23) | csig]]], dtype=np.uint32)
                    for rho in (RNE, RZ):
                        q = p.with_(out_round=rho)
                        assert np.array_equal(o2lib.emulate_mma(q, A, B, C, fm.FP16, fm.FP16)[0],
                                              emulate_mma(q, A, B, C, fm.FP16, fm.FP16)), (mode, ec, csig, sgn, rho)


def test_o2_rejects_odd_group_for_gtr():
    p = ModelParams(group_len=3, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD_EVEN_ODD)
    A = np.zeros((1, 1, 3), dtype=np.uint16)
    with pytest.raises(ValueError):
        o2lib.emulate_mma(p, A, A, np.zeros((1, 1, 1), dtype=np.uint32), fm.FP16, fm.FP16)
    with pytest.raises(ValueError):
        emulate_mma(p, A, A, np.zeros((1, 1, 1), dtype=np.uint32), fm.FP16, fm.FP16)


# ------------------------------------------------------------------ variations beyond the paper's two algorithms
from oracle.fdpa import SPLIT_NONE, SPLIT_EVEN_ODD, SPLIT_HALVES


def test_gtr_by_name_is_tr_with_even_odd_split_and_special_truncation():
    rng = np.random.default_rng(8)
    q = GTR.with_(c_mode=C_AFTER_RD, split=SPLIT_EVEN_ODD, acc_special_truncation=True)
    A = synth.random_bits(rng, (2, 4, 32), fm.E4M3)
    B = synth.random_bits(rng, (2, 4, 32), fm.E5M2)
    C = synth.narrow_exponent_bits(rng, (2, 4, 4), fm.FP32, 100, 150)
    assert np.array_equal(emulate_mma(GTR, A, B, C, fm.E4M3, fm.E5M2), emulate_mma(q, A, B, C, fm.E4M3, fm.E5M2))
    assert np.array_equal(o2lib.emulate_mma(GTR, A, B, C, fm.E4M3, fm.E5M2)[0], o2lib.emulate_mma(q, A, B, C, fm.E4M3, fm.E5M2)[0])


def test_halves_split():
    # first half: 2^13 * 2^10 (e = 23); second half: -0.25.  Same arithmetic as the even/odd case above, other partition.
    p = GTR.with_(c_mode=C_AFTER_RD, split=SPLIT_HALVES, acc_special_truncation=True)
    a = [2.0 ** 13] + [0.0] * 7 + [-0.25] + [0.0] * 7
    b = [2.0 ** 10] + [0.0] * 7 + [1.0] + [0.0] * 7
    assert bits_f32(_run(p, a, b, 0.0, L=16)) == 2.0 ** 23 - 0.5
    # both in the first half: truncated toward zero at the shared maximum
    assert bits_f32(_run(p, [2.0 ** 13, -0.25], [2.0 ** 10, 1.0], 0.0, L=16)) == 2.0 ** 23


def test_separate_precisions():
    # F = 13 for the products, F_m = F_c = 24: a product 2^-14 below the largest one of its half is dropped ...
    p = ModelParams(group_len=16, frac_bits=13, frac_bits_merge=24, frac_bits_acc=24, frac_bits2=31, c_mode=C_AFTER_RD, split=SPLIT_HALVES)
    assert bits_f32(_run(p, [1.0, 2.0 ** -14], [1.0, 1.0], 0.0, L=16)) == 1.0
    assert bits_f32(_run(p, [1.0, 2.0 ** -13], [1.0, 1.0], 0.0, L=16)) == 1.0 + 2.0 ** -13
    # ... but in the other half it is aligned at its own exponent and survives the merge at 24 bits
    a = [1.0] + [0.0] * 7 + [2.0 ** -14] + [0.0] * 7
    assert bits_f32(_run(p, a, [1.0] * 16, 0.0, L=16)) == 1.0 + 2.0 ** -14
    # the accumulator keeps 24 bits: 1 + 2^-23 survives next to a product of 1
    assert bits_f32(_run(p, [1.0], [1.0], 2.0 ** -23, L=16)) == 1.0 + 2.0 ** -23
    # with F_c = F = 13 it does not
    assert bits_f32(_run(p.with_(frac_bits_acc=0), [1.0], [1.0], 2.0 ** -23, L=16)) == 1.0


def test_skip_zero_terms():
    # 0 * 2^15 carries the exponent (1 - 15) + 15 = 1 into e_max in the literal reading; the live product
    # (1 + 2^-10)^2 2^-8 = 2^-8 + 2^-17 + 2^-28 then loses its last bit below the unit 2^(1-24)
    a, b = [0.0, 1.0 + 2.0 ** -10], [2.0 ** 15, 2.0 ** -8 * (1.0 + 2.0 ** -10)]
    exact = (1 + 2.0 ** -10) ** 2 * 2.0 ** -8
    assert bits_f32(_run(TR, a, b, 0.0)) == 2.0 ** -8 + 2.0 ** -17
    assert bits_f32(_run(TR.with_(skip_zero_terms=True), a, b, 0.0)) == exact          # 21 significant bits: a binary32 number
    # all products zero: the accumulator passes through, also a negative tiny one (no round-down at a foreign exponent)
    for c in (-2.0 ** -140, 2.0 ** -140, -1.5, 0.0):
        assert _run(TR.with_(skip_zero_terms=True), [0.0], [3.0], c) == f32_bits(c)
    assert _run(TR, [0.0], [3.0], -2.0 ** -140) == f32_bits(-2.0 ** -37)               # literal: e_max = -14 + 1, RD_24 of c is -2^(-13-24)
    # a zero accumulator still sets E (only products are skipped): it has the exponent of the subnormals.  Products
    # 2^-150 + 2^-151 with F2 = 24: the sum is rounded down at E = -126 to a multiple of 2^-150, a tie of the subnormal
    # grid that goes to 0, with and without the switch (E = e_max would keep 1.5 * 2^-150, which rounds up to 2^-149)
    p = ModelParams(group_len=2, frac_bits=24, frac_bits2=24, c_mode=C_AFTER_RD)
    a2, b2 = [bf16_bits(2.0 ** -75)] * 2, [bf16_bits(2.0 ** -75), bf16_bits(2.0 ** -76)]
    assert fdpa_group(p, a2, b2, 0, fm.BF16, fm.BF16) == 0
    assert fdpa_group(p.with_(skip_zero_terms=True), a2, b2, 0, fm.BF16, fm.BF16) == 0
    assert fdpa_group(p.with_(skip_zero_terms=True, frac_bits2=25), a2, b2, 0, fm.BF16, fm.BF16) == 1
    # exact zero stays +0.0 in every mode
    for mode in (C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD):
        q = ModelParams(group_len=2, frac_bits=24, frac_bits2=31, c_mode=mode, skip_zero_terms=True)
        assert fdpa_group(q, [0, 0x8000], [0x3C00, 0x3C00], 0x80000000, fm.FP16, fm.FP16) == 0


def test_f2_below_the_leading_bit():
    # c = 2^30 (2 - 2^-23); products 128, 128 and 0.5 (e_max = 7): in units of 2^30, T = 2^-22 + 2^-31 and
    # S = 2 + 2^-23 + 2^-31.  S has its leading bit one place above 2^E.  Binary32 spacing there is 2^-22, so
    # 2 + 2^-23 is a tie.  Counted below 2^E the 2^-31 bit is kept: above the tie, rounds up.  Counted below the
    # leading bit the unit is 2^-30: the bit is dropped and the tie goes to the even neighbour 2.
    c = bits_f32(0x4EFFFFFF)
    assert _run(TR, [128.0, 128.0, 0.5], [1.0, 1.0, 1.0], c) == 0x4F000001
    assert _run(TR.with_(f2_at_leading_bit=True), [128.0, 128.0, 0.5], [1.0, 1.0, 1.0], c) == 0x4F000000
    # one place of cancellation keeps one bit more: c = -2^30, products 2^29 - 2^6 ... : S = -(1/2 + 2^-24 ...)
    # c = -2^30 (1 + 2^-23)... simpler: c = 2^30, products -(2^29) and -(2^-2 + 2^-3): in units of 2^30,
    # S = 1/2 - 2^-32 - 2^-33.  Below 2^E: RD_31 of T = -(1/2 + 2^-32 + 2^-33) gives -(1/2 + 2^-31), S = 1/2 - 2^-31.
    # Below the leading bit (2^-2 after the borrow... S < 1/2, leading bit 2^-2): unit 2^-33, S is kept exactly.
    # Both are below 1/2 by far less than half a binary32 place (2^-26): the two anchors agree on 0x4DFFFFFF? No:
    # 1/2 - 2^-31 and 1/2 - 2^-32 - 2^-33 both round to 1/2 (spacing below 1/2 is 2^-25).  Agreement is the point:
    d0 = _run(TR, [-(2.0 ** 15), -0.25, -0.125], [2.0 ** 14, 1.0, 1.0], 2.0 ** 30)
    d1 = _run(TR.with_(f2_at_leading_bit=True), [-(2.0 ** 15), -0.25, -0.125], [2.0 ** 14, 1.0, 1.0], 2.0 ** 30)
    assert d0 == d1 == f32_bits(2.0 ** 29)


def test_zero_result_positive():
    p = ModelParams(group_len=1, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
    a, b = [bf16_bits(-(2.0 ** -80))], [bf16_bits(2.0 ** -80)]
    assert fdpa_group(p, a, b, 0, fm.BF16, fm.BF16) == 0x80000000
    assert fdpa_group(p.with_(zero_result_positive=True), a, b, 0, fm.BF16, fm.BF16) == 0
    q = ModelParams(group_len=1, frac_bits=24, ftz_out=True, zero_result_positive=True)
    assert fdpa_group(q, [bf16_bits(-(2.0 ** -70))], [bf16_bits(2.0 ** -70)], 0, fm.BF16, fm.BF16) == 0


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3), (fm.E4M3, fm.BF16)])
def test_o2_equals_rational_oracle_variations(ta, tb):
    rng = np.random.default_rng(700 + 8 * ta + tb)
    for trial in range(24):
        L = int(rng.choice([2, 4, 8, 16, 0]))
        k = int(rng.choice([8, 16, 32])) if L == 0 else L * int(rng.integers(1, 3))
        F = int(rng.choice([0, 5, 13, 24, 25, 40]))
        p = ModelParams(group_len=L, frac_bits=F, frac_bits2=int(rng.choice([max(F - 3, 0), 24, 31, 36, min(F + 40, 48)])),
                        c_mode=int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD, C_AFTER_RD])),
                        out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)))
        if p.c_mode == C_AFTER_RD:
            p = p.with_(split=int(rng.integers(0, 4 if (L or k) % 4 == 0 else 3)), acc_special_truncation=bool(rng.integers(0, 2)),
                        frac_bits_merge=int(rng.choice([0, 13, 24, 31])), frac_bits_acc=int(rng.choice([0, 13, 24, 30])),
                        f2_at_leading_bit=bool(rng.integers(0, 2)),
                        sum_drop_distance=int(rng.choice([0, 0, 5, 20, 28])))
            fc = p.frac_bits_acc or p.frac_bits
            if p.frac_bits2 > fc + 40:
                p = p.with_(frac_bits2=fc + 40)
        else:
            p = p.with_(frac_bits2=0)
            if p.c_mode == C_AFTER_EXACT and p.frac_bits > 32:
                p = p.with_(frac_bits=32)
        nb, m, n = 2, 3, 4
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        # plenty of zeros so that skip_zero_terms matters, whole zero rows included
        A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.2)
        A[0, 0, :] = 0
        lo, hi = ((90, 165) if trial % 4 < 2 else (1, 254))
        if ta == fm.BF16 and tb == fm.BF16 and trial % 4 < 2:
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 100, 150)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, lo, hi)
        C[0, 0, 0] = 0
        C[0, 0, 1] = 0x80000000
        if trial % 5 == 0:
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.02)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.05)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (p, np.argwhere(got != want)[:3])


def test_sum_drop_distance():
    # eight products of 1.5 * 1.5 (e_max = 0, T = 18) next to c = 2^28: in units of binary32 places of c (2^5) T is
    # 0.5625 places and rounds c up by one; with the drop at distance 28 the sum is ignored altogether
    p = TR.with_(sum_drop_distance=28)
    a = [1.5] * 8
    assert _run(TR, a, a, 2.0 ** 28) == f32_bits(2.0 ** 28) + 1
    assert _run(p, a, a, 2.0 ** 28) == f32_bits(2.0 ** 28)
    assert _run(p, a, a, 2.0 ** 27) == f32_bits(2.0 ** 27 + 16)       # distance 27: kept (18 = 1.125 places of 16)
    assert _run(p, a, a, -(2.0 ** 28)) == f32_bits(-(2.0 ** 28))


def test_split_into_quarters():
    # four sub-groups of two products each (L = 8), F = 4 inside a sub-group, 24 bits across.  Products (value, by
    # construction): quarter 0: 1 and 2^-5 (the small one lies below the unit 2^-4 of its own quarter: cut);
    # quarter 1: 2^-5 alone with 0: kept, its quarter's maximum is its own exponent; merged at the overall maximum
    # with 24 bits it survives: 1 + 2^-5.  As halves of four the small product of quarter 1 would share the maximum
    # 2^0 of quarter 0 and be cut as well: 1.
    from oracle.fdpa import SPLIT_QUARTERS, SPLIT_HALVES
    p = ModelParams(group_len=8, frac_bits=4, frac_bits2=31, c_mode=C_AFTER_RD, frac_bits_merge=24, frac_bits_acc=24,
                    split=SPLIT_QUARTERS, skip_zero_terms=True)
    a = [1.0, 2.0 ** -5, 2.0 ** -5, 0.0, 0.0, 0.0, 0.0, 0.0]
    b = [1.0] * 8
    assert bits_f32(_run(p, a, b, 0.0, L=8)) == 1.0 + 2.0 ** -5
    assert bits_f32(_run(p.with_(split=SPLIT_HALVES), a, b, 0.0, L=8)) == 1.0
    # quarters with one product each are a plain sum rounded down at 24 bits: every term kept
    q = p.with_(group_len=4)
    assert bits_f32(_run(q, [1.0, 2.0 ** -5, 2.0 ** -9, 2.0 ** -13], [1.0] * 4, 0.0, L=4)) == 1.0 + 2.0 ** -5 + 2.0 ** -9 + 2.0 ** -13
    # the merge rounds every quarter down: -2^-30 in a quarter of its own next to 1 becomes -2^-24, and the sum
    # 1 - 2^-24 is a binary32 number
    assert bits_f32(_run(q, [1.0, -2.0 ** -12, 0.0, 0.0], [2.0 ** 0, 2.0 ** -14], 0.0, L=4)) == 1.0 - 2.0 ** -24
    with pytest.raises(ValueError):
        _run(p.with_(group_len=6), [1.0] * 6, [1.0] * 6, 0.0, L=6)
