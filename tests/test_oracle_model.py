"""Pins for the oracle's model (oracle/fdpa.py) against what the paper prints and what
the mathematics fixes.  Each test names the passage it checks."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import formats as fm
from oracle.fdpa import (ModelParams, emulate_element, fdpa_group, e_fdpa, exact_value, exact_width,
                         C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, NVIDIA_NAN)
from oracle.rounding import RNE, RZ, rne_fp32
from helpers import f32_bits, bits_f32, ENCODERS, fp16_bits, bf16_bits
from paper_2511_10909_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
FMT_ID = {"fp16": fm.FP16, "bf16": fm.BF16, "e5m2": fm.E5M2, "tf32": fm.TF32}
WIDE = 700   # more fractional bits than any pair of supported operands can span


def _rows(name):
    with open(os.path.join(GOLD, name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- Sec. 5 worked example
@pytest.mark.parametrize("row", _rows("table_d00.txt"), ids=lambda r: r[0])
def test_table_d00(row):
    label, typ, lmax, F, rho, want = row
    enc, t = ENCODERS[typ], FMT_ID[typ]
    K = 32
    a = [enc(-2.0 ** 13), enc(-0.5), enc(-0.25), enc(-0.125)] + [0] * (K - 4)
    b = [enc(2.0 ** 10), enc(1.0), enc(1.0), enc(1.0)] + [0] * (K - 4)
    c = f32_bits(2.0 ** 23)
    p = ModelParams(group_len=int(lmax), frac_bits=WIDE if F == "exact" else (24 if F == "-" else int(F)),
                    out_round=RZ if rho == "RZ" else RNE)
    if rho in ("TR", "GTR"):
        p = p.with_(frac_bits2=31, c_mode=C_AFTER_RD if rho == "TR" else C_AFTER_RD_EVEN_ODD)
    if rho == "ADDMUL":
        p = ModelParams(group_len=int(lmax), family=1)
    if rho == "FMA":
        p = ModelParams(group_len=1, frac_bits=24, c_mode=C_AFTER_EXACT)
    got = emulate_element(p, a, b, c, t, t)
    assert bits_f32(got) == float(want)
    if float(want) == 0.0:
        assert got == 0          # +0.0


def test_table_d00_derived_wider_F():
    # not printed: with F >= 26 nothing is truncated and the exact -0.875 appears
    a = [fp16_bits(-2.0 ** 13), fp16_bits(-0.5), fp16_bits(-0.25), fp16_bits(-0.125)]
    b = [fp16_bits(2.0 ** 10), fp16_bits(1.0), fp16_bits(1.0), fp16_bits(1.0)]
    for F in (26, 27, 40):
        got = emulate_element(ModelParams(group_len=4, frac_bits=F), a, b, f32_bits(2.0 ** 23), fm.FP16, fm.FP16)
        assert bits_f32(got) == -0.875


# ---------------------------------------------------------------- Sec. 3.1 Step 2, Fig. "summation trees"
def _trees():
    out, cur = {}, None
    for r in _rows("fig2_trees.txt"):
        if r[0] == "tree":
            cur = out.setdefault(r[1], [])
        else:
            cur.append([int(x) for x in r])
    return out


def _probe(p, i, j, eu_half, t, enc):
    """d^(i,j)/v for K=4: p_i = U, p_j = -U, others v = 1, with U = 2^(2*eu_half)."""
    K = 4
    a, b = [enc(1.0)] * K, [enc(1.0)] * K
    c = f32_bits(1.0)
    U = 2.0 ** eu_half
    for idx, sgn in ((i, 1.0), (j, -1.0)):
        if idx == K:
            c = f32_bits(sgn * U * U)
        else:
            a = a[:idx] + [enc(sgn * U)] + a[idx + 1:]
            b = b[:idx] + [enc(U)] + b[idx + 1:]
    d = bits_f32(emulate_element(p, a, b, c, t, t))
    assert d == int(d) and 0 <= d < K
    return int(d)


@pytest.mark.parametrize("tree,params,eu_half", [
    # chain of FMAs == chained FDPA with L = 1 and no truncation
    ("a_chain_of_binary_sums", ModelParams(group_len=1, frac_bits=WIDE), 15),
    # CDNA1 bf16: E-FDPA with L = 2, chained
    ("c_nonswamped_3term_fused", ModelParams(group_len=2, frac_bits=WIDE), 15),
    # one truncated 5-term fused sum, e_u - e_v = 30 > F
    ("d_swamped_5term_fused", ModelParams(group_len=4, frac_bits=24, out_round=RZ), 15),
])
def test_fig2_trees(tree, params, eu_half):
    table = _trees()[tree]
    for t, enc in ((fm.BF16, bf16_bits), (fm.FP16, fp16_bits)):
        if t == fm.FP16 and eu_half > 15:
            continue
        for i in range(4):
            for jj, want in enumerate(table[i]):
                j = i + 1 + jj
                assert _probe(params, i, j, eu_half, t, enc) == want, (tree, i, j)


def test_fig2_footnote_walkthrough():
    # footnote of Sec. 3.1 Step 2: chain, i=0, j=1: c+a0b0 = v+U = U; U-U = 0; 0+v = v; v+v = 2v
    p = ModelParams(group_len=1, frac_bits=WIDE)
    assert _probe(p, 0, 1, 15, fm.BF16, bf16_bits) == 2


def test_fig2_derived_chained_narrow():
    # not printed: chained L=2 with F=24 and U = 2^40 (bf16), v = 1
    p = ModelParams(group_len=2, frac_bits=24)
    want = [[2, 0, 0, 2], [0, 0, 2], [0, 0], [0]]
    for i in range(4):
        for jj, w in enumerate(want[i]):
            assert _probe(p, i, i + 1 + jj, 20, fm.BF16, bf16_bits) == w


# ---------------------------------------------------------------- Alg. "E-FDPA" as closed form
@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2),
                                   (fm.E5M2, fm.E4M3), (fm.FP16, fm.E4M3), (fm.BF16, fm.FP16)])
def test_wide_F_equals_correctly_rounded_exact(ta, tb):
    rng = np.random.default_rng(10 + ta * 8 + tb)
    for _ in range(150):
        L = int(rng.integers(1, 9))
        a = synth.random_bits(rng, L, ta).tolist()
        b = synth.random_bits(rng, L, tb).tolist()
        c = int(synth.random_bits(rng, 1, fm.FP32)[0])
        need = exact_width(a, b, c, ta, tb)
        assert need <= WIDE
        for F in (need, WIDE):
            got = fdpa_group(ModelParams(frac_bits=F), a, b, c, ta, tb)
            want = rne_fp32(exact_value(a, b, c, ta, tb))
            assert got == want == e_fdpa(a, b, c, ta, tb)


def test_exact_sum_against_libm_when_double_is_exact():
    # exponent fields restricted so that c + sum a_k b_k is exact in binary64:
    # math.fsum of exact double products is then the exact value, and the hardware
    # double->float conversion is a single correct rounding, independent of rounding.py
    import math
    rng = np.random.default_rng(11)
    for _ in range(400):
        L = int(rng.integers(1, 17))
        a = synth.narrow_exponent_bits(rng, L, fm.FP16, 10, 20)
        b = synth.narrow_exponent_bits(rng, L, fm.FP16, 10, 20)
        c = synth.narrow_exponent_bits(rng, 1, fm.FP32, 120, 135)
        av = a.view(np.float16).astype(np.float64)
        bv = b.view(np.float16).astype(np.float64)
        cv = float(c.view(np.float32)[0])
        exact = math.fsum([cv] + [float(x) * float(y) for x, y in zip(av, bv)])
        assert Fraction(exact) == exact_value(a.tolist(), b.tolist(), int(c[0]), fm.FP16, fm.FP16)
        got = fdpa_group(ModelParams(frac_bits=WIDE), a.tolist(), b.tolist(), int(c[0]), fm.FP16, fm.FP16)
        assert got == f32_bits(exact) or (exact == 0 and got == 0)


def test_chain_is_chain_of_rounded_groups_not_one_exact_dot():
    # Alg. "Phi_FDPA": each group's result is rounded before it feeds the next
    a = [bf16_bits(1.0), bf16_bits(2.0 ** -30), bf16_bits(2.0 ** -30), bf16_bits(-1.0)]
    b = [bf16_bits(1.0)] * 4
    chained = emulate_element(ModelParams(group_len=2, frac_bits=WIDE), a, b, 0, fm.BF16, fm.BF16)
    fused = emulate_element(ModelParams(group_len=0, frac_bits=WIDE), a, b, 0, fm.BF16, fm.BF16)
    assert bits_f32(chained) == 2.0 ** -30                # group 1: 1 + 2^-30 rounds to 1; group 2: 1 + 2^-30 - 1 exactly
    assert bits_f32(fused) == 2.0 ** -29
    a2 = [bf16_bits(1.0), bf16_bits(2.0 ** -30), bf16_bits(-1.0), bf16_bits(2.0 ** -30)]
    chained2 = emulate_element(ModelParams(group_len=2, frac_bits=WIDE), a2, b, 0, fm.BF16, fm.BF16)
    assert bits_f32(chained2) == 2.0 ** -30               # first group rounds to 1, second: 1 - 1 + 2^-30


# ---------------------------------------------------------------- brute force, FP8, k = 1
@pytest.mark.parametrize("ta,tb,tda,tdb", [
    (fm.E4M3, fm.E4M3, torch.float8_e4m3fn, torch.float8_e4m3fn),
    (fm.E4M3, fm.E5M2, torch.float8_e4m3fn, torch.float8_e5m2),
    (fm.E5M2, fm.E4M3, torch.float8_e5m2, torch.float8_e4m3fn),
    (fm.E5M2, fm.E5M2, torch.float8_e5m2, torch.float8_e5m2)])
def test_all_fp8_pairs_k1(ta, tb, tda, tdb):
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    va = codes.view(tda).to(torch.float64).numpy()
    vb = codes.view(tdb).to(torch.float64).numpy()
    ma, mb = fm.FORMATS[ta].mbits, fm.FORMATS[tb].mbits
    wide = ModelParams(frac_bits=80)
    narrow_F = 3
    narrow = ModelParams(frac_bits=narrow_F, out_round=RZ)
    for x in range(256):
        for y in range(256):
            px, py = va[x], vb[y]
            if not (np.isfinite(px) and np.isfinite(py)):
                continue
            prod = float(px) * float(py)                   # exact: at most 8 significant bits
            got = fdpa_group(wide, [x], [y], 0, ta, tb)
            assert got == (0 if prod == 0 else f32_bits(prod)), (x, y)
            # narrow F: one number truncated (magnitude) at 2^(e_max - F), e_max = max(Exp a + Exp b, Exp c = -126)
            e = fm.decode(x, ta).exp + fm.decode(y, tb).exp
            q = 2.0 ** (e - narrow_F)
            want = np.trunc(prod / q) * q
            got = fdpa_group(narrow, [x], [y], 0, ta, tb)
            assert bits_f32(got) == want, (x, y)


def test_k1_with_accumulator_is_fma():
    # one product plus c with wide F is the IEEE fused multiply-add; checked through binary64
    # (fp16*fp16 + fp32 with close exponents is exact in a double)
    rng = np.random.default_rng(12)
    for _ in range(2000):
        a = synth.narrow_exponent_bits(rng, 1, fm.FP16, 8, 22)
        b = synth.narrow_exponent_bits(rng, 1, fm.FP16, 8, 22)
        c = synth.narrow_exponent_bits(rng, 1, fm.FP32, 115, 135)
        exact = float(a.view(np.float16)[0]) * float(b.view(np.float16)[0]) + float(c.view(np.float32)[0])
        got = fdpa_group(ModelParams(frac_bits=WIDE), [int(a[0])], [int(b[0])], int(c[0]), fm.FP16, fm.FP16)
        assert got == (0 if exact == 0 else f32_bits(exact))


# ---------------------------------------------------------------- Sec. 6.1 error bounds
@pytest.mark.parametrize("F,L,rho", [(13, 16, RZ), (24, 8, RNE), (24, 8, RZ), (14, 32, RNE), (27, 16, RNE)])
def test_error_bound(F, L, rho):
    # |D - exact| <= (L+1) 2^(e_max - F) + {0.5, 1} ulp(D)   (Table "Sources and upper bounds")
    rng = np.random.default_rng(13 + F + L)
    ta = tb = fm.FP16
    p = ModelParams(frac_bits=F, out_round=rho)
    for _ in range(150):
        a = synth.random_bits(rng, L, ta).tolist()
        b = synth.random_bits(rng, L, tb).tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 90, 160)[0])
        d = fdpa_group(p, a, b, c, ta, tb)
        e_max = max([fm.decode(x, ta).exp + fm.decode(y, tb).exp for x, y in zip(a, b)] + [fm.decode(c, fm.FP32).exp])
        ulp = Fraction(2) ** (max((d >> 23) & 0xFF, 1) - 127 - 23)
        bound = (L + 1) * Fraction(2) ** (e_max - F) + (Fraction(1, 2) if rho == RNE else 1) * ulp
        assert abs(Fraction(bits_f32(d)) - exact_value(a, b, c, ta, tb)) <= bound


def test_truncation_is_toward_zero_per_term():
    # two negative terms each just below one unit of 2^(e_max - F) vanish separately
    # (RZ on each aligned term), they are not summed first
    a = [fp16_bits(1.0), fp16_bits(-(2.0 ** -4) * 1.5), fp16_bits(-(2.0 ** -4) * 1.5)]
    b = [fp16_bits(1.0)] * 3
    # F = 3: unit 2^-3; each small term is 0.75 units -> 0 ; their sum would be 1.5 units
    d = fdpa_group(ModelParams(frac_bits=3), a, b, 0, fm.FP16, fm.FP16)
    assert bits_f32(d) == 1.0
    a[1] = a[2] = fp16_bits((2.0 ** -4) * 1.5)
    d = fdpa_group(ModelParams(frac_bits=3), a, b, 0, fm.FP16, fm.FP16)
    assert bits_f32(d) == 1.0
    # and a single negative term of 1.75 units truncates to -1 unit (toward zero), not -2 (down)
    a = [fp16_bits(1.0), fp16_bits(-(2.0 ** -3) * 1.75)]
    d = fdpa_group(ModelParams(frac_bits=3), a, [fp16_bits(1.0)] * 2, 0, fm.FP16, fm.FP16)
    assert bits_f32(d) == 1.0 - 0.125


def test_emax_includes_accumulator_and_zero_products():
    one = fp16_bits(1.0)
    # accumulator sets e_max: product 2^-20 is below 2^(0 - 8) and vanishes
    d = fdpa_group(ModelParams(frac_bits=8), [fp16_bits(2.0 ** -10)], [fp16_bits(2.0 ** -10)], f32_bits(1.0), fm.FP16, fm.FP16)
    assert bits_f32(d) == 1.0
    # with C_AFTER_EXACT the accumulator is outside the truncated sum and the product survives
    d = fdpa_group(ModelParams(frac_bits=8, c_mode=C_AFTER_EXACT), [fp16_bits(2.0 ** -10)], [fp16_bits(2.0 ** -10)],
                   f32_bits(1.0), fm.FP16, fm.FP16)
    assert Fraction(bits_f32(d)) == 1 + Fraction(1, 1 << 20)
    # literal reading: a zero operand keeps Exp = 1 - bias, so 0 * 2^15 has e = -14 + 15 = 1 and
    # raises e_max above the product 2^-14 * 2^-10 ... (e = -24): with F = 20 the unit is 2^(1-20)
    a = [0, fp16_bits(2.0 ** -14)]
    b = [fp16_bits(2.0 ** 15), fp16_bits(2.0 ** -10)]
    d = fdpa_group(ModelParams(frac_bits=20), a, b, 0, fm.FP16, fm.FP16)
    assert d == 0
    d = fdpa_group(ModelParams(frac_bits=20), a[1:], b[1:], 0, fm.FP16, fm.FP16)
    assert bits_f32(d) == 2.0 ** -24


# ---------------------------------------------------------------- Sec. 6.2 symmetry
@pytest.mark.parametrize("rho", [RNE, RZ])
def test_sign_symmetry(rho):
    # RZ alignment with RNE/RZ output is symmetric: Phi(-A, B, -C) = -Phi(A, B, C)
    # (bitwise except that an exact-zero result is +0.0 on both sides)
    rng = np.random.default_rng(14)
    p = ModelParams(group_len=4, frac_bits=12, out_round=rho)
    for _ in range(300):
        a = synth.random_bits(rng, 8, fm.FP16)
        b = synth.random_bits(rng, 8, fm.FP16)
        c = synth.narrow_exponent_bits(rng, 1, fm.FP32, 100, 150)
        d1 = emulate_element(p, a.tolist(), b.tolist(), int(c[0]), fm.FP16, fm.FP16)
        d2 = emulate_element(p, (a ^ 0x8000).tolist(), b.tolist(), int(c[0]) ^ 0x80000000, fm.FP16, fm.FP16)
        if d1 & 0x7FFFFFFF:
            assert d2 == d1 ^ 0x80000000
        else:
            assert d2 & 0x7FFFFFFF == 0


# ---------------------------------------------------------------- Sec. 4.2 special values
def test_special_values():
    p = ModelParams(frac_bits=24)
    one, inf, ninf, nan, zero = fp16_bits(1.0), 0x7C00, 0xFC00, 0x7E00, 0
    f = lambda a, b, c, pp=p: fdpa_group(pp, a, b, c, fm.FP16, fm.FP16)
    assert f([nan, one], [one, one], 0) == 0x7FC00000                 # NaN * x
    assert f([nan, one], [zero, one], 0) == 0x7FC00000                # NaN * 0
    assert f([one], [one], 0x7FC12345) == 0x7FC00000                  # NaN + x, canonical encoding
    assert f([one], [one], 0x7FC12345, p.with_(nan_bits=NVIDIA_NAN)) == 0x7FFFFFFF
    assert f([inf, one], [one, one], f32_bits(5.0)) == 0x7F800000     # inf + y
    assert f([inf, one], [fp16_bits(-2.0), one], 0) == 0xFF800000     # inf * z = inf * sign(z)
    assert f([ninf], [fp16_bits(-2.0)], 0) == 0x7F800000
    assert f([inf], [zero], 0) == 0x7FC00000                          # inf * 0
    assert f([inf], [0x8000], 0) == 0x7FC00000
    assert f([inf, ninf], [one, one], 0) == 0x7FC00000                # inf - inf among products
    assert f([inf], [one], 0xFF800000) == 0x7FC00000                  # inf (product) - inf (c)
    assert f([one], [one], 0xFF800000) == 0xFF800000
    assert f([inf], [0x0001], 0) == 0x7F800000                        # inf * subnormal
    assert f([inf], [0x0001], 0, p.with_(ftz_in=True)) == 0x7FC00000  # flushed first: inf * 0
    # E4M3 has a NaN but no infinity
    assert fdpa_group(p, [0x7F], [0x38], 0, fm.E4M3, fm.E4M3) == 0x7FC00000
    assert bits_f32(fdpa_group(p, [0x7E], [0x38], 0, fm.E4M3, fm.E4M3)) == 448.0
    # chains carry specials forward
    assert emulate_element(p.with_(group_len=1), [inf, one, one], [one] * 3, 0, fm.FP16, fm.FP16) == 0x7F800000
    assert emulate_element(p.with_(group_len=1), [inf, ninf, one], [one] * 3, 0, fm.FP16, fm.FP16) == 0x7FC00000


def test_output_overflow():
    big = 0x7F7FFFFF
    a, b = [bf16_bits(2.0 ** 100)], [bf16_bits(2.0 ** 27)]
    assert fdpa_group(ModelParams(frac_bits=24), a, b, big, fm.BF16, fm.BF16) == 0x7F800000
    assert fdpa_group(ModelParams(frac_bits=24, out_round=RZ), a, b, big, fm.BF16, fm.BF16) == 0x7F7FFFFF
    a[0] ^= 0x8000
    assert fdpa_group(ModelParams(frac_bits=24, out_round=RZ), a, b, big ^ 0x80000000, fm.BF16, fm.BF16) == 0xFF7FFFFF


# ---------------------------------------------------------------- flush rules
def test_input_flush_to_positive_zero():
    # Alg. "Phi_FTZ-AddMul": A, B and C subnormals become +0.0 before anything else
    sub16, one = 0x83FF, fp16_bits(1.0)
    p = ModelParams(frac_bits=40)
    assert fdpa_group(p, [sub16], [one], 0, fm.FP16, fm.FP16) != 0
    assert fdpa_group(p.with_(ftz_in=True), [sub16], [one], 0, fm.FP16, fm.FP16) == 0
    assert fdpa_group(p.with_(ftz_in=True), [one], [sub16], 0, fm.FP16, fm.FP16) == 0
    csub = 0x807FFFFF
    pw = ModelParams(frac_bits=WIDE)   # (the zero product 0*0 has e = -28 and sets e_max, so F must reach down to 2^-149)
    assert fdpa_group(pw, [0], [0], csub, fm.FP16, fm.FP16) == csub
    assert fdpa_group(pw.with_(ftz_in=True), [0], [0], csub, fm.FP16, fm.FP16) == 0
    # smallest normal is not flushed
    assert fdpa_group(p.with_(ftz_in=True), [0x0400], [one], 0, fm.FP16, fm.FP16) == f32_bits(2.0 ** -14)


def test_output_flush_keeps_sign():
    # Alg. "FTZ-Add/FTZ-Mul": |z| < 2^-126 -> z * 0.0
    p = ModelParams(frac_bits=40)
    a, b = [bf16_bits(-(2.0 ** -100))], [bf16_bits(2.0 ** -30)]
    assert fdpa_group(p, a, b, 0, fm.BF16, fm.BF16) == f32_bits(-(2.0 ** -130))
    assert fdpa_group(p.with_(ftz_out=True), a, b, 0, fm.BF16, fm.BF16) == 0x80000000
    b = [bf16_bits(2.0 ** -26)]
    assert fdpa_group(p.with_(ftz_out=True), a, b, 0, fm.BF16, fm.BF16) == f32_bits(-(2.0 ** -126))
    # applied after every group: a subnormal partial result cannot reach the next group
    a2 = [bf16_bits(2.0 ** -100), bf16_bits(2.0 ** -100)]
    b2 = [bf16_bits(2.0 ** -30), bf16_bits(2.0 ** -30)]
    chained = emulate_element(p.with_(ftz_out=True, group_len=1), a2, b2, 0, fm.BF16, fm.BF16)
    assert chained == 0
    fused = emulate_element(p.with_(ftz_out=True, group_len=2), a2, b2, 0, fm.BF16, fm.BF16)
    assert fused == 0   # 2^-129 is still subnormal
    a3 = [bf16_bits(2.0 ** -100)] * 16
    b3 = [bf16_bits(2.0 ** -30)] * 16
    assert emulate_element(p.with_(ftz_out=True, group_len=16), a3, b3, 0, fm.BF16, fm.BF16) == f32_bits(2.0 ** -126)
    assert emulate_element(p.with_(ftz_out=True, group_len=8), a3, b3, 0, fm.BF16, fm.BF16) == 0


def test_exact_zero_is_positive():
    one, mone = fp16_bits(1.0), fp16_bits(-1.0)
    p = ModelParams(frac_bits=24)
    assert fdpa_group(p, [one, mone], [one, one], 0, fm.FP16, fm.FP16) == 0
    assert fdpa_group(p, [0x8000], [one], 0x80000000, fm.FP16, fm.FP16) == 0
    assert fdpa_group(p.with_(c_mode=C_AFTER_EXACT), [0x8000], [one], 0x80000000, fm.FP16, fm.FP16) == 0


def test_c_after_exact_mode():
    # T over the products only (e_max over products), then rho(T 2^e_max + c) exactly
    rng = np.random.default_rng(15)
    p = ModelParams(frac_bits=WIDE, c_mode=C_AFTER_EXACT)
    for _ in range(200):
        a = synth.random_bits(rng, 4, fm.BF16).tolist()
        b = synth.random_bits(rng, 4, fm.BF16).tolist()
        c = int(synth.random_bits(rng, 1, fm.FP32)[0])
        assert fdpa_group(p, a, b, c, fm.BF16, fm.BF16) == e_fdpa(a, b, c, fm.BF16, fm.BF16)
    # narrow F: products truncated relative to their own maximum, c never truncated
    a = [bf16_bits(1.0), bf16_bits(2.0 ** -9)]
    b = [bf16_bits(1.0), bf16_bits(1.0)]
    d = fdpa_group(ModelParams(frac_bits=8, c_mode=C_AFTER_EXACT), a, b, f32_bits(2.0 ** -20), fm.BF16, fm.BF16)
    assert Fraction(bits_f32(d)) == 1 + Fraction(1, 1 << 20)
    d = fdpa_group(ModelParams(frac_bits=8, c_mode=C_IN_GROUP), a, b, f32_bits(2.0 ** -20), fm.BF16, fm.BF16)
    assert bits_f32(d) == 1.0


def test_group_length_rules():
    p = ModelParams(group_len=8)
    one = fp16_bits(1.0)
    with pytest.raises(ValueError):
        emulate_element(p, [one] * 12, [one] * 12, 0, fm.FP16, fm.FP16)   # K % L != 0 is rejected
    # L = min(K, L_max)
    assert bits_f32(emulate_element(ModelParams(group_len=64), [one] * 16, [one] * 16, 0, fm.FP16, fm.FP16)) == 16.0


def test_rz_e8m13_conversion():
    # Table "Conversion functions": RZ-E8M13 keeps 13 mantissa bits, toward zero
    from oracle.rounding import RZ as _RZ
    p = ModelParams(group_len=2, frac_bits=30, out_round=_RZ, out_mant_bits=13)
    one = fp16_bits(1.0)
    # 1 + 2^-13 + 2^-14: the 2^-14 part is cut; negative likewise toward zero
    a, b = [one, fp16_bits(2.0 ** -13 + 2.0 ** -14)], [one, one]
    assert bits_f32(fdpa_group(p, a, b, 0, fm.FP16, fm.FP16)) == 1.0 + 2.0 ** -13
    a = [fp16_bits(-1.0), fp16_bits(-(2.0 ** -13 + 2.0 ** -14))]
    assert bits_f32(fdpa_group(p, a, b, 0, fm.FP16, fm.FP16)) == -(1.0 + 2.0 ** -13)
    # every result has its low 10 bits clear, and equals the RZ-FP32 result cut there
    rng = np.random.default_rng(2)
    for _ in range(200):
        a = synth.random_bits(rng, 2, fm.FP16).tolist()
        b = synth.random_bits(rng, 2, fm.FP16).tolist()
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 100, 150)[0])
        d13 = fdpa_group(p, a, b, c, fm.FP16, fm.FP16)
        d23 = fdpa_group(p.with_(out_mant_bits=23), a, b, c, fm.FP16, fm.FP16)
        assert d13 == d23 & 0xFFFFFC00
    with pytest.raises(ValueError):
        fdpa_group(p.with_(out_round=RNE), a, b, c, fm.FP16, fm.FP16)


# ---------------------------------------------------------------- invariants of the fused sum (Algorithm "T-FDPA")
@pytest.mark.parametrize("cm", [C_IN_GROUP, C_AFTER_EXACT])
def test_order_inside_a_group_does_not_matter_but_groups_do(cm):
    # every term of a group is aligned to the same maximum and the integer sum is exact: permuting the products of a
    # group changes nothing; moving a product to another group of the chain generally does
    rng = np.random.default_rng(41)
    p = ModelParams(group_len=8, frac_bits=13, c_mode=cm, out_round=RZ)
    moved = 0
    for _ in range(60):
        A = synth.narrow_exponent_bits(rng, (1, 4, 16), fm.FP16, 8, 22)
        B = synth.narrow_exponent_bits(rng, (1, 3, 16), fm.FP16, 8, 22)
        C = synth.narrow_exponent_bits(rng, (1, 4, 3), fm.FP32, 110, 140)
        want, _ = o2lib_emulate(p, A, B, C)
        perm = np.concatenate([rng.permutation(8), 8 + rng.permutation(8)])
        got, _ = o2lib_emulate(p, A[:, :, perm], B[:, :, perm], C)
        assert np.array_equal(got, want)
        swap = np.arange(16); swap[[0, 8]] = swap[[8, 0]]
        other, _ = o2lib_emulate(p, A[:, :, swap], B[:, :, swap], C)
        moved += int((other != want).sum())
    assert moved > 0


def test_scaling_by_a_power_of_two_shifts_the_result():
    # Exp enters only through differences to e_max and through the final scale: A * 2^s and C * 2^s give D * 2^s
    # bit for bit while nothing leaves the normal ranges
    rng = np.random.default_rng(42)
    for trial in range(40):
        p = ModelParams(group_len=int(rng.choice([4, 8])), frac_bits=int(rng.choice([13, 24])), out_round=int(rng.integers(0, 2)),
                        c_mode=int(rng.integers(0, 2)))
        A = synth.narrow_exponent_bits(rng, (1, 3, 8), fm.BF16, 110, 140)
        B = synth.narrow_exponent_bits(rng, (1, 3, 8), fm.BF16, 110, 140)
        C = synth.narrow_exponent_bits(rng, (1, 3, 3), fm.FP32, 100, 150)
        s = int(rng.integers(-20, 21))
        want, _ = o2lib_emulate(p, A, B, C, ta=fm.BF16)
        got, _ = o2lib_emulate(p, (A.astype(np.int64) + (s << 7)).astype(np.uint16), B, (C.astype(np.int64) + (s << 23)).astype(np.uint32), ta=fm.BF16)
        nz = (want & 0x7FFFFFFF) != 0
        assert np.array_equal(got[nz].astype(np.int64), want[nz].astype(np.int64) + (s << 23)), trial
        assert not (got[~nz] & 0x7FFFFFFF).any()


def o2lib_emulate(p, A, B, C, ta=fm.FP16):
    from oracle import o2lib
    return o2lib.emulate_mma(p, A, B, C, ta, ta)
