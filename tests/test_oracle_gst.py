"""CPU tests of GST-FDPA (paper Algorithm "GST-FDPA", Sec. 4.1.3; Table "GST-FDPA parameter selection").  The paper
prints no worked value for it; the pins are what the definition fixes: closed form (nothing truncated: rho of the exact
scaled dot product), the exactness of the dot product inside a group against its truncation across groups (hand-derived),
the scale factor decodings, special values, and the reduction to plain T-FDPA when every group is one product of unit
exponent."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import formats as fm
from oracle.gst import gst_fdpa, emulate_element, decode_scale, SCALE_E8M0, SCALE_UE4M3
from oracle.rounding import to_fp32, RNE, RZ
from helpers import f32_bits, bits_f32

FP4 = {0.0: 0, 0.5: 1, 1.0: 2, 1.5: 3, 2.0: 4, 3.0: 5, 4.0: 6, 6.0: 7}


def f4(x):
    return FP4[abs(x)] | (8 if x < 0 else 0)


def test_scale_decodings():
    assert decode_scale(127, SCALE_E8M0) == (1, 0) and decode_scale(130, SCALE_E8M0) == (1, 3) and decode_scale(0, SCALE_E8M0) == (1, -127)
    assert decode_scale(255, SCALE_E8M0) is None
    # UE4M3: 0x38 = 1.0 (E = 7), 0x3C = 1.5, 0x7E = 448 = 1.75 * 2^8, 0x01 = 2^-9 = 0.001b * 2^-6, 0x7F NaN
    assert decode_scale(0x38, SCALE_UE4M3) == (1, 0) and decode_scale(0x3C, SCALE_UE4M3) == (Fraction(3, 2), 0)
    assert decode_scale(0x7E, SCALE_UE4M3) == (Fraction(7, 4), 8) and decode_scale(0x01, SCALE_UE4M3) == (Fraction(1, 8), -6)
    assert decode_scale(0x7F, SCALE_UE4M3) is None and decode_scale(0xFF, SCALE_UE4M3) is None
    assert decode_scale(0xB8, SCALE_UE4M3) == (1, 0)                 # the top bit is ignored


@pytest.mark.parametrize("fmt,kb", [(SCALE_UE4M3, 16), (SCALE_E8M0, 32)])
def test_wide_f_is_rho_of_the_exact_scaled_dot_product(fmt, kb):
    rng = np.random.default_rng(5 + fmt)
    L, G = 64, 16
    for _ in range(60):
        a, b = rng.integers(0, 16, L).tolist(), rng.integers(0, 16, L).tolist()
        al = (rng.integers(0x20, 0x58, L // kb) if fmt == SCALE_UE4M3 else rng.integers(120, 135, L // kb)).tolist()
        be = (rng.integers(0x20, 0x58, L // kb) if fmt == SCALE_UE4M3 else rng.integers(120, 135, L // kb)).tolist()
        c = f32_bits(float(rng.standard_normal()) * 64)
        exact = fm.decode(c, fm.FP32).value
        for k in range(L):
            sa, sb = decode_scale(al[k // kb], fmt), decode_scale(be[k // kb], fmt)
            exact += fm.decode(a[k], fm.E2M1).value * fm.decode(b[k], fm.E2M1).value * sa[0] * sb[0] * Fraction(2) ** (sa[1] + sb[1])
        for rho in (RNE, RZ):
            assert gst_fdpa(a, b, c, al, be, G, kb, 90, rho, fmt) == to_fp32(exact, rho)


def test_exact_inside_a_group_truncated_across_groups():
    # G = 2, two groups, unit scales (E8M0 127): e_g = 0 for both groups and e_c = Exp(c).
    # group 0: 6*6 + 0.5*0.5 = 36.25, group 1: 0.5*0.5 + 0 = 0.25; c = 2^10: e_max = 10, F = 11: unit 2^-1.
    # Inside group 0 the dot product is exact (36.25), only then truncated: 36.0; group 1 alone is cut to 0.
    a = [f4(6), f4(0.5), f4(0.5), f4(0)]
    b = [f4(6), f4(0.5), f4(0.5), f4(0)]
    u = [127, 127]
    c = f32_bits(1024.0)
    assert bits_f32(gst_fdpa(a, b, c, u, u, 2, 2, 11, RZ, SCALE_E8M0)) == 1024.0 + 36.0
    assert bits_f32(gst_fdpa(a, b, c, u, u, 2, 2, 12, RZ, SCALE_E8M0)) == 1024.0 + 36.25 + 0.25
    # with G = 4 both small products join the one exact dot product 36.5 and survive F = 11 together
    assert bits_f32(gst_fdpa(a, b, c, [127], [127], 4, 4, 11, RZ, SCALE_E8M0)) == 1024.0 + 36.5
    # the exponent of a group is that of its scale factors only: with c = 0 (Exp = -126) and unit scales e_max = 0,
    # so F = 2 keeps quarters however large the dot product is
    assert bits_f32(gst_fdpa(a, b, 0, u, u, 2, 2, 2, RZ, SCALE_E8M0)) == 36.5
    assert bits_f32(gst_fdpa(a, b, 0, u, u, 2, 2, 1, RZ, SCALE_E8M0)) == 36.0      # 36.25 -> 36.0, 0.25 -> 0
    # a scale factor moves e_g: group 1 scaled by 2^12 (e = 12) becomes the maximum, F = 11 leaves group 0 a unit of 2
    assert bits_f32(gst_fdpa(a, b, 0, [127, 133], [127, 133], 2, 2, 11, RZ, SCALE_E8M0)) == 0.25 * 4096 + 36.0
    # UE4M3 significands multiply the dot product: 36.25 * 1.5 * 1.25 at exponent 0
    assert bits_f32(gst_fdpa(a[:2], b[:2], 0, [0x3C], [0x3A], 2, 2, 20, RZ, SCALE_UE4M3)) == 36.25 * 1.5 * 1.25


def test_specials_and_chain():
    a, b = [f4(1)] * 4, [f4(1)] * 4
    u = [127, 127]
    assert gst_fdpa(a, b, 0x7FC00000, u, u, 2, 2, 35, RZ, SCALE_E8M0) == 0x7FFFFFFF
    assert gst_fdpa(a, b, 0, [255, 127], u, 2, 2, 35, RZ, SCALE_E8M0) == 0x7FFFFFFF
    assert gst_fdpa(a, b, 0xFF800000, u, u, 2, 2, 35, RZ, SCALE_E8M0) == 0xFF800000
    assert gst_fdpa([0] * 4, b, 0x80000000, u, u, 2, 2, 35, RZ, SCALE_E8M0) == 0
    # chain of two operations of length 4 (K = 8): the intermediate is rounded to binary32 (RZ)
    a8, b8 = [f4(1)] * 8, [f4(1)] * 8
    c = f32_bits(2.0 ** 24)
    assert bits_f32(emulate_element(a8, b8, c, [127] * 4, [127] * 4, 4, 2, 2, 35, RZ, SCALE_E8M0)) == 2.0 ** 24 + 8
    # four products of 0.25 add 1 per operation: 2^24 + 1 is cut back to 2^24 by RZ-FP32 both times; in one operation
    # of length 8 the sum 2 is kept
    assert bits_f32(emulate_element([f4(0.5)] * 8, [f4(0.5)] * 8, c, [127] * 4, [127] * 4, 4, 2, 2, 35, RZ, SCALE_E8M0)) == 2.0 ** 24
    assert bits_f32(emulate_element([f4(0.5)] * 8, [f4(0.5)] * 8, c, [127] * 4, [127] * 4, 8, 2, 2, 35, RZ, SCALE_E8M0)) == 2.0 ** 24 + 2
    with pytest.raises(ValueError):
        gst_fdpa(a, b, 0, u, u, 4, 2, 35, RZ, SCALE_E8M0)           # a group across two blocks


@pytest.mark.parametrize("fmt,kb", [(SCALE_UE4M3, 16), (SCALE_E8M0, 32), (SCALE_UE4M3, 32)])
def test_c_form_matches_rational_form(fmt, kb):
    from oracle import o2lib
    rng = np.random.default_rng(40 + fmt + kb)
    for trial in range(10):
        L, G = (64, 16) if trial % 2 == 0 else (32, int(rng.choice([4, 8, 16])))
        F = int(rng.choice([8, 20, 35]))
        rho = int(rng.integers(0, 2))
        nb, m, n, k = 2, 3, 3, 128
        A = rng.integers(0, 16, (nb, m, k)).astype(np.uint8)
        B = rng.integers(0, 16, (nb, n, k)).astype(np.uint8)
        lo, hi = ((0x08, 0x7F) if trial % 3 else (0x00, 0x100)) if fmt == SCALE_UE4M3 else ((110, 140) if trial % 3 else (0, 256))
        SA = rng.integers(lo, hi, (nb, m, k // kb)).astype(np.uint8)
        SB = rng.integers(lo, hi, (nb, n, k // kb)).astype(np.uint8)
        C = (rng.standard_normal((nb, m, n)) * 2.0 ** rng.integers(-20, 20, (nb, m, n))).astype(np.float32).view(np.uint32)
        C[0, 0, 0] = 0x7F800000
        C[0, 0, 1] = 0x7FC00001
        got = o2lib.emulate_gst(A, B, C, SA, SB, L, G, kb, F, rho, fmt)
        for t in range(nb):
            for i in range(m):
                for j in range(n):
                    want = emulate_element(A[t, i].tolist(), B[t, j].tolist(), int(C[t, i, j]), SA[t, i].tolist(), SB[t, j].tolist(),
                                           L, G, kb, F, rho, fmt)
                    assert int(got[t, i, j]) == want, (trial, t, i, j, hex(int(got[t, i, j])), hex(want))
