"""Sec. 6.2.4 on the CPU: the variant of TR-FDPA whose round-downs truncate toward zero (rd_toward_zero), the
deviation histogram of oracle/exact.py, and the bias itself.  What pins them: hand-derived cases worked out beside the
assertions, the sign symmetry that truncation has and round-down has not, and the C form against the rational form."""
from fractions import Fraction

import numpy as np

from oracle import formats as fm, o2lib
from oracle import gen as ogen
from oracle.exact import deviation_hist, DEVIATION_BINS
from oracle.fdpa import ModelParams, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, SPLIT_HALVES, emulate_mma, fdpa_group
from helpers import f32_bits, fp16_bits, bits_f32

TR = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)          # the CDNA3 FP16 / BF16 set
TRZ = TR.with_(rd_toward_zero=True)


def group(p, a, b, c):
    return fdpa_group(p, [fp16_bits(x) for x in a], [fp16_bits(x) for x in b], f32_bits(c), fm.FP16, fm.FP16)


def test_hand_cases_product_sum():
    # One product -(1 + 2^-10) beside c = 2^24.  E = 24, so with F2 = 24 the sum T is brought to units of 1:
    # RD(-1.0009..) = -2, RZ(-1.0009..) = -1.  Both 2^24 - 2 and 2^24 - 1 are binary32 numbers.
    a = [-1.0] + [0.0] * 7
    b = [1.0 + 2.0 ** -10] + [0.0] * 7
    p = TR.with_(frac_bits2=24)
    assert group(p, a, b, 2.0 ** 24) == f32_bits(2.0 ** 24 - 2)
    assert group(p.with_(rd_toward_zero=True), a, b, 2.0 ** 24) == f32_bits(2.0 ** 24 - 1)
    # a positive sum is cut the same way by both
    a[0] = 1.0
    assert group(p, a, b, 2.0 ** 24) == group(p.with_(rd_toward_zero=True), a, b, 2.0 ** 24) == f32_bits(2.0 ** 24 + 1)


def test_hand_cases_accumulator():
    # Product 2^10 * 2^14 = 2^24, c = -(1 + 2^-23): E = 24, F = 24: the accumulator in units of 1:
    # RD(-1.00000012) = -2, RZ = -1.
    a = [2.0 ** 10] + [0.0] * 7
    b = [2.0 ** 14] + [0.0] * 7
    c = -(1.0 + 2.0 ** -23)
    assert group(TR, a, b, c) == f32_bits(2.0 ** 24 - 2)
    assert group(TRZ, a, b, c) == f32_bits(2.0 ** 24 - 1)
    # the merge of a split group: halves -(1 + 2^-10) * 2^-10 (first) and 2^14 * 2^0 (second), merged at F_m = 14 bits
    # below e_max = 14: units of 1: RD(-0.00097..) = -1, RZ = 0
    p = TR.with_(split=SPLIT_HALVES, frac_bits_merge=14, frac_bits2=31)
    a = [-(1.0 + 2.0 ** -10), 0, 0, 0, 2.0 ** 14, 0, 0, 0]
    b = [2.0 ** -10, 0, 0, 0, 1.0, 0, 0, 0]
    assert group(p, a, b, 0.0) == f32_bits(2.0 ** 14 - 1)
    assert group(p.with_(rd_toward_zero=True), a, b, 0.0) == f32_bits(2.0 ** 14)


def test_truncation_is_sign_symmetric_round_down_is_not():
    # every step of the truncating variant commutes with negation (RZ alignment, RZ in place of RD, RNE at the end):
    # Phi'(-A, B, -C) = -Phi'(A, B, C) bit for bit; the printed algorithm breaks this on a good share of inputs
    rng = np.random.default_rng(5)
    A = (rng.standard_normal((4, 16, 8)) * 1000).astype(np.float16).view(np.uint16)
    B = (rng.standard_normal((4, 16, 8)) * 1000).astype(np.float16).view(np.uint16)
    C = rng.standard_normal((4, 16, 16)).astype(np.float32).view(np.uint32)
    An, Cn = A ^ np.uint16(0x8000), C ^ np.uint32(0x80000000)
    for p in (TRZ, TRZ.with_(c_mode=C_AFTER_RD_EVEN_ODD, group_len=8), TRZ.with_(f2_at_leading_bit=True, skip_zero_terms=True)):
        d, dn = emulate_mma(p, A, B, C, fm.FP16, fm.FP16), emulate_mma(p, An, B, Cn, fm.FP16, fm.FP16)
        assert np.array_equal(d ^ np.uint32(0x80000000), dn)
    d, dn = emulate_mma(TR, A, B, C, fm.FP16, fm.FP16), emulate_mma(TR, An, B, Cn, fm.FP16, fm.FP16)
    assert (d ^ np.uint32(0x80000000) != dn).mean() > 0.05


def test_c_form_equals_rational_form_with_truncation():
    rng = np.random.default_rng(11)
    for trial in range(24):
        L = int(rng.choice([2, 4, 8, 16]))
        p = ModelParams(group_len=L, frac_bits=int(rng.integers(8, 30)), frac_bits2=int(rng.integers(8, 36)), c_mode=C_AFTER_RD,
                        split=int(rng.integers(0, 3)) if L % 4 == 0 else 0, acc_special_truncation=bool(rng.integers(0, 2)),
                        f2_at_leading_bit=bool(rng.integers(0, 2)), skip_zero_terms=bool(rng.integers(0, 2)),
                        frac_bits_merge=int(rng.integers(0, 2)) * 20, rd_toward_zero=True, out_round=int(rng.integers(0, 2)))
        t = [fm.FP16, fm.BF16, fm.E5M2][trial % 3]
        A = ogen_bits(rng, (2, 5, 2 * L), t)
        B = ogen_bits(rng, (2, 6, 2 * L), t)
        C = rng.standard_normal((2, 5, 6)).astype(np.float32).view(np.uint32)
        assert np.array_equal(o2lib.emulate_mma(p, A, B, C, t, t)[0], emulate_mma(p, A, B, C, t, t)), p


def ogen_bits(rng, shape, t):
    f = fm.FORMATS[t]
    bias, e = f.bias, rng.integers(-6, 7, size=shape)
    sign = rng.integers(0, 2, size=shape)
    mant = rng.integers(0, 1 << f.mbits, size=shape)
    return ((sign << (f.ebits + f.mbits)) | ((e + bias) << f.mbits) | mant).astype(np.uint16 if f.width == 16 else np.uint8)


def test_deviation_hist_hand_cases():
    # k = 2: 1 * 1 + 3 * 0.5 + c = 2.75 with c = 0.25
    A = np.array([[[fp16_bits(1.0), fp16_bits(3.0)]]], dtype=np.uint16)
    B = np.array([[[fp16_bits(1.0), fp16_bits(0.5)]]], dtype=np.uint16)
    C = np.array([[[f32_bits(0.25)]]], dtype=np.uint32)

    def one(dval, bin_exp=-2):
        return deviation_hist(A, B, C, np.array([[[f32_bits(dval)]]], dtype=np.uint32), fm.FP16, fm.FP16, 1, bin_exp)

    h = one(3.0)                                  # delta = +0.25 = one bin width: bin 33
    assert h["n_positive"] == 1 and h["bins"][33] == 1 and h["sum"] == 0.25 and h["sum_sq"] == 0.0625
    h = one(2.5)                                  # delta = -0.25: floor(-1) = -1: bin 31
    assert h["n_negative"] == 1 and h["bins"][31] == 1 and h["sum"] == -0.25 and h["sum_abs"] == 0.25
    h = one(2.75)                                 # exact: bin 32, the one that starts at zero
    assert h["n_zero"] == 1 and h["bins"][32] == 1 and h["sum"] == 0.0
    h = one(2.75 - 2.0 ** -20)                    # a hair below: still bin 31
    assert h["bins"][31] == 1 and h["sum"] == -2.0 ** -20
    h = one(2.75 + 0.25 - 2.0 ** -20)             # a hair below one width: bin 32
    assert h["bins"][32] == 1
    assert one(100.0)["bins"][63] == 1 and one(-100.0)["bins"][0] == 1      # beyond the range
    assert one(2.75 + 31 * 0.25)["bins"][63] == 1 and one(2.75 - 32 * 0.25)["bins"][0] == 1   # the last bins proper
    h = one(float("inf"))
    assert h["n_skipped"] == 1 and h["n_samples"] == 0 and sum(h["bins"]) == 0
    # no accumulator array: c = 0, real = 2.5
    h = deviation_hist(A, B, None, np.array([[[f32_bits(2.5)]]], dtype=np.uint32), fm.FP16, fm.FP16, 1, -2)
    assert h["n_zero"] == 1
    # stride and accumulation into an existing histogram
    A4, B4 = np.repeat(A, 4, axis=1), np.repeat(B, 3, axis=1)
    D4 = np.full((1, 4, 3), f32_bits(3.0), dtype=np.uint32)
    h = deviation_hist(A4, B4, None, D4, fm.FP16, fm.FP16, 5, -2)          # indices 0, 5, 10 of 12; delta = 0.5
    assert h["n_samples"] == 3 and h["bins"][34] == 3
    h = deviation_hist(A4, B4, None, D4, fm.FP16, fm.FP16, 1, -2, hist=h)
    assert h["n_samples"] == 15 and h["sum"] == 7.5


def test_bias_of_round_down_and_symmetry_of_truncation():
    # the paper's experiment at small size: A, B ~ 1000 N(0,1) in FP16, C ~ N(0,1), 32x32x8 tiles
    gp = lambda op, **kw: ogen.GenParams(family=ogen.GEN_NORMAL, seed=3, operand=op, **kw)
    nt = 6
    A = ogen.generate(gp(0, scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0), fm.FP16, 32 * 8, 0, nt).reshape(nt, 32, 8).astype(np.uint16)
    B = ogen.generate(gp(1, scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0), fm.FP16, 32 * 8, 0, nt).reshape(nt, 32, 8).astype(np.uint16)
    C = ogen.generate(gp(2), fm.FP32, 32 * 32, 0, nt).reshape(nt, 32, 32).astype(np.uint32)
    vals = A.view(np.float16).astype(np.float64)
    assert 900 < vals.std() < 1100 and abs(vals.mean()) < 60                # the factor really is 1000
    res = {}
    for name, p in (("rd", TR), ("rz", TRZ)):
        D = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)[0]
        res[name] = deviation_hist(A, B, C, D, fm.FP16, fm.FP16, 3, -5)
    n = res["rd"]["n_samples"]
    assert n == res["rz"]["n_samples"] == (nt * 1024 + 2) // 3
    for name in ("rd", "rz"):
        h = res[name]
        assert h["n_negative"] + h["n_zero"] + h["n_positive"] == n == sum(h["bins"])
    mean = {k: h["sum"] / n for k, h in res.items()}
    sigma = {k: (h["sum_sq"] / n - mean[k] ** 2) ** 0.5 / n ** 0.5 for k, h in res.items()}      # of the mean
    assert mean["rd"] < -6 * sigma["rd"]                                     # biased toward the negative side
    assert abs(mean["rz"]) < 4 * sigma["rz"]                                 # centred
    assert res["rd"]["n_negative"] > 1.2 * res["rd"]["n_positive"]
    assert 0.9 < res["rz"]["n_negative"] / res["rz"]["n_positive"] < 1.1
