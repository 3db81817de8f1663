"""FP32 operands.  The paper's FP32 instructions are chains of fused multiply-adds (Sec. 4.1.2, Algorithms "FMA" and
"Phi_FMA"; Sec. 5: every FP32 / FP64 instruction gives -0.875 on the worked example): one product per step, exact,
added to the accumulator exactly, rounded once.  In this oracle that is the chained model with L = 1, the accumulator
added after the exact product (C_AFTER_EXACT) and F wide enough for a 48-bit product (F >= 46).

Pins: the C library's fmaf (an independent, correctly rounded implementation of the same operation); the worked
example; equality with BF16 / FP16 operands of the same values under the truncating models."""
import ctypes
import ctypes.util

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_mma, emulate_element, fdpa_group, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from helpers import f32_bits, bits_f32

FMA = ModelParams(group_len=1, frac_bits=46, c_mode=C_AFTER_EXACT, out_round=RNE)

_libm = ctypes.CDLL(ctypes.util.find_library("m"))
_libm.fmaf.restype = ctypes.c_float
_libm.fmaf.argtypes = [ctypes.c_float] * 3


def _f(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


def fmaf_chain(a_bits, b_bits, c_bits):
    d = float(_f(c_bits))
    for x, y in zip(a_bits, b_bits):
        d = _libm.fmaf(float(_f(x)), float(_f(y)), d)
    return int(np.array([d], dtype=np.float32).view(np.uint32)[0])


def same(got, want):
    nan = lambda b: (b & 0x7FFFFFFF) > 0x7F800000
    return (nan(got) and nan(want)) or got == want


@pytest.mark.parametrize("family", ["normal", "narrow", "subnormal", "cancel", "bits"])
def test_fma_chain_equals_libm_fmaf(family):
    rng = np.random.default_rng({"normal": 1, "narrow": 2, "subnormal": 3, "cancel": 4, "bits": 5}[family])
    n, k = 300, 4
    if family == "normal":
        A = rng.standard_normal((n, k)).astype(np.float32).view(np.uint32)
        B = rng.standard_normal((n, k)).astype(np.float32).view(np.uint32)
        C = rng.standard_normal(n).astype(np.float32).view(np.uint32)
    elif family == "narrow":
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 120, 134)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 120, 134)
        C = synth.narrow_exponent_bits(rng, n, fm.FP32, 110, 140)
    elif family == "subnormal":         # products and sums around 2^-126 and below: gradual underflow of the single rounding
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 0, 70)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 60, 127)
        C = synth.narrow_exponent_bits(rng, n, fm.FP32, 0, 12)
    elif family == "cancel":            # c close to -a b: the low product bits decide the result
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 126, 128)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 126, 128)
        C = (-(A[:, 0].view(np.float32).astype(np.float64) * B[:, 0].view(np.float32).astype(np.float64))).astype(np.float32).view(np.uint32)
    else:
        A = synth.random_bits(rng, (n, k), fm.FP32, finite=False)
        B = synth.random_bits(rng, (n, k), fm.FP32, finite=False)
        C = synth.random_bits(rng, n, fm.FP32, finite=False)
    got2, _ = o2lib.emulate_mma(FMA, A.reshape(n, 1, k), B.reshape(n, 1, k), C.reshape(n, 1, 1), fm.FP32, fm.FP32)
    for i in range(n):
        want = fmaf_chain(A[i].tolist(), B[i].tolist(), int(C[i]))
        assert same(int(got2[i, 0, 0]), want), (family, i, hex(int(got2[i, 0, 0])), hex(want))
        if i < 60:
            got1 = emulate_element(FMA, A[i].tolist(), B[i].tolist(), int(C[i]), fm.FP32, fm.FP32)
            assert same(got1, want), (family, i, hex(got1), hex(want))


def test_worked_example_with_fp32_operands():
    # Sec. 5: the FMA chain keeps every bit of the example (-0.875); the truncating models give their own values
    a = [f32_bits(-2.0 ** 13), f32_bits(-0.5), f32_bits(-0.25), f32_bits(-0.125)]
    b = [f32_bits(2.0 ** 10), f32_bits(1.0), f32_bits(1.0), f32_bits(1.0)]
    c = f32_bits(2.0 ** 23)
    assert bits_f32(emulate_element(FMA, a, b, c, fm.FP32, fm.FP32)) == -0.875
    assert bits_f32(emulate_element(ModelParams(group_len=4, frac_bits=24, out_round=RZ), a, b, c, fm.FP32, fm.FP32)) == -0.5
    # F below 46 cuts product bits: (1 + 2^-23)^2 - 1 needs all 46
    x = f32_bits(1.0 + 2.0 ** -23)
    exact = emulate_element(FMA, [x], [x], f32_bits(-1.0), fm.FP32, fm.FP32)
    assert bits_f32(exact) == np.float32(2.0 ** -22 + 2.0 ** -46)
    cut = emulate_element(FMA.with_(frac_bits=45), [x], [x], f32_bits(-1.0), fm.FP32, fm.FP32)
    assert bits_f32(cut) == np.float32(2.0 ** -22)


@pytest.mark.parametrize("tn", [fm.BF16, fm.FP16])
def test_fp32_operands_holding_narrow_values_behave_like_the_narrow_type(tn):
    rng = np.random.default_rng(30 + tn)
    lo, hi = (100, 150) if tn == fm.BF16 else (5, 25)
    for trial in range(12):
        cm = [C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD][trial % 3]
        p = ModelParams(group_len=int(rng.choice([2, 4, 8])), frac_bits=int(rng.choice([13, 24, 25])), c_mode=cm, out_round=int(rng.integers(0, 2)))
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=31)
        A = synth.narrow_exponent_bits(rng, (2, 3, 8), tn, lo, hi)
        B = synth.narrow_exponent_bits(rng, (2, 3, 8), tn, lo, hi)
        C = synth.narrow_exponent_bits(rng, (2, 3, 3), fm.FP32, 100, 150)
        if tn == fm.BF16:
            A32, B32 = A.astype(np.uint32) << 16, B.astype(np.uint32) << 16
        else:
            A32 = A.view(np.float16).astype(np.float32).view(np.uint32)
            B32 = B.view(np.float16).astype(np.float32).view(np.uint32)
        want = emulate_mma(p, A, B, C, tn, tn)
        assert np.array_equal(emulate_mma(p, A32, B32, C, fm.FP32, fm.FP32), want), (trial, p)
        got2, _ = o2lib.emulate_mma(p, A32, B32, C, fm.FP32, fm.FP32)
        assert np.array_equal(got2, want), (trial, p)


def test_c_form_equals_rational_form_on_fp32_operands():
    rng = np.random.default_rng(77)
    for trial in range(16):
        cm = [C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD][trial % 3]
        L = int(rng.choice([1, 2, 4]))
        F = int(rng.choice([13, 24, 30, 40, 46])) if cm != C_AFTER_RD else int(rng.choice([13, 24, 30]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)),
                        ftz_out=bool(rng.integers(0, 2)))
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=int(rng.choice([24, 31])), f2_at_leading_bit=bool(rng.integers(0, 2)), skip_zero_terms=bool(rng.integers(0, 2)))
        if trial % 2:
            A = synth.random_bits(rng, (2, 3, 8), fm.FP32, finite=trial % 4 == 1)
            B = synth.random_bits(rng, (2, 3, 8), fm.FP32)
            C = synth.random_bits(rng, (2, 3, 3), fm.FP32)
        else:
            A = synth.narrow_exponent_bits(rng, (2, 3, 8), fm.FP32, 100, 150)
            B = synth.narrow_exponent_bits(rng, (2, 3, 8), fm.FP32, 100, 150)
            C = synth.narrow_exponent_bits(rng, (2, 3, 3), fm.FP32, 80, 170)
        want = emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
        got, _ = o2lib.emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
        assert np.array_equal(got, want), (trial, p)


def test_nan_payload_rule():
    # the variation `nan_propagate`: which NaN comes out of a chain of FMAs that pass payloads on.  Cases written out
    # from the rule's order of precedence (a, then b, then an invalid product, then the accumulator, then infinities of
    # both signs), step by step along the chain.
    one, inf, ninf, zero = f32_bits(1.0), 0x7F800000, 0xFF800000, 0
    qa, qb, qc, qd = 0x7FC00AAA, 0xFFC00BBB, 0x7FC00CCC, 0x7FC00DDD
    sa, sc = 0x7F800AAA, 0x7F800CCC                                   # signalling: come out quiet, payload kept
    gen = 0xFFC00000
    p = FMA.with_(nan_propagate=True, nan_bits=gen)
    cases = [
        (([qa, one, one, one], [one] * 4, one), qa),
        (([one] * 4, [one, qb, one, one], one), qb),
        (([one] * 4, [one] * 4, qc), qc),
        (([qa, one, one, one], [qb, one, one, one], one), qa),       # a before b in one step
        (([qa, one, one, one], [one] * 4, qc), qa),                  # a before the accumulator
        (([one] * 4, [qb, one, one, one], qc), qb),                  # b before the accumulator
        (([one, qa, one, one], [qb, one, one, one], one), qa),       # the later step's operand over the running NaN
        (([qa, one, one, one], [one, qb, one, one], one), qb),
        (([qa, qd, one, one], [one] * 4, one), qd),
        (([sa, one, one, one], [one] * 4, one), qa),
        (([one] * 4, [one] * 4, sc), qc),
        (([inf, one, one, one], [zero, one, one, one], one), gen),   # infinity times zero: the model's own pattern
        (([inf, one, one, one], [zero, one, one, one], qc), gen),    # ... also over a NaN accumulator
        (([inf, one, one, one], [one] * 4, ninf), gen),              # infinities of both signs
        (([inf, qa, one, one], [zero, one, one, one], one), qa),     # a later operand NaN over the generated one
        (([qa, inf, one, one], [one, zero, one, one], one), gen),    # a later invalid product over the running NaN
        (([inf, one, one, one], [one] * 4, one), inf),               # no NaN at all: unchanged
    ]
    A = np.array([c[0][0] for c in cases], dtype=np.uint32).reshape(len(cases), 1, 4)
    B = np.array([c[0][1] for c in cases], dtype=np.uint32).reshape(len(cases), 1, 4)
    C = np.array([c[0][2] for c in cases], dtype=np.uint32).reshape(len(cases), 1, 1)
    got2, _ = o2lib.emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
    for i, ((a, b, c), want) in enumerate(cases):
        assert emulate_element(p, a, b, c, fm.FP32, fm.FP32) == want, (i, hex(emulate_element(p, a, b, c, fm.FP32, fm.FP32)), hex(want))
        assert int(got2[i, 0, 0]) == want, (i, hex(int(got2[i, 0, 0])), hex(want))
    # inside one group of several products the order is a_0, b_0, a_1, b_1, ...
    g = ModelParams(group_len=4, frac_bits=24, nan_propagate=True, nan_bits=gen)
    assert emulate_element(g, [one, qa, one, one], [qb, one, one, one], one, fm.FP32, fm.FP32) == qb
    assert emulate_element(g, [one, qa, one, one], [one, one, qb, one], qc, fm.FP32, fm.FP32) == qa
    assert emulate_element(g, [inf, one, one, one], [zero, one, one, one], qc, fm.FP32, fm.FP32) == gen
    # without the variation: one pattern whatever the operands hold; numbers are the same either way
    assert emulate_element(FMA.with_(nan_bits=gen), [qa, one, one, one], [one] * 4, one, fm.FP32, fm.FP32) == gen
    rng = np.random.default_rng(91)
    A = synth.random_bits(rng, (3, 4, 8), fm.FP32, finite=False)
    B = synth.random_bits(rng, (3, 5, 8), fm.FP32, finite=False)
    C = synth.random_bits(rng, (3, 4, 5), fm.FP32, finite=False)
    A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[fm.FP32] + [qa, sa], 0.05)
    B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[fm.FP32] + [qb], 0.05)
    for q in (p, g, g.with_(group_len=2, c_mode=C_AFTER_RD, frac_bits2=31)):
        with_rule = emulate_mma(q, A, B, C, fm.FP32, fm.FP32)
        plain = emulate_mma(q.with_(nan_propagate=False), A, B, C, fm.FP32, fm.FP32)
        isnan = (plain & 0x7FFFFFFF) > 0x7F800000
        assert np.array_equal(with_rule[~isnan], plain[~isnan]) and ((with_rule[isnan] & 0x7FFFFFFF) > 0x7F800000).all()
        assert isnan.any() and (with_rule[isnan] != plain[isnan]).any()
        got, _ = o2lib.emulate_mma(q, A, B, C, fm.FP32, fm.FP32)
        assert np.array_equal(got, with_rule)
    with pytest.raises(ValueError):
        emulate_element(p, [0x7E00], [0x3C00], one, fm.FP16, fm.FP16)
