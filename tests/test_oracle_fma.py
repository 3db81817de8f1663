"""Phi_FMA (Sec. 4.1.2, Algorithms "FMA" and "Phi_FMA") in the oracle: oracle/fma.py.

Pins: the C library's fmaf (an independent, correctly rounded implementation of IEEE-754's fusedMultiplyAdd, signs
of zero included), on random chains of every input family and on every triple of a small set of critical values; the
standard's table of zero signs written out; the worked example of Sec. 5; overflow and the tie at the top of the
range; the payload rule written out case by case; agreement with the FDPA-family chain (group of one product,
accumulator added exactly) everywhere except the one sign the two define differently."""
import ctypes
import ctypes.util
import itertools

import numpy as np
import pytest

from oracle import fma as ofma, formats as fm
from oracle.fdpa import ModelParams, emulate_element as fdpa_element, C_AFTER_EXACT
from oracle.rounding import RNE
from paper_2511_10909_amd import synth
from helpers import f32_bits, bits_f32

_libm = ctypes.CDLL(ctypes.util.find_library("m"))
_libm.fmaf.restype = ctypes.c_float
_libm.fmaf.argtypes = [ctypes.c_float] * 3

NAN = lambda b: (b & 0x7FFFFFFF) > 0x7F800000


def _f(bits):
    return float(np.array([bits], dtype=np.uint32).view(np.float32)[0])


def _bits(x):
    return int(np.array([x], dtype=np.float32).view(np.uint32)[0])


def libm_chain(a_bits, b_bits, c_bits):
    d = _f(c_bits)
    for x, y in zip(a_bits, b_bits):
        d = _libm.fmaf(_f(x), _f(y), d)
    return _bits(d)


def same(got, want):
    return (NAN(got) and NAN(want)) or got == want


CRITICAL = [0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF, 0x00800000, 0x80800000, 0x3F800000, 0xBF800000,
            0x3FC00000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000, 0x7FC00000, 0x33800000, 0xB3800000]


def test_single_fma_equals_libm_on_every_triple_of_critical_values():
    # zeros of both signs, the smallest and the largest subnormal, the smallest normal, +-1, 1.5, +-max, infinities, a NaN,
    # +-2^-24: 17^3 triples cover every sign combination of exact zeros, underflow to zero, overflow and the invalid cases
    for a, b, c in itertools.product(CRITICAL, repeat=3):
        got, want = ofma.fma(a, b, c), _bits(_libm.fmaf(_f(a), _f(b), _f(c)))
        assert same(got, want), (hex(a), hex(b), hex(c), hex(got), hex(want))


@pytest.mark.parametrize("family", ["normal", "narrow", "subnormal", "cancel", "bits", "critical"])
def test_chain_equals_libm_fmaf(family):
    rng = np.random.default_rng({"normal": 1, "narrow": 2, "subnormal": 3, "cancel": 4, "bits": 5, "critical": 6}[family])
    n, k = 300, 4
    if family == "normal":
        A = rng.standard_normal((n, k)).astype(np.float32).view(np.uint32)
        B = rng.standard_normal((n, k)).astype(np.float32).view(np.uint32)
        C = rng.standard_normal(n).astype(np.float32).view(np.uint32)
    elif family == "narrow":
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 120, 134)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 120, 134)
        C = synth.narrow_exponent_bits(rng, n, fm.FP32, 110, 140)
    elif family == "subnormal":
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 0, 70)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 60, 127)
        C = synth.narrow_exponent_bits(rng, n, fm.FP32, 0, 12)
    elif family == "cancel":
        A = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 126, 128)
        B = synth.narrow_exponent_bits(rng, (n, k), fm.FP32, 126, 128)
        C = (-(A[:, 0].view(np.float32).astype(np.float64) * B[:, 0].view(np.float32).astype(np.float64))).astype(np.float32).view(np.uint32)
    elif family == "bits":
        A = synth.random_bits(rng, (n, k), fm.FP32, finite=False)
        B = synth.random_bits(rng, (n, k), fm.FP32, finite=False)
        C = synth.random_bits(rng, n, fm.FP32, finite=False)
    else:
        # mostly zeros of both signs, with +-1 and the smallest subnormals between them: short chains, many exact zeros
        crit = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 0x00000001, 0x80000001], dtype=np.uint32)
        k = 2
        A, B, C = crit[rng.integers(0, len(crit), (n, k))], crit[rng.integers(0, len(crit), (n, k))], crit[rng.integers(0, len(crit), n)]
    negative_zero = 0
    for i in range(n):
        got = ofma.emulate_element(A[i].tolist(), B[i].tolist(), int(C[i]))
        want = libm_chain(A[i].tolist(), B[i].tolist(), int(C[i]))
        assert same(got, want), (family, i, hex(got), hex(want))
        negative_zero += got == 0x80000000
    if family == "critical":
        assert negative_zero > 10           # the family does reach the sign rule


def test_zero_signs_follow_the_standard():
    pz, nz, one, mone = 0, 0x80000000, f32_bits(1.0), f32_bits(-1.0)
    assert ofma.fma(pz, one, pz) == pz
    assert ofma.fma(pz, one, nz) == pz            # (+0) + (-0) = +0
    assert ofma.fma(nz, one, pz) == pz
    assert ofma.fma(nz, one, nz) == nz            # zeros of one sign keep it
    assert ofma.fma(pz, mone, nz) == nz           # the product's sign is the XOR of its factors' signs
    assert ofma.fma(nz, mone, nz) == pz
    assert ofma.fma(one, one, mone) == pz         # exact cancellation of non-zero terms: +0
    assert ofma.fma(mone, one, one) == pz
    assert ofma.fma(0x80000001, 0x00000001, pz) == nz      # a negative result too small for the format: -0 (underflow, not an exact zero)
    assert ofma.fma(0x80000001, 0x00000001, nz) == nz
    assert ofma.fma(0x00000001, 0x00000001, nz) == pz


def test_worked_example_and_range_ends():
    # Sec. 5: every FP32 / FP64 instruction gives -0.875 on the example
    a = [f32_bits(-2.0 ** 13), f32_bits(-0.5), f32_bits(-0.25), f32_bits(-0.125)]
    b = [f32_bits(2.0 ** 10), f32_bits(1.0), f32_bits(1.0), f32_bits(1.0)]
    assert bits_f32(ofma.emulate_element(a, b, f32_bits(2.0 ** 23))) == -0.875
    # one rounding of the exact a b + c: (1 + 2^-23)^2 - 1 = 2^-22 + 2^-46 exactly
    x = f32_bits(1.0 + 2.0 ** -23)
    assert bits_f32(ofma.fma(x, x, f32_bits(-1.0))) == np.float32(2.0 ** -22 + 2.0 ** -46)
    # overflow: max + half an ulp is a tie that goes to the even neighbour 2^128, i.e. infinity; just below stays finite
    mx, one = 0x7F7FFFFF, f32_bits(1.0)
    assert ofma.fma(mx, one, f32_bits(2.0 ** 103)) == 0x7F800000
    assert ofma.fma(mx, one, f32_bits(2.0 ** 103 * (1 - 2.0 ** -24))) == mx
    assert ofma.fma(mx, f32_bits(2.0), 0) == 0x7F800000
    assert ofma.fma(mx, f32_bits(-2.0), 0) == 0xFF800000
    # gradual underflow: 2^-126 * 2^-23 = 2^-149, the smallest subnormal; half of it ties to even (zero)
    assert ofma.fma(0x00800000, f32_bits(2.0 ** -23), 0) == 0x00000001
    assert ofma.fma(0x00800000, f32_bits(2.0 ** -24), 0) == 0
    assert ofma.fma(0x00800000, f32_bits(2.0 ** -24), 0x00000001) == 0x00000002     # 1.5 units: tie to even (2)


def test_special_values_and_payload_rule():
    one, inf, ninf, zero = f32_bits(1.0), 0x7F800000, 0xFF800000, 0
    assert ofma.fma(inf, zero, one, nan_bits=0x7FFFFFFF) == 0x7FFFFFFF
    assert ofma.fma(inf, one, ninf, nan_bits=0x7FFFFFFF) == 0x7FFFFFFF
    assert ofma.fma(0x7FC00123, one, one, nan_bits=0x7FFFFFFF) == 0x7FFFFFFF
    assert ofma.fma(inf, f32_bits(-1.0), one) == ninf
    assert ofma.fma(one, one, ninf) == ninf
    qa, qb, qc, qd = 0x7FC00AAA, 0xFFC00BBB, 0x7FC00CCC, 0x7FC00DDD
    sa, sc = 0x7F800AAA, 0x7F800CCC
    gen = 0xFFC00000
    cases = [
        (([qa, one, one, one], [one] * 4, one), qa),
        (([one] * 4, [one, qb, one, one], one), qb),
        (([one] * 4, [one] * 4, qc), qc),
        (([qa, one, one, one], [qb, one, one, one], one), qa),
        (([qa, one, one, one], [one] * 4, qc), qa),
        (([one] * 4, [qb, one, one, one], qc), qb),
        (([one, qa, one, one], [qb, one, one, one], one), qa),
        (([qa, one, one, one], [one, qb, one, one], one), qb),
        (([qa, qd, one, one], [one] * 4, one), qd),
        (([sa, one, one, one], [one] * 4, one), qa),
        (([one] * 4, [one] * 4, sc), qc),
        (([inf, one, one, one], [zero, one, one, one], one), gen),
        (([inf, one, one, one], [zero, one, one, one], qc), gen),
        (([inf, one, one, one], [one] * 4, ninf), gen),
        (([inf, qa, one, one], [zero, one, one, one], one), qa),
        (([qa, inf, one, one], [one, zero, one, one], one), gen),
        (([inf, one, one, one], [one] * 4, one), inf),
    ]
    chain = ModelParams(group_len=1, frac_bits=46, c_mode=C_AFTER_EXACT, out_round=RNE, nan_propagate=True, nan_bits=gen)
    for i, ((a, b, c), want) in enumerate(cases):
        assert ofma.emulate_element(a, b, c, nan_bits=gen, nan_propagate=True) == want, i
        assert fdpa_element(chain, a, b, c, fm.FP32, fm.FP32) == want, i


def test_fdpa_chain_differs_only_in_the_sign_of_an_exact_zero():
    # the FDPA family gives +0.0 for every exact zero; Phi_FMA keeps the sign of zeros that agree
    chain = ModelParams(group_len=1, frac_bits=46, c_mode=C_AFTER_EXACT, out_round=RNE)
    rng = np.random.default_rng(11)
    crit = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 0x00000001, 0x80000001], dtype=np.uint32)
    differ = 0
    for trial in range(400):
        if trial % 2:
            a, b, c = crit[rng.integers(0, len(crit), 2)].tolist(), crit[rng.integers(0, len(crit), 2)].tolist(), int(crit[rng.integers(0, len(crit))])
        else:
            a = synth.random_bits(rng, 4, fm.FP32, finite=False).tolist()
            b = synth.random_bits(rng, 4, fm.FP32, finite=False).tolist()
            c = int(synth.random_bits(rng, 1, fm.FP32, finite=False)[0])
        x, y = ofma.emulate_element(a, b, c), fdpa_element(chain, a, b, c, fm.FP32, fm.FP32)
        if x != y:
            assert x == 0x80000000 and y == 0, (trial, hex(x), hex(y))
            differ += 1
    assert differ > 0


def test_matrix_form_indexing():
    rng = np.random.default_rng(5)
    A = synth.narrow_exponent_bits(rng, (2, 3, 4), fm.FP32, 120, 134)
    B = synth.narrow_exponent_bits(rng, (2, 5, 4), fm.FP32, 120, 134)
    C = synth.narrow_exponent_bits(rng, (2, 3, 5), fm.FP32, 120, 134)
    D = ofma.emulate_mma(A, B, C)
    for t, i, j in [(0, 0, 0), (1, 2, 4), (0, 1, 3)]:
        assert int(D[t, i, j]) == libm_chain(A[t, i].tolist(), B[t, j].tolist(), int(C[t, i, j]))
