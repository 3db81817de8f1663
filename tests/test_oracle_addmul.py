"""CPU tests of the oracle's Phi_FTZ-AddMul model (paper Sec. 4.1.1, Algorithms "FTZ-Add and FTZ-Mul" and
"Phi_FTZ-AddMul").  The paper's printed values for it (CDNA2 rows of the d00 table: 0.0 and -0.375) are checked with
the other rows in test_oracle_model.py / test_oracle_o2.py; here: its printed summation-tree table, the IEEE
arithmetic it reduces to when nothing is flushed, the flush rules, special values, and the C form."""
import numpy as np
import pytest

from oracle import formats as fm, o2lib, addmul
from oracle.fdpa import ModelParams, emulate_mma, emulate_element, FAMILY_FTZ_ADDMUL, C_AFTER_EXACT
from helpers import f32_bits, bits_f32, fp16_bits, bf16_bits
from paper_2511_10909_amd import synth, probes
from test_oracle_model import _trees
from test_probes import OracleInterface, full_table


def P(p):
    return ModelParams(group_len=p, family=FAMILY_FTZ_ADDMUL)


def test_summation_tree_is_the_papers_pairwise_then_accumulate():
    # Figure "Examples of summation trees", (b): "e.g. AMD CDNA2 mfma_f32_32x32x4bf16_1k"
    iface = OracleInterface(P(4), 1, 1, 4, fm.BF16, fm.BF16)
    table = probes.summation_table(iface)
    assert table == full_table(_trees()["b_pairwise_then_accumulate"])
    assert probes.tree_to_string(probes.infer_tree(table)) == "(((p0 + p1) + (p2 + p3)) + p4)"
    # P = 2: pairs accumulated one after the other
    iface = OracleInterface(P(2), 1, 1, 4, fm.BF16, fm.BF16)
    assert probes.tree_to_string(probes.infer_tree(probes.summation_table(iface))) == "(((p0 + p1) + p4) + (p2 + p3))"


@pytest.mark.parametrize("t,npdt", [(fm.FP16, np.float16), (fm.BF16, None)])
@pytest.mark.parametrize("p", [2, 4])
def test_equals_ieee_binary32_arithmetic_when_nothing_is_flushed(t, npdt, p):
    # operands of moderate size: no subnormal appears anywhere, and the model is plain binary32 arithmetic
    # in the stated order (numpy's float32 + and * are IEEE-754 basic operations)
    rng = np.random.default_rng(5 + p + t)
    K = 16
    lo, hi = ((8, 22) if t == fm.FP16 else (118, 136))
    for _ in range(200):
        a = synth.narrow_exponent_bits(rng, K, t, lo, hi)
        b = synth.narrow_exponent_bits(rng, K, t, lo, hi)
        c = synth.narrow_exponent_bits(rng, 1, fm.FP32, 110, 140)
        af = a.view(np.float16).astype(np.float32) if t == fm.FP16 else (a.astype(np.uint32) << 16).view(np.float32)
        bf = b.view(np.float16).astype(np.float32) if t == fm.FP16 else (b.astype(np.uint32) << 16).view(np.float32)
        d = c.view(np.float32)[0]
        for k in range(0, K, p):
            pr = [af[k + l] * bf[k + l] for l in range(p)]
            s = pr[0] + pr[1]
            if p == 4:
                s = s + (pr[2] + pr[3])
            d = d + s
        want = int(np.float32(d).view(np.uint32))
        got = addmul.emulate_element(p, a.tolist(), b.tolist(), int(c[0]), t, t)
        assert got == want


def test_flush_rules():
    tiny = bf16_bits(2.0 ** -70)
    one = bf16_bits(1.0)
    # a product below 2^-126 is flushed, sign kept: (-2^-70)(2^-70) -> -0; the next add gives c back
    assert addmul.ftz_mul(tiny | 0x8000, fm.BF16, tiny, fm.BF16, 0x7FC00000) == 0x80000000
    assert addmul.emulate_element(2, [tiny | 0x8000, 0], [tiny, 0], f32_bits(3.0), fm.BF16, fm.BF16) == f32_bits(3.0)
    # a product that is a binary32 subnormal (2^-130) is flushed although binary32 could hold it
    a, b = bf16_bits(2.0 ** -65), bf16_bits(2.0 ** -65)
    assert addmul.ftz_mul(a, fm.BF16, b, fm.BF16, 0x7FC00000) == 0
    # sums are flushed too: 2^-126 - 2^-127 * 1.5 = 2^-128: subnormal -> +0
    x, y = f32_bits(2.0 ** -126), f32_bits(-1.5 * 2.0 ** -127)
    assert addmul.ftz_add(x, y, 0x7FC00000) == 0
    assert addmul.ftz_add(f32_bits(-(2.0 ** -126)), f32_bits(1.5 * 2.0 ** -127), 0x7FC00000) == 0x80000000
    # input subnormals become +0.0 whatever their sign; a subnormal accumulator too
    sub = 0x8001
    assert addmul.emulate_element(2, [sub, one], [one, one], 0x80000001, fm.BF16, fm.BF16) == f32_bits(1.0)
    assert addmul.emulate_element(2, [sub, 0], [one, 0], 0x80000001, fm.BF16, fm.BF16) == 0      # (+0 * 1 + 0) + (+0) = +0
    # -0 inputs are not subnormal: (-0 * 1) + (-0 * 1) = -0, and -0 + -0 = -0
    assert addmul.emulate_element(2, [0x8000, 0x8000], [one, one], 0x80000000, fm.BF16, fm.BF16) == 0x80000000
    # exact cancellation gives +0
    assert addmul.emulate_element(2, [one, one | 0x8000], [one, one], 0x80000000, fm.BF16, fm.BF16) == 0


def test_special_values():
    nan, inf, ninf, one, zero = 0x7FC0, 0x7F80, 0xFF80, bf16_bits(1.0), 0
    nb = 0x7FFFABCD
    run = lambda a, b, c: addmul.emulate_element(2, a, b, c, fm.BF16, fm.BF16, nb)
    assert run([nan, one], [one, one], 0) == nb
    assert run([inf, one], [zero, one], 0) == nb                # inf * 0
    assert run([inf, one], [one, one], 0) == 0x7F800000
    assert run([inf, ninf], [one, one], 0) == nb                # inf - inf inside a pair
    assert run([inf, one], [one, one], 0xFF800000) == nb        # against the accumulator
    assert run([one, one], [one, one], 0x7FA00000) == nb        # NaN accumulator, model's encoding
    big = bf16_bits(2.0 ** 100)
    assert run([big, zero], [big, zero], 0) == 0x7F800000       # product overflow by rounding
    assert run([big, big], [big, big | 0x8000], 0) == nb        # +inf + -inf from two overflows


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.FP16, fm.BF16), (fm.E5M2, fm.E4M3)])
def test_o2_equals_rational_form(ta, tb):
    rng = np.random.default_rng(40 + ta + tb)
    for trial in range(12):
        p = P(2 if trial % 2 else 4).with_(nan_bits=0x7FC00000 if trial % 3 else 0xFFC00000)
        k = 4 * int(rng.integers(1, 5))
        nb, m, n = 2, 3, 4
        if trial % 4 == 0:
            A = synth.random_bits(rng, (nb, m, k), ta)
            B = synth.random_bits(rng, (nb, n, k), tb)
            C = synth.random_bits(rng, (nb, m, n), fm.FP32)
        else:     # products and sums around the flush threshold, subnormal inputs included
            lo = {fm.BF16: (50, 80), fm.FP16: (0, 6), fm.E5M2: (0, 6), fm.E4M3: (0, 4)}
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo[ta])
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *lo[tb])
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 0, 6 if ta == fm.BF16 else 110)
        if trial % 5 == 0:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.03)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.05)
        want = emulate_mma(p, A, B, C, ta, tb)
        got, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        assert np.array_equal(got, want), (p, np.argwhere(got != want)[:3])


def test_fma_chain_is_group_length_one_with_exact_two_term_sum():
    # Algorithms "FMA" / "Phi_FMA" (Sec. 4.1.2): d <- RNE-FP32(a_k b_k + d), one product at a time.  On operands whose
    # products are exact rationals this is the chained model with L = 1 and the accumulator added exactly.
    from fractions import Fraction
    from oracle.rounding import rne_fp32
    rng = np.random.default_rng(3)
    p = ModelParams(group_len=1, frac_bits=24, c_mode=C_AFTER_EXACT)
    for _ in range(100):
        a = synth.narrow_exponent_bits(rng, 6, fm.BF16, 90, 160)      # finite, no overflow anywhere
        b = synth.narrow_exponent_bits(rng, 6, fm.BF16, 90, 160)
        c = int(synth.narrow_exponent_bits(rng, 1, fm.FP32, 60, 190)[0])
        d = c
        for x, y in zip(a.tolist(), b.tolist()):
            v = fm.decode(x, fm.BF16).value * fm.decode(y, fm.BF16).value + fm.decode(d, fm.FP32).value
            d = rne_fp32(v) if v != 0 else 0
        assert emulate_element(p, a.tolist(), b.tolist(), c, fm.BF16, fm.BF16) == d
