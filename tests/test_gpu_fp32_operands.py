"""GPU parity for FP32 operands (Phi_FMA on FP32 inputs, Sec. 4.1.2; and the truncating models on FP32 inputs)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_mma as o1_emulate, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, SPLIT_HALVES
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from test_gpu_parity import gpu_emulate, assert_same, mm                                     # noqa: F401  (mm is a fixture)


def fp32_case(rng, nb, m, n, k, trial):
    if trial % 3 == 0:
        A = synth.random_bits(rng, (nb, m, k), fm.FP32, finite=trial % 2 == 0)
        B = synth.random_bits(rng, (nb, n, k), fm.FP32)
        C = synth.random_bits(rng, (nb, m, n), fm.FP32)
    elif trial % 3 == 1:
        A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP32, 100, 150)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP32, 100, 150)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 80, 170)
    else:           # results around and below 2^-126
        A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP32, 0, 70)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP32, 60, 127)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 0, 12)
    if trial % 4 == 1:
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[fm.FP32], 0.03)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[fm.FP32], 0.03)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.03)
    return A, B, C


def test_fma_chain_on_fp32_operands(mm):
    from paper_2511_10909_amd import presets
    kw = presets.PAPER[("fma_chain", "fp32")]
    p = ModelParams(group_len=kw["group_len"], frac_bits=kw["frac_bits"], c_mode=kw["c_mode"], out_round=kw["out_round"])
    rng = np.random.default_rng(4100)
    for trial in range(9):
        nb, m, n, k = int(rng.integers(1, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 40)), int(rng.choice([1, 2, 4, 7, 16]))
        A, B, C = fp32_case(rng, nb, m, n, k, trial)
        print("case", trial, (nb, m, n, k), flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
        got = gpu_emulate(mm, p, A, B, C, fm.FP32, fm.FP32)
        assert gpu_emulate.last_kernel == "general"
        assert_same(got, want, "fma chain, trial %d" % trial)
    # and against the rational form directly
    A, B, C = fp32_case(rng, 2, 5, 6, 4, 1)
    assert_same(gpu_emulate(mm, p, A, B, C, fm.FP32, fm.FP32), o1_emulate(p, A, B, C, fm.FP32, fm.FP32), "vs rational form")


def test_fp32_operands_random_parameters(mm):
    rng = np.random.default_rng(4101)
    for trial in range(24):
        L = int(rng.choice([1, 2, 4, 8]))
        k = L * int(rng.integers(1, 4))
        cm = int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        F = int(rng.choice([0, 13, 24, 30, 40, 46, 48])) if cm != C_AFTER_RD else int(rng.choice([0, 13, 24, 30]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)),
                        ftz_out=bool(rng.integers(0, 2)), nan_bits=0x7FFFFFFF if trial % 2 else 0x7FC00000)
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=int(rng.choice([24, 31])), f2_at_leading_bit=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)))
            if L >= 2 and trial % 2:
                p = p.with_(split=SPLIT_HALVES, frac_bits_merge=max(F, 24))
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        A, B, C = fp32_case(rng, nb, m, n, k, trial)
        print("case", trial, p, (nb, m, n, k), flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
        got = gpu_emulate(mm, p, A, B, C, fm.FP32, fm.FP32)
        assert_same(got, want, "fp32 operands %s" % (p,))


def test_wide_f_on_narrow_operands_runs_in_the_general_kernel(mm):
    # frac_bits above 40 (allowed outside the RD modes) with 16-bit operands
    rng = np.random.default_rng(4102)
    for cm, F in ((C_IN_GROUP, 48), (C_AFTER_EXACT, 45), (C_IN_GROUP, 44)):      # (the C oracle takes F + 2 + log2 L <= 50 here)
        p = ModelParams(group_len=8, frac_bits=F, c_mode=cm)
        A = synth.narrow_exponent_bits(rng, (2, 16, 16), fm.BF16, 100, 150)
        B = synth.narrow_exponent_bits(rng, (2, 16, 16), fm.BF16, 100, 150)
        C = synth.narrow_exponent_bits(rng, (2, 16, 16), fm.FP32, 80, 170)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)
        got = gpu_emulate(mm, p, A, B, C, fm.BF16, fm.BF16)
        assert gpu_emulate.last_kernel == "general"
        assert_same(got, want, "F = %d" % F)


def test_fp32_argument_errors(mm):
    from gpu_utils import dev_empty
    x = dev_empty(4096)
    h = mm.model_create(group_len=1, frac_bits=46, c_mode=mm.C_AFTER_EXACT)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, x, x, x, x, 4, 4, 4, 1, (mm.FP32, mm.BF16, mm.FP32, mm.FP32))      # FP32 pairs with itself
    assert ei.value.status == 2
    mm.model_destroy(h)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.model_create(group_len=1, frac_bits=49)
    assert ei.value.status == 2
    with pytest.raises(mm.MmaemuError) as ei:
        mm.model_create(group_len=4, frac_bits=44, frac_bits2=31, c_mode=mm.C_AFTER_RD)       # the RD modes stop at 40
    assert ei.value.status == 2


def test_nan_payload_rule_matches_oracle(mm):
    # `nan_propagate`: NaN results carry payloads (first NaN operand in the order a_0, b_0, a_1, ..., made quiet; the
    # model's own pattern for invalid products; then the accumulator)
    rng = np.random.default_rng(4103)
    qa, sa, qb = 0x7FC00AAA, 0x7F800AAA, 0xFFC00BBB
    for trial in range(8):
        L = int(rng.choice([1, 1, 2, 4]))
        k = L * int(rng.integers(1, 5))
        cm = C_AFTER_EXACT if L == 1 else int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        p = ModelParams(group_len=L, frac_bits=46 if (L == 1) else 24, c_mode=cm, nan_bits=0xFFC00000, nan_propagate=True,
                        ftz_in=bool(trial % 2))
        if cm == C_AFTER_RD:
            p = p.with_(frac_bits2=31)
        nb, m, n = 3, int(rng.integers(1, 24)), int(rng.integers(1, 24))
        A = synth.random_bits(rng, (nb, m, k), fm.FP32, finite=False)
        B = synth.random_bits(rng, (nb, n, k), fm.FP32, finite=False)
        C = synth.random_bits(rng, (nb, m, n), fm.FP32, finite=False)
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[fm.FP32] + [qa, sa], 0.06)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[fm.FP32] + [qb], 0.06)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32] + [0x7FC00CCC], 0.06)
        print("case", trial, p, (nb, m, n, k), flush=True)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP32, fm.FP32)
        got = gpu_emulate(mm, p, A, B, C, fm.FP32, fm.FP32)
        assert_same(got, want, "payload rule, trial %d" % trial)
        assert ((want & 0x7FFFFFFF) > 0x7F800000).any() and (want != o2lib.emulate_mma(p.with_(nan_propagate=False), A, B, C, fm.FP32, fm.FP32)[0]).any()
    h = mm.model_create(group_len=1, frac_bits=24, c_mode=mm.C_AFTER_EXACT, nan_propagate=True)
    from gpu_utils import dev_empty
    x = dev_empty(4096)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, x, x, x, x, 4, 4, 4, 1, (mm.BF16, mm.BF16, mm.FP32, mm.FP32))           # FP32 operands only
    assert ei.value.status == 2
    mm.model_destroy(h)
