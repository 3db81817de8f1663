"""GPU parity of the TR-FDPA and GTR-FDPA modes (paper Sec. 4.1.3, Algorithms "TR-FDPA" and "GTR-FDPA",
Sec. 4.2 product overflow) against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_mma as o1_emulate, C_AFTER_RD, C_AFTER_RD_EVEN_ODD
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from helpers import f32_bits, fp16_bits, bf16_bits
from test_gpu_parity import mm, gpu_emulate, make_case, assert_same, PAIRS  # noqa: F401

TR = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)
GTR = ModelParams(group_len=16, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD_EVEN_ODD)


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_tr_gtr_random_parameters(mm, ta, tb):
    rng = np.random.default_rng(900 + 8 * ta + tb)
    for trial in range(12):
        mode = C_AFTER_RD if trial % 2 else C_AFTER_RD_EVEN_ODD
        L = int(rng.choice([2, 4, 8, 16, 32, 0]))
        k = int(rng.choice([8, 16, 64])) if L == 0 else L * int(rng.integers(1, 5))
        F = int(rng.choice([0, 5, 13, 23, 24, 25, 31, 40]))
        F2 = min(int(rng.choice([0, 24, 31, 31, 31, 36, 44])), F + 40)      # limit of the C form of the oracle
        p = ModelParams(group_len=L, frac_bits=F, frac_bits2=F2, c_mode=mode, out_round=int(rng.integers(0, 2)),
                        ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        nan_bits=0x7FFFFFFF if trial % 3 == 0 else 0x7FC00000)
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        c_exp = (90, 165) if trial % 4 < 2 else None
        A, B, C = make_case(rng, ta, tb, nb, m, n, k, special_frac=0.01 if trial % 3 == 0 else 0.0, c_exp=c_exp)
        if ta == fm.BF16 and tb == fm.BF16 and trial % 4 < 2:
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 100, 150)
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 100, 150)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert_same(got, want, "%s %s" % (p, gpu_emulate.last_kernel))


@pytest.mark.parametrize("p,ta,tb", [(TR, fm.FP16, fm.FP16), (TR, fm.BF16, fm.BF16), (GTR, fm.E4M3, fm.E5M2),
                                     (GTR, fm.E5M2, fm.E5M2), (GTR, fm.E4M3, fm.E4M3)])
def test_preset_models_on_instruction_tiles(mm, p, ta, tb):
    # the shapes the models are meant for: many 32x32xL and 16x16x(2L) tiles, accumulators near the products
    rng = np.random.default_rng(40 + ta + tb)
    L = p.group_len
    for (nb, m, n, k) in ((37, 32, 32, L), (65, 16, 16, 2 * L)):
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *((120, 134) if ta == fm.BF16 else (1, 30 if ta != fm.E4M3 else 14)))
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *((120, 134) if tb == fm.BF16 else (1, 30 if tb != fm.E4M3 else 14)))
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 100, 150)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert_same(got, want, "%s %s" % (p, gpu_emulate.last_kernel))
        # a sample also against the rational form
        want1 = o1_emulate(p, A[:1, :4], B[:1, :4], C[:1, :4, :4], ta, tb)
        assert_same(got[:1, :4, :4], want1, "rational form")


def test_hand_derived_cases_on_the_gpu(mm):
    # the worked cases of tests/test_oracle_tr.py, batched as 1x1xL tiles
    def pad(v, L, enc):
        return [enc(x) for x in v] + [enc(0.0)] * (L - len(v))
    cases8 = [([1.0], [1.0], -2.0 ** -30, 0x3F7FFFFF), ([1.0], [1.0], 2.0 ** -30, 0x3F800000),
              ([1.0], [1.0], -2.0 ** -126, 0x3F7FFFFF), ([1.0], [1.0], -2.0 ** -26, 0x3F7FFFFF),
              ([2.0 ** 13, -0.25], [2.0 ** 10, 1.0], 0.0, f32_bits(2.0 ** 23))]
    A = np.array([[pad(a, 8, fp16_bits)] for a, _, _, _ in cases8], dtype=np.uint16)
    B = np.array([[pad(b, 8, fp16_bits)] for _, b, _, _ in cases8], dtype=np.uint16)
    C = np.array([[[f32_bits(c)]] for _, _, c, _ in cases8], dtype=np.uint32)
    got = gpu_emulate(mm, TR, A, B, C, fm.FP16, fm.FP16).ravel()
    assert [int(x) for x in got] == [w for _, _, _, w in cases8]
    cases16 = [([1.0], [1.0], -2.0 ** -30, 0x3F800000), ([1.0], [1.0], -2.0 ** -25, 0x3F7FFFFF),
               ([1.0], [1.0], -2.0 ** -26, 0x3F800000),
               ([2.0 ** 13, -0.25], [2.0 ** 10, 1.0], 0.0, f32_bits(2.0 ** 23 - 0.5)),
               ([2.0 ** 13, 0.25], [2.0 ** 10, 1.0], 0.0, f32_bits(2.0 ** 23)),
               ([2.0 ** 12, 2.0 ** -12], [1.0, 1.0], -(2.0 ** 12), f32_bits(2.0 ** -12)),
               ([2.0 ** 12, 2.0 ** -13], [1.0, 1.0], -(2.0 ** 12), 0)]
    A = np.array([[pad(a, 16, fp16_bits)] for a, _, _, _ in cases16], dtype=np.uint16)
    B = np.array([[pad(b, 16, fp16_bits)] for _, b, _, _ in cases16], dtype=np.uint16)
    C = np.array([[[f32_bits(c)]] for _, _, c, _ in cases16], dtype=np.uint32)
    got = gpu_emulate(mm, GTR, A, B, C, fm.FP16, fm.FP16).ravel()
    assert [int(x) for x in got] == [w for _, _, _, w in cases16]


def test_product_overflow_on_the_gpu(mm):
    p = TR.with_(group_len=2)
    big, nbig, half = bf16_bits(2.0 ** 64), bf16_bits(-(2.0 ** 64)), bf16_bits(-(2.0 ** 63))
    near = bf16_bits(2.0 ** 64 - 2.0 ** 56)
    A = np.array([[[big, half]], [[big, big]], [[nbig, 0]], [[near, 0]], [[1, 0]]], dtype=np.uint16)
    B = np.array([[[big, big]], [[nbig, big]], [[big, 0]], [[near, 0]], [[bf16_bits(2.0 ** 127), 0]]], dtype=np.uint16)
    C = np.zeros((5, 1, 1), dtype=np.uint32)
    got = gpu_emulate(mm, p, A, B, C, fm.BF16, fm.BF16).ravel()
    want = [0x7F800000, p.nan_bits, 0xFF800000, f32_bits((2.0 ** 64 - 2.0 ** 56) ** 2), f32_bits(2.0 ** -6)]
    assert [int(x) for x in got] == want
    assert_same(got.reshape(5, 1, 1), o1_emulate(p, A, B, C, fm.BF16, fm.BF16), "rational form")


def test_rd_mode_limits_are_errors(mm):
    import torch
    z = torch.zeros(64, dtype=torch.int32, device="cuda")
    h = mm.model_create(group_len=3, frac_bits=24, frac_bits2=31, c_mode=mm.C_AFTER_RD_EVEN_ODD)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, z, z, z, z, 1, 1, 3, 1, (mm.FP16, mm.FP16, mm.FP32, mm.FP32))
    assert ei.value.status == 3          # MMAEMU_ERR_SHAPE
    mm.model_destroy(h)
    h = mm.model_create(group_len=0, frac_bits=40, frac_bits2=48, c_mode=mm.C_AFTER_RD)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, z, z, z, z, 1, 1, 16, 1, (mm.FP16, mm.FP16, mm.FP32, mm.FP32))
    assert ei.value.status == 2          # MMAEMU_ERR_UNSUPPORTED: 48 + 3 + 4 > 53
    mm.model_destroy(h)


# ------------------------------------------------------------------ variations of the RD mode
from oracle.fdpa import C_IN_GROUP, C_AFTER_EXACT, SPLIT_HALVES


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3),
                                   (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.E4M3, fm.BF16)])
def test_variations_random_parameters(mm, ta, tb):
    rng = np.random.default_rng(1700 + 8 * ta + tb)
    for trial in range(20):
        L = int(rng.choice([2, 4, 8, 16, 32, 0]))
        k = int(rng.choice([8, 16, 64])) if L == 0 else L * int(rng.integers(1, 4))
        F = int(rng.choice([0, 5, 13, 24, 25, 40]))
        p = ModelParams(group_len=L, frac_bits=F, frac_bits2=int(rng.choice([max(F - 3, 0), 24, 31, 36, min(F + 40, 44)])),
                        c_mode=int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD, C_AFTER_RD])),
                        out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)))
        if p.c_mode == C_AFTER_RD:
            split = int(rng.integers(0, 3))
            p = p.with_(split=split, acc_special_truncation=bool(rng.integers(0, 2)),
                        frac_bits_merge=int(rng.choice([0, 13, 24, 31])) if split else 0,
                        frac_bits_acc=int(rng.choice([0, 13, 24, 30])), f2_at_leading_bit=bool(rng.integers(0, 2)),
                        sum_drop_distance=int(rng.choice([0, 0, 5, 20, 28])))
            fc = p.frac_bits_acc or p.frac_bits
            if p.frac_bits2 > fc + 40:
                p = p.with_(frac_bits2=fc + 40)
        else:
            p = p.with_(frac_bits2=0)
            if p.c_mode == C_AFTER_EXACT and p.frac_bits > 30:
                p = p.with_(frac_bits=30)
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 24)), int(rng.integers(1, 24))
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.2)
        A[0, 0, :] = 0
        lo, hi = ((90, 165) if trial % 4 < 2 else (1, 254))
        if ta == fm.BF16 and tb == fm.BF16 and trial % 4 < 2:
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 100, 150)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, lo, hi)
        C[0, 0, 0] = 0
        if trial % 5 == 0:
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.02)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.05)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert_same(got, want, "%s %s" % (p, gpu_emulate.last_kernel))
