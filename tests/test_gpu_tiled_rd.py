"""GPU parity of the tiled kernels in the RD accumulation mode (paper Algorithm "TR-FDPA" and the variations that
`mmaemu.h` documents) against the CPU oracle, bit for bit.  Shapes, operand families and the expectation that the
tiled route is taken follow tests/test_gpu_tiled.py."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_AFTER_RD
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from test_gpu_parity import gpu_emulate, assert_same, mm  # noqa: F401  (fixture)
from test_gpu_tiled import operands, SHAPES, PAIRS

GFX950_16BIT = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, skip_zero_terms=True,
                           f2_at_leading_bit=True, zero_result_positive=True, sum_drop_distance=28, nan_bits=0xFFC00000)
CDNA3_16BIT = ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD)


def random_rd_params(rng, k):
    Ls = [L for L in (4, 8, 16, 32, 0, 64, 24, 2) if (L == 0 or k % L == 0 or L > k)]
    L = int(rng.choice(Ls))
    F = int(rng.choice([0, 3, 13, 16, 24, 25, 27, 29, 30, 32, 36, 40]))
    Fc = int(rng.choice([0, 0, 13, 24, 30]))
    F2 = int(rng.choice([max(F - 2, 0), 24, 31, 31, 36, 44]))
    F2 = min(F2, (Fc or F) + 40)
    return ModelParams(group_len=L, frac_bits=F, frac_bits2=F2, frac_bits_acc=Fc, c_mode=C_AFTER_RD,
                       out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 4) == 0), ftz_out=bool(rng.integers(0, 4) == 0),
                       acc_special_truncation=bool(rng.integers(0, 2)), skip_zero_terms=bool(rng.integers(0, 2)),
                       f2_at_leading_bit=bool(rng.integers(0, 2)), zero_result_positive=bool(rng.integers(0, 2)),
                       sum_drop_distance=int(rng.choice([0, 0, 6, 20, 28])), nan_bits=0xFFC00000 if rng.integers(0, 2) else 0x7FC00000)


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_tiled_rd_parameter_sweep(mm, ta, tb):
    rng = np.random.default_rng(5000 + 8 * ta + tb)
    used_tiled = expected_tiled = 0
    for (m, n, k, nb) in SHAPES:
        for mode in ("narrow", "full", "special", "zeros"):
            p = random_rd_params(rng, k)
            A, B, C = operands(rng, ta, tb, nb, m, n, k, "narrow" if mode == "zeros" else mode)
            if mode == "zeros":     # plenty of zero operands and accumulators, whole zero rows
                A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.3)
                A[0, 0, :] = 0
                B[0, 1, :] = 0
                C = np.where(rng.random(C.shape) < 0.3, np.uint32(0x80000000), C).astype(np.uint32)
            print("tiled rd", ta, tb, (m, n, k, nb), mode, p, flush=True)
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert_same(got, want, "tiled rd %s %s %s %s" % ((m, n, k, nb), mode, p, gpu_emulate.last_kernel))
            Leff = k if p.group_len == 0 else min(p.group_len, k)
            fast_shape = (m % 16 == 0 and n % 16 == 0 and k % 16 == 0) or (m % 32 == 0 and n % 32 == 0 and k % 8 == 0)
            if fast_shape and Leff in (4, 8, 16, 32, k) and not (Leff == 32 and k % 32) and not (Leff == 4 and k % 4):
                used_tiled += gpu_emulate.last_kernel.startswith("tiled")
                expected_tiled += 1
    assert expected_tiled > 10 and used_tiled >= 0.8 * expected_tiled, (used_tiled, expected_tiled)


@pytest.mark.parametrize("p", [GFX950_16BIT, CDNA3_16BIT], ids=["gfx950", "cdna3"])
def test_tiled_rd_accumulator_sweep(mm, p):
    # the accumulator's exponent swept from far below to far above the products', both signs, zeros among the operands
    rng = np.random.default_rng(81)
    for ta, lo in ((fm.FP16, 13), (fm.BF16, 125)):
        nb, m, n, k = 6, 32, 32, 8
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, lo, lo + 4)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), ta, lo, lo + 4)
        A = synth.sprinkle(rng, A, np.array([0, 0x8000], dtype=A.dtype), 0.05)
        for c_exp in ((60, 100), (100, 126), (120, 134), (130, 150), (148, 162), (0, 2), (250, 254)):
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, *c_exp)
            for rho in (RNE, RZ):
                q = p.with_(out_round=rho)
                want, _ = o2lib.emulate_mma(q, A, B, C, ta, ta)
                assert_same(gpu_emulate(mm, q, A, B, C, ta, ta), want, "acc sweep %s %s" % (c_exp, q))
                assert gpu_emulate.last_kernel.startswith("tiled 32x32"), gpu_emulate.last_kernel


def test_tiled_rd_same_sign_products_far_below(mm):
    # all products positive and at one exponent, accumulator 20..34 places above: the sum drops out at the stated distance
    rng = np.random.default_rng(82)
    nb, m, n, k = 4, 16, 16, 16
    A = (synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP16, 16, 16) & 0x7FFF).astype(np.uint16)
    B = (synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP16, 16, 16) & 0x7FFF).astype(np.uint16)
    for shift in range(20, 35):
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 127 + 2 + shift, 127 + 2 + shift)
        for p in (GFX950_16BIT, CDNA3_16BIT, GFX950_16BIT.with_(sum_drop_distance=25)):
            want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
            assert_same(gpu_emulate(mm, p, A, B, C, fm.FP16, fm.FP16), want, "far below %d %s" % (shift, p))


def test_tiled_rd_cancellation_and_ties(mm):
    rng = np.random.default_rng(83)
    nb, m, n, k = 6, 16, 16, 16
    A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP16, 10, 20)
    B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP16, 10, 20)
    A[:, :, 1::2] = A[:, :, 0::2] ^ 0x8000
    B[:, :, 1::2] = B[:, :, 0::2]
    flip = rng.random(B.shape) < 0.05
    B = np.where(flip, B ^ 1, B).astype(np.uint16)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 90, 140)
    for L in (4, 8, 16):
        for base in (GFX950_16BIT, CDNA3_16BIT):
            for F2 in (24, 31):
                for rho in (RNE, RZ):
                    p = base.with_(group_len=L, frac_bits2=F2, out_round=rho)
                    want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
                    assert_same(gpu_emulate(mm, p, A, B, C, fm.FP16, fm.FP16), want, "cancel %s" % (p,))


def test_tiled_rd_bf16_product_overflow(mm):
    # products at and above 2^128 count as infinities in this mode (Sec. 4.2): whole tiles of large bf16 operands
    rng = np.random.default_rng(84)
    nb, m, n, k = 3, 16, 16, 16
    A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.BF16, 185, 195)
    B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.BF16, 185, 195)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 200, 254)
    for p in (GFX950_16BIT, CDNA3_16BIT):
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)
        got = gpu_emulate(mm, p, A, B, C, fm.BF16, fm.BF16)
        assert_same(got, want, "overflow %s" % (p,))
        assert ((want & 0x7F800000) == 0x7F800000).mean() > 0.2     # the case does produce infinities / NaN


# ------------------------------------------------------------------ split groups (GTR-FDPA and the halves variant)
from oracle.fdpa import SPLIT_EVEN_ODD, SPLIT_HALVES, SPLIT_QUARTERS, C_AFTER_RD_EVEN_ODD

GFX950_FP8 = ModelParams(group_len=16, frac_bits=13, frac_bits_merge=24, frac_bits_acc=24, frac_bits2=31, c_mode=C_AFTER_RD,
                         split=SPLIT_HALVES, acc_special_truncation=True, skip_zero_terms=True, f2_at_leading_bit=True,
                         zero_result_positive=True, sum_drop_distance=28, nan_bits=0xFFC00000)
CDNA3_FP8 = ModelParams(group_len=16, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD_EVEN_ODD)
SPLIT_PAIRS = [(fm.E4M3, fm.E4M3), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.FP16), (fm.E4M3, fm.FP16)]


@pytest.mark.parametrize("ta,tb", SPLIT_PAIRS)
def test_tiled_split_parameter_sweep(mm, ta, tb):
    rng = np.random.default_rng(7000 + 8 * ta + tb)
    used_tiled = expected_tiled = 0
    for (m, n, k, nb) in SHAPES:
        for mode in ("narrow", "full", "special", "zeros"):
            Ls = [L for L in (8, 16, 32) if k % L == 0]
            if not Ls:
                continue
            L = int(rng.choice(Ls))
            p = random_rd_params(rng, k).with_(group_len=L, split=int(rng.choice([SPLIT_EVEN_ODD, SPLIT_HALVES] + ([SPLIT_QUARTERS] * 2 if L >= 16 else []))),
                                               frac_bits=int(rng.choice([5, 13, 20, 24])), frac_bits_merge=int(rng.choice([0, 13, 24, 28])))
            fc = p.frac_bits_acc or p.frac_bits
            p = p.with_(frac_bits2=min(p.frac_bits2, fc + 40))
            A, B, C = operands(rng, ta, tb, nb, m, n, k, "narrow" if mode == "zeros" else mode)
            if mode == "zeros":
                A = synth.sprinkle(rng, A, np.array([0, 1 << (A.dtype.itemsize * 8 - 1)], dtype=A.dtype), 0.3)
                A[0, 0, :] = 0
                A[0, 1, : k // 2] = 0                       # one whole half without a live term
                A[1 % nb, 3, : 3 * (k // 4)] = 0            # three quarters of every group of the row
                A[0, 2, 0::2] = 0                           # all even products zero
                C = np.where(rng.random(C.shape) < 0.3, np.uint32(0x80000000), C).astype(np.uint32)
            print("tiled split", ta, tb, (m, n, k, nb), mode, p, flush=True)
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert_same(got, want, "tiled split %s %s %s %s" % ((m, n, k, nb), mode, p, gpu_emulate.last_kernel))
            fast_shape = (m % 16 == 0 and n % 16 == 0 and k % 16 == 0) or (m % 32 == 0 and n % 32 == 0 and k % 8 == 0)
            if fast_shape and not (p.group_len == 32 and k % 32) and not (p.group_len == 16 and k % 16):
                used_tiled += gpu_emulate.last_kernel.startswith("tiled")
                expected_tiled += 1
    assert expected_tiled > 10 and used_tiled >= 0.7 * expected_tiled, (used_tiled, expected_tiled)


@pytest.mark.parametrize("p", [GFX950_FP8, CDNA3_FP8], ids=["gfx950", "cdna3"])
def test_tiled_split_presets_on_instruction_tiles(mm, p):
    rng = np.random.default_rng(91)
    for ta, tb in ((fm.E4M3, fm.E4M3), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2)):
        for mode in ("narrow", "full", "special"):
            A, B, C = operands(rng, ta, tb, 33, 16, 16, 32, mode)
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            assert_same(gpu_emulate(mm, p, A, B, C, ta, tb), want, "split preset %s %s" % (mode, p))
            assert gpu_emulate.last_kernel.startswith("tiled 16x16"), gpu_emulate.last_kernel
        # accumulator far above / below the products
        A, B, _ = operands(rng, ta, tb, 9, 16, 16, 32, "narrow")
        for c_exp in ((60, 100), (120, 134), (140, 165), (0, 2)):
            C = synth.narrow_exponent_bits(rng, (9, 16, 16), fm.FP32, *c_exp)
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            assert_same(gpu_emulate(mm, p, A, B, C, ta, tb), want, "split preset c %s %s" % (c_exp, p))


@pytest.mark.parametrize("ta,tb", [(fm.BF16, fm.BF16), (fm.BF16, fm.FP16), (fm.E5M2, fm.BF16)])
def test_tiled_rd_products_around_the_overflow_threshold(mm, ta, tb):
    # Sec. 4.2: a finite product of 2^128 and more counts as an infinity.  Exponents chosen so that a group's largest
    # product lies a few binary places either side of 2^128: groups that only might overflow, groups that do, with
    # both signs (NaN), next to NaN / infinity operands and accumulators, with and without the input flush
    rng = np.random.default_rng(4242 + 8 * ta + tb)
    nb, m, n, k = 4, 32, 32, 32
    hi_a = {fm.BF16: (183, 191), fm.E5M2: (24, 30)}[ta]
    hi_b = {fm.BF16: (183, 191), fm.FP16: (24, 30)}[tb]
    if ta != fm.BF16:
        hi_b = (232, 240)              # the partner of a narrow-range type carries the large exponent
    if tb != fm.BF16:
        hi_a = (232, 240)
    for trial in range(6):
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *hi_a)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *hi_b)
        if trial % 2:                                   # mostly small values, a few large ones per group
            small_a = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *({fm.BF16: (100, 130), fm.E5M2: (8, 20)}[ta]))
            small_b = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *({fm.BF16: (100, 130), fm.FP16: (8, 20)}[tb]))
            A = np.where(rng.random(A.shape) < 0.1, A, small_a)
            B = np.where(rng.random(B.shape) < 0.1, B, small_b)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 100, 254)
        if trial >= 4:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.01)
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.01)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.01)
        for p in (GFX950_16BIT, CDNA3_16BIT, CDNA3_16BIT.with_(ftz_in=True)):
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert gpu_emulate.last_kernel.startswith("tiled"), gpu_emulate.last_kernel
            assert_same(got, want, "overflow threshold %d %s" % (trial, p))
        special = ((want & 0x7F800000) == 0x7F800000).mean()
        assert 0.002 < special < 0.98, special              # both kinds of outputs occur


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.FP16, fm.BF16)])
def test_four_product_shapes(mm, ta, tb):
    """32x32x4 and 16x16x4 tiles (the blocks of the four-product instructions) and odd multiples of four products, groups
    of four: the tiled kernels stage one quad of k per row; both the fused and the round-down modes."""
    from oracle.fdpa import C_IN_GROUP
    from oracle.fdpa import emulate_mma as o1_emulate
    rng = np.random.default_rng(5200 + 8 * ta + tb)
    tiled = cases = 0
    for (m, n, k, nb) in ((32, 32, 4, 7), (16, 16, 4, 21), (16, 16, 12, 5), (32, 32, 20, 3)):
        for mode in ("narrow", "full", "special"):
            for cm in (C_IN_GROUP, C_AFTER_RD):
                if cm == C_AFTER_RD:
                    p = random_rd_params(rng, k).with_(group_len=4)
                else:
                    p = ModelParams(group_len=4, frac_bits=int(rng.choice([3, 13, 24, 25, 27, 28])), c_mode=cm, out_round=int(rng.integers(0, 2)),
                                    ftz_in=bool(rng.integers(0, 4) == 0), ftz_out=bool(rng.integers(0, 4) == 0))
                A, B, C = operands(rng, ta, tb, nb, m, n, k, mode)
                print("four products", ta, tb, (m, n, k, nb), mode, p, flush=True)
                want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
                got = gpu_emulate(mm, p, A, B, C, ta, tb)
                what = "four products %s %s %s %s" % ((m, n, k, nb), mode, p, gpu_emulate.last_kernel)
                assert_same(got, want, what)
                cases += 1
                tiled += "kc=4" in gpu_emulate.last_kernel
                if cm == C_IN_GROUP:
                    assert "kc=4 L=4" in gpu_emulate.last_kernel, what
                # a few outputs against the rational form
                for (t, i, j) in [(nb - 1, m - 1, n - 1)] + [(int(rng.integers(nb)), int(rng.integers(m)), int(rng.integers(n))) for _ in range(3)]:
                    one = o1_emulate(p, A[t:t + 1, i:i + 1, :], B[t:t + 1, j:j + 1, :], C[t:t + 1, i:i + 1, j:j + 1], ta, tb)[0, 0, 0]
                    assert got[t, i, j] == one, "%s: output %s: got %08x, the rational form gives %08x" % (what, (t, i, j), got[t, i, j], one)
    assert tiled >= 0.7 * cases, (tiled, cases)          # (some of the random round-down variations run in the general kernel)
