"""GPU parity of the tiled (fast-path) emulation kernels against the CPU oracle, bit for bit.

Shapes are chosen so that the library takes its tiled kernels (whole 16x16 / 32x32 tiles, or
64x64 blocks of a larger problem) with several workgroups and a ragged last workgroup; operand
exponents are drawn both narrowly (every element on the fast route) and over the whole format
(elements outside the fast route's range, NaN and infinities mixed in)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from test_gpu_parity import gpu_emulate, assert_same, mm  # noqa: F401  (fixture)

PAIRS = [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3),
         (fm.E4M3, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16), (fm.BF16, fm.E4M3), (fm.E5M2, fm.FP16)]
SHAPES = [(16, 16, 16, 37), (16, 16, 32, 5), (32, 32, 8, 9), (32, 32, 16, 3), (64, 64, 64, 1), (128, 64, 96, 2),
          (64, 192, 32, 1), (96, 32, 24, 2), (48, 80, 16, 3)]
MID = {fm.FP16: (1, 30), fm.BF16: (100, 150), fm.E4M3: (0, 15), fm.E5M2: (0, 30)}


def operands(rng, ta, tb, nb, m, n, k, mode):
    if mode == "narrow":      # every element inside the fast route's range
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *MID[ta])
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *MID[tb])
        if ta == fm.E4M3:
            A = np.where((A & 0x7F) == 0x7F, A & 0x80, A).astype(A.dtype)
        if tb == fm.E4M3:
            B = np.where((B & 0x7F) == 0x7F, B & 0x80, B).astype(B.dtype)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 100, 150)
        zero = rng.random((nb, m, n)) < 0.1
        C = np.where(zero, 0, C).astype(np.uint32)
    elif mode == "full":      # whole format, finite
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.random_bits(rng, (nb, m, n), fm.FP32)
    else:                     # narrow with special values and zeros sprinkled in
        A, B, C = operands(rng, ta, tb, nb, m, n, k, "narrow")
        A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.01)
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.01)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.02)
    return A, B, C


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_tiled_parameter_sweep(mm, ta, tb):
    rng = np.random.default_rng(3000 + 8 * ta + tb)
    trial = 0
    used_tiled = expected_tiled = 0
    for (m, n, k, nb) in SHAPES:
        for mode in ("narrow", "full", "special"):
            for rep in range(2):
                trial += 1
                Ls = [L for L in (4, 8, 16, 32, 0, 64, 24, 2) if (L == 0 or k % L == 0 or L > k)]
                L = int(rng.choice(Ls))
                F = int(rng.choice([0, 3, 13, 14, 16, 20, 24, 25, 27, 28, 29, 30, 32, 35, 40]))
                p = ModelParams(group_len=L, frac_bits=F, c_mode=int(rng.integers(0, 2)),
                                out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 4) == 0),
                                ftz_out=bool(rng.integers(0, 4) == 0))
                if p.out_round == RZ and trial % 3 == 0:
                    p = p.with_(out_mant_bits=13)                # RZ-E8M13
                if p.c_mode == C_AFTER_EXACT and F + 2 + int(np.ceil(np.log2(max(k if L == 0 else min(L, k), 1)))) > 40:
                    p = p.with_(frac_bits=30)                   # limit of the C oracle for this mode
                A, B, C = operands(rng, ta, tb, nb, m, n, k, mode)
                print("tiled", ta, tb, (m, n, k, nb), mode, p, flush=True)
                want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
                got = gpu_emulate(mm, p, A, B, C, ta, tb)
                assert_same(got, want, "tiled %s %s %s" % ((m, n, k, nb), mode, p))
                Leff = k if L == 0 else min(L, k)
                fast_shape = (m % 16 == 0 and n % 16 == 0 and k % 16 == 0) or (m % 32 == 0 and n % 32 == 0 and k % 8 == 0)
                if fast_shape and Leff in (4, 8, 16, 32, k) and not (Leff == 32 and k % 32) and not (Leff == 4 and k % 4):
                    used_tiled += gpu_emulate.last_kernel.startswith("tiled")
                    expected_tiled += 1
    assert expected_tiled > 20 and used_tiled >= 0.8 * expected_tiled, (used_tiled, expected_tiled)


def test_tiled_paper_presets(mm):
    # parameter sets of the paper's Table "T-FDPA and ST-FDPA parameter selection" on whole tiles
    rng = np.random.default_rng(77)
    presets = [(fm.FP16, 4, 23, RZ, 23), (fm.FP16, 8, 24, RZ, 23), (fm.BF16, 8, 24, RZ, 23), (fm.FP16, 16, 25, RZ, 23),
               (fm.BF16, 16, 25, RZ, 23), (fm.E5M2, 16, 13, RZ, 13), (fm.E4M3, 32, 13, RZ, 13), (fm.E4M3, 32, 25, RZ, 23)]
    for t, L, F, rho, mant in presets:
        for mode in ("narrow", "special"):
            A, B, C = operands(rng, t, t, 21, 16, 16, 32, mode)
            p = ModelParams(group_len=L, frac_bits=F, out_round=rho, out_mant_bits=mant, nan_bits=0x7FFFFFFF)
            want, _ = o2lib.emulate_mma(p, A, B, C, t, t)
            assert_same(gpu_emulate(mm, p, A, B, C, t, t), want, "preset %s" % (p,))
            assert gpu_emulate.last_kernel.startswith("tiled 16x16"), gpu_emulate.last_kernel


def test_tiled_accumulator_extremes(mm):
    # accumulators near overflow, subnormal and zero, with in-range operands: conversion edge cases
    rng = np.random.default_rng(78)
    for ta, tb in ((fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2)):
        A, B, _ = operands(rng, ta, tb, 8, 16, 16, 16, "narrow")
        for c_exp in ((250, 254), (0, 3), (1, 40), (200, 254)):
            C = synth.narrow_exponent_bits(rng, (8, 16, 16), fm.FP32, *c_exp)
            for cm in (C_IN_GROUP, C_AFTER_EXACT):
                for rho in (RNE, RZ):
                    for fo in (False, True):
                        p = ModelParams(group_len=8, frac_bits=24, c_mode=cm, out_round=rho, ftz_out=fo, ftz_in=fo)
                        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
                        assert_same(gpu_emulate(mm, p, A, B, C, ta, tb), want, "extremes %s %s" % (c_exp, p))
    # all-zero operand rows with tiny accumulators (bf16: e_max far below the accumulator's range)
    A = np.zeros((4, 16, 16), dtype=np.uint16)
    B = synth.narrow_exponent_bits(rng, (4, 16, 16), fm.BF16, 100, 150)
    C = synth.narrow_exponent_bits(rng, (4, 16, 16), fm.FP32, 0, 2)
    for cm in (C_IN_GROUP, C_AFTER_EXACT):
        p = ModelParams(group_len=16, frac_bits=24, c_mode=cm)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)
        assert_same(gpu_emulate(mm, p, A, B, C, fm.BF16, fm.BF16), want, "zero rows")


def test_tiled_cancellation_and_ties(mm):
    # adversarial sums (paper Sec. 3.1 Step 4, second input family): pairs that cancel exactly or nearly,
    # so that the truncated sum is tiny against its terms and conversions hit ties
    rng = np.random.default_rng(79)
    nb, m, n, k = 6, 16, 16, 16
    A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.FP16, 10, 20)
    B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.FP16, 10, 20)
    A[:, :, 1::2] = A[:, :, 0::2] ^ 0x8000            # a_(2q+1) = -a_(2q)
    B[:, :, 1::2] = B[:, :, 0::2]                     # b_(2q+1) =  b_(2q)   -> products cancel pairwise
    flip = rng.random(B.shape) < 0.05
    B = np.where(flip, B ^ 1, B).astype(np.uint16)    # a few last-place perturbations
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 90, 140)
    for L in (4, 8, 16):
        for F in (10, 24, 27):
            for cm in (C_IN_GROUP, C_AFTER_EXACT):
                for rho in (RNE, RZ):
                    p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=rho)
                    want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
                    assert_same(gpu_emulate(mm, p, A, B, C, fm.FP16, fm.FP16), want, "cancel %s" % (p,))


def test_tiled_unaligned_pointers(mm):
    # C and D 4 bytes off a 16-byte boundary (the tiled kernels then move C/D element by element);
    # A and B 2 bytes off an 8-byte boundary (the library then takes its general kernel)
    import torch
    from gpu_utils import to_dev, to_host
    rng = np.random.default_rng(80)
    nb, m, n, k = 5, 16, 16, 16
    A, B, C = operands(rng, fm.FP16, fm.FP16, nb, m, n, k, "narrow")
    p = ModelParams(group_len=8, frac_bits=24)
    want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
    h = mm.model_create(group_len=8, frac_bits=24)
    dt = (fm.FP16, fm.FP16, fm.FP32, fm.FP32)
    dA, dB = to_dev(A), to_dev(B)
    cbuf = torch.zeros(C.size + 1, dtype=torch.int32, device="cuda")
    dbuf = torch.zeros(C.size + 1, dtype=torch.int32, device="cuda")
    cbuf[1:] = to_dev(C).flatten()
    mm.emulate_mma(h, dA, dB, cbuf[1:], dbuf[1:], m, n, k, nb, dt)
    assert mm.last_kernel().startswith("tiled")
    assert_same(to_host(dbuf[1:], np.uint32).reshape(nb, m, n), want, "C/D off by 4 bytes")
    abuf = torch.zeros(A.size + 1, dtype=torch.int16, device="cuda")
    bbuf = torch.zeros(B.size + 1, dtype=torch.int16, device="cuda")
    abuf[1:] = dA.flatten()
    bbuf[1:] = dB.flatten()
    dD = torch.zeros(C.size, dtype=torch.int32, device="cuda")
    mm.emulate_mma(h, abuf[1:], bbuf[1:], to_dev(C), dD, m, n, k, nb, dt)
    assert mm.last_kernel() == "general"
    assert_same(to_host(dD, np.uint32).reshape(nb, m, n), want, "A/B off by 2 bytes")
    mm.model_destroy(h)


@pytest.mark.parametrize("ta,tb", [(fm.BF16, fm.BF16), (fm.FP16, fm.FP16), (fm.E5M2, fm.E5M2), (fm.E4M3, fm.E5M2), (fm.BF16, fm.E5M2)])
def test_all_bit_patterns_in_the_tiled_kernels(mm, ta, tb):
    # Sec. 3.1 Step 4's third input type (random bit streams, NaN and infinities included) and Sec. 4.2: most groups hold
    # a special value, or (BF16 under TR-FDPA) a finite product of 2^128 or more.  The kernels settle those groups from
    # the staged values; every output against the C form of the oracle, a sample against the rational form.
    from oracle.fdpa import emulate_mma as o1_emulate, C_AFTER_RD
    rng = np.random.default_rng(7100 + 8 * ta + tb)
    for (m, n, k, nb, L) in ((16, 16, 32, 6, 16), (32, 32, 8, 3, 8), (64, 64, 32, 1, 4), (16, 16, 16, 9, 8)):
        A = synth.random_bits(rng, (nb, m, k), ta, finite=False)
        B = synth.random_bits(rng, (nb, n, k), tb, finite=False)
        C = np.where(rng.random((nb, m, n)) < 0.5, synth.random_bits(rng, (nb, m, n), fm.FP32, finite=False),
                     synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 100, 150)).astype(np.uint32)
        models = [ModelParams(group_len=L, frac_bits=24), ModelParams(group_len=L, frac_bits=13, c_mode=C_AFTER_EXACT, out_round=RZ, ftz_in=True, ftz_out=True),
                  ModelParams(group_len=L, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, nan_bits=0xFFC00000),
                  ModelParams(group_len=L, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, ftz_in=True, skip_zero_terms=True, f2_at_leading_bit=True,
                              zero_result_positive=True, sum_drop_distance=28)]
        for p in models:
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert gpu_emulate.last_kernel.startswith("tiled"), gpu_emulate.last_kernel
            assert_same(got, want, "all bit patterns %s %s" % ((m, n, k, nb), p))
            assert_same(got[:1, :2, :n], o1_emulate(p, A[:1, :2], B[:1], C[:1, :2], ta, tb), "rational form %s" % (p,))
            special = ((want & 0x7F800000) == 0x7F800000).mean()
            assert 0.05 < special < 0.999, special
