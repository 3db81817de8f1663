"""GPU tests of block-scaled operation (paper Algorithm "ST-FDPA"): mmaemu_emulate_mma_scaled against the CPU oracle, bit
for bit, and the register layout of the block-scaled native instruction."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from paper_2511_10909_amd import synth
from gpu_utils import to_dev, dev_empty, to_host
from test_gpu_parity import mm, assert_same, _small_int_codes, NP  # noqa: F401


def gpu_emulate_scaled(mm, p, A, B, C, SA, SB, block, ta, tb):
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(group_len=p.group_len, frac_bits=p.frac_bits, frac_bits2=p.frac_bits2, c_mode=p.c_mode, out_round=p.out_round,
                        ftz_in=p.ftz_in, ftz_out=p.ftz_out, nan_bits=p.nan_bits, split=p.split,
                        acc_special_truncation=p.acc_special_truncation, frac_bits_merge=p.frac_bits_merge,
                        frac_bits_acc=p.frac_bits_acc, f2_at_leading_bit=p.f2_at_leading_bit,
                        skip_zero_terms=p.skip_zero_terms, zero_result_positive=p.zero_result_positive,
                        sum_drop_distance=p.sum_drop_distance, out_mant_bits=p.out_mant_bits,
                        wide_products=p.wide_products, rd_toward_zero=p.rd_toward_zero)
    try:
        dD = dev_empty((nb, m, n), np.uint32)
        mm.emulate_mma_scaled(h, to_dev(A.astype(NP[ta])), to_dev(B.astype(NP[tb])), to_dev(C.astype(np.uint32)), dD,
                              to_dev(SA.astype(np.uint8)), to_dev(SB.astype(np.uint8)), block, m, n, k, nb, (ta, tb, fm.FP32, fm.FP32))
        return to_host(dD, np.uint32)
    finally:
        mm.model_destroy(h)


@pytest.mark.parametrize("ta,tb", [(fm.E4M3, fm.E4M3), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16)])
def test_scaled_emulation_matches_oracle(mm, ta, tb):
    rng = np.random.default_rng(3300 + 8 * ta + tb)
    for trial in range(14):
        block = int(rng.choice([8, 16, 32]))
        k = block * int(rng.integers(1, 5))
        L = int(rng.choice([x for x in (2, 4, 8, 16, 32, 0) if x == 0 or k % x == 0]))
        mode = int(rng.choice([C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([8, 13, 24, 25, 30])), c_mode=mode, out_round=int(rng.integers(0, 2)),
                        skip_zero_terms=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)))
        if mode == C_AFTER_RD:
            p = p.with_(frac_bits2=31, split=int(rng.integers(0, 4 if (L or k) % 4 == 0 else 3)) if (L or k) % 2 == 0 else 0, f2_at_leading_bit=bool(rng.integers(0, 2)),
                        acc_special_truncation=bool(rng.integers(0, 2)), sum_drop_distance=int(rng.choice([0, 28])),
                        wide_products=bool(rng.integers(0, 2)))
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 20)), int(rng.integers(1, 20))
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 60, 200)
        lo, hi = [(90, 165), (40, 215)][trial % 2]
        SA = rng.integers(lo, hi, size=(nb, m, k // block)).astype(np.uint8)
        SB = rng.integers(lo, hi, size=(nb, n, k // block)).astype(np.uint8)
        if trial % 4 == 0:
            SA[0, 0, 0] = 0xFF
            SB[-1, -1, 0] = 0
            SA[-1, 0, -1] = 254
        want, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, block, ta, tb)
        got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, block, ta, tb)
        assert_same(got, want, "scaled %s block %d" % (p, block))
        assert mm.last_kernel().startswith("general, block-scaled")


TILED_SHAPES = [(3, 16, 16, 64), (2, 32, 32, 64), (1, 64, 64, 128), (5, 16, 16, 128), (1, 64, 128, 32), (1, 2048, 1024, 32)]


@pytest.mark.parametrize("ta,tb", [(fm.E4M3, fm.E4M3), (fm.E5M2, fm.E4M3), (fm.E4M3, fm.FP16), (fm.FP16, fm.FP16)])
def test_scaled_tiled_kernels_match_oracle(mm, ta, tb):
    # groups inside one block of scales: the tiled kernels (value mode 3), every accumulation mode and split
    rng = np.random.default_rng(5100 + 8 * ta + tb)
    for trial in range(18):
        nb, m, n, k = TILED_SHAPES[trial % len(TILED_SHAPES)]
        if m * n * k * nb > (1 << 24) and trial >= len(TILED_SHAPES):
            nb, m, n, k = 2, 32, 32, 64
        block = int(rng.choice([b for b in (16, 32, 64) if k % b == 0]))
        L = int(rng.choice([x for x in (4, 8, 16, 32) if block % x == 0 and x <= m]))     # (16 x 16 tiles are staged 16 k at a time)
        mode = [C_IN_GROUP, C_AFTER_RD, C_AFTER_RD, C_AFTER_EXACT][trial % 4]
        F = int(rng.choice([13, 24, 25]))
        p = ModelParams(group_len=L, frac_bits=F, c_mode=mode, out_round=int(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)))
        if mode == C_AFTER_RD:
            p = p.with_(frac_bits2=31, split=int(rng.integers(0, 4 if L >= 16 else 3)) if L >= 8 else 0, f2_at_leading_bit=bool(rng.integers(0, 2)),
                        acc_special_truncation=bool(rng.integers(0, 2)), sum_drop_distance=int(rng.choice([0, 28])),
                        wide_products=bool(rng.integers(0, 2)), skip_zero_terms=bool(rng.integers(0, 2)),
                        zero_result_positive=bool(rng.integers(0, 2)))
            if p.split:
                p = p.with_(frac_bits_merge=int(rng.choice([0, 24])), frac_bits_acc=int(rng.choice([0, 24])))
        A = synth.random_bits(rng, (nb, m, k), ta)
        B = synth.random_bits(rng, (nb, n, k), tb)
        if trial % 3 == 0:          # zeros with large exponents next to them, no specials: the fast route throughout
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 1, 14)
            A[rng.random(A.shape) < 0.2] = 0
        lo, hi = [(115, 140), (30, 225), (0, 256)][trial % 3]
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, max(1, lo + lo - 127 - 30), min(254, hi + hi - 127 + 30))
        SA = rng.integers(lo, hi, size=(nb, m, k // block)).astype(np.uint8)
        SB = rng.integers(lo, hi, size=(nb, n, k // block)).astype(np.uint8)
        want, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, block, ta, tb)
        print("scaled tiled", trial, (nb, m, n, k), block, p, flush=True)
        got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, block, ta, tb)
        assert mm.last_kernel().startswith("tiled") and "vm=3" in mm.last_kernel(), mm.last_kernel()
        assert_same(got, want, "scaled tiled %s block %d" % (p, block))
        assert len(np.unique(want)) > want.size // 64


def test_scaled_groups_across_blocks_use_the_general_kernel(mm):
    rng = np.random.default_rng(8)
    p = ModelParams(group_len=32, frac_bits=24)
    A = synth.random_bits(rng, (1, 32, 64), fm.E4M3)
    B = synth.random_bits(rng, (1, 32, 64), fm.E4M3)
    C = synth.narrow_exponent_bits(rng, (1, 32, 32), fm.FP32, 100, 150)
    SA = rng.integers(110, 140, size=(1, 32, 4)).astype(np.uint8)
    SB = rng.integers(110, 140, size=(1, 32, 4)).astype(np.uint8)
    want, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, 16, fm.E4M3, fm.E4M3)
    got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, 16, fm.E4M3, fm.E4M3)
    assert mm.last_kernel().startswith("general, block-scaled")
    assert_same(got, want, "group of two blocks")


def test_wide_products_without_scales(mm):
    # BF16 products far beyond 2^128 that keep their value: the general kernel's integer range, not the tiled kernels
    from test_gpu_parity import gpu_emulate
    rng = np.random.default_rng(41)
    for trial in range(10):
        L = int(rng.choice([4, 8, 16]))
        p = ModelParams(group_len=L, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD, wide_products=True, split=int(rng.integers(0, 3)),
                        skip_zero_terms=bool(rng.integers(0, 2)), out_round=int(rng.integers(0, 2)))
        nb, m, n, k = 2, 17, 9, 32
        A = synth.narrow_exponent_bits(rng, (nb, m, k), fm.BF16, 172, 191)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), fm.BF16, 172, 191)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 200, 254)
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.BF16, fm.BF16)
        got = gpu_emulate(mm, p, A, B, C, fm.BF16, fm.BF16)
        assert_same(got, want, "wide products %s" % (p,))
        assert mm.last_kernel().startswith("general")
        assert len(np.unique(want)) > 8


def test_scaled_argument_errors(mm):
    import torch
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    h = mm.model_create(group_len=8, frac_bits=24)
    dt = (mm.E4M3, mm.E4M3, mm.FP32, mm.FP32)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma_scaled(h, z, z, z, z, z, z, 32, 1, 1, 48, 1, dt)
    assert ei.value.status == 3
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma_scaled(h, z, z, z, z, None, z, 32, 1, 1, 64, 1, dt)
    assert ei.value.status == 1
    mm.model_destroy(h)
    h = mm.model_create(group_len=4, family=mm.FAMILY_FTZ_ADDMUL)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma_scaled(h, z, z, z, z, z, z, 32, 1, 1, 64, 1, dt)
    assert ei.value.status == 2
    mm.model_destroy(h)


@pytest.mark.parametrize("instr", list(range(10, 35)) + list(range(43, 68)))
def test_scaled_mfma_register_layout(mm, instr):
    # small-integer operands and scales of 2^-4 .. 2^4: every arithmetic is exact, so any mistake in the operand,
    # scale or result register layout shows, whatever the instruction does inside
    info = mm.mfma_info(instr)
    ta, tb = info["a"], info["b"]
    M = info["m"]
    assert (info["m"], info["n"], info["k"]) == ((16, 16, 128) if instr < 43 else (32, 32, 64))
    rng = np.random.default_rng(instr)
    for k in ((128, 64, 32) if M == 16 else (64, 32)):
        nb = 9
        A, av = _small_int_codes(rng, (nb, M, k), ta)
        B, bv = _small_int_codes(rng, (nb, M, k), tb)
        SA = rng.integers(123, 132, size=(nb, M, k // 32)).astype(np.uint8)
        SB = rng.integers(123, 132, size=(nb, M, k // 32)).astype(np.uint8)
        cv = rng.integers(-100, 100, size=(nb, M, M))
        C = cv.astype(np.float32).view(np.uint32)
        want = cv.astype(np.float64)
        for q in range(k // 32):
            blockdot = np.einsum("bik,bjk->bij", av[:, :, 32 * q:32 * q + 32], bv[:, :, 32 * q:32 * q + 32]).astype(np.float64)
            want = want + blockdot * 2.0 ** (SA[:, :, q].astype(np.int64)[:, :, None] + SB[:, :, q].astype(np.int64)[:, None, :] - 254)
        want = want.astype(np.float32).view(np.uint32)
        dD = dev_empty((nb, M, M), np.uint32)
        print("scaled mfma", instr, k, flush=True)
        mm.mfma_probe_scaled(instr, to_dev(A), to_dev(B), to_dev(C), dD, to_dev(SA), to_dev(SB), k, nb)
        got = to_host(dD, np.uint32)
        assert_same(np.where(got == 0x80000000, 0, got), want, "scaled mfma layout")
