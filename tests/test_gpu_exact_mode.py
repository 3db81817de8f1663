"""GPU parity of c_mode = C_EXACT (Algorithm "E-FDPA": exact sum of the group's products and the accumulator, one
conversion) against the rational-arithmetic oracle, bit for bit: every operand type, whole exponent ranges (BF16 and
FP32 sums span more than 500 binary places), special values, chained groups, both conversions and both flushes."""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm
from oracle.fdpa import ModelParams, C_EXACT
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from helpers import f32_bits, fp16_bits, bf16_bits
from o1_jobs import run_pool
from test_gpu_parity import mm, gpu_emulate, assert_same  # noqa: F401

PAIRS = [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E5M2), (fm.TF32, fm.TF32), (fm.FP32, fm.FP32),
         (fm.E2M3, fm.E2M1), (fm.FP16, fm.BF16), (fm.E3M2, fm.E4M3)]


def test_exact_mode_matches_the_rational_oracle(mm):
    rng = np.random.default_rng(4242)
    gpu, jobs, names = [], [], []
    for idx, (ta, tb) in enumerate(PAIRS):
        for variant in range(3):
            L = [4, 2, 16][variant]
            k = L * (1 + (idx + variant) % 3)
            p = ModelParams(group_len=L if variant != 2 else 0, c_mode=C_EXACT, out_round=RZ if variant == 1 else RNE,
                            ftz_in=variant == 1, ftz_out=variant == 2, nan_bits=0x7FFFFFFF if variant == 0 else 0x7FC00000)
            if variant == 2:
                k = 16
            nb, m, n = 2, 17, 13
            A = synth.random_bits(rng, (nb, m, k), ta)             # whole exponent range of the type
            B = synth.random_bits(rng, (nb, n, k), tb)
            if variant == 0:                                        # near-cancelling sums: pairs of equal magnitude, opposite sign
                A[:, :, 1::2] = A[:, :, 0::2] ^ (1 << (synth.WIDTH[ta] - 1) if ta not in (fm.TF32, fm.FP32) else 1 << 31)
                B[:, :, 1::2] = B[:, :, 0::2]
                B[:, ::3, 1] ^= 1                                   # ... up to a last place here and there
            C = synth.random_bits(rng, (nb, m, n), fm.FP32) if variant else synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 1, 254)
            if variant == 1:
                A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.02)
                C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.03)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert gpu_emulate.last_kernel == "e-fdpa, one thread per output", gpu_emulate.last_kernel
            # in place the accumulators do not outlive the first launch: the general kernel, which finishes every output itself
            in_place = gpu_emulate(mm, p, A, B, C, ta, tb, in_place=True)
            assert gpu_emulate.last_kernel == "general, exact sum", gpu_emulate.last_kernel
            assert_same(in_place, got, "in place against out of place, types %d x %d, variant %d" % (ta, tb, variant))
            gpu.append(got)
            jobs.append((dataclasses.asdict(p), A, B, C, ta, tb, None, None, 0))
            names.append("types %d x %d, variant %d" % (ta, tb, variant))
    want = run_pool(jobs, workers=12)
    bad = []
    for name, g, w in zip(names, gpu, want):
        if not np.array_equal(g, w):
            i = tuple(np.argwhere(g != w)[0])
            bad.append("%s: %d of %d differ, first at %s: gpu %08x, oracle %08x" % (name, int((g != w).sum()), g.size, i, int(g[i]), int(w[i])))
    assert not bad, "\n".join(bad)
    assert sum(g.size for g in gpu) > 10000


def test_worked_example_and_limits_on_the_gpu(mm):
    a = [-2.0 ** 13, -0.5, -0.25, -0.125] + [0.0] * 12
    b = [2.0 ** 10, 1.0, 1.0, 1.0] + [0.0] * 12
    C = np.array([[[f32_bits(2.0 ** 23)]]], dtype=np.uint32)
    for enc, t, L in ((fp16_bits, fm.FP16, 4), (bf16_bits, fm.BF16, 2)):
        A = np.array([[[enc(x) for x in a]]], dtype=np.uint16)
        B = np.array([[[enc(x) for x in b]]], dtype=np.uint16)
        got = gpu_emulate(mm, ModelParams(group_len=L, c_mode=C_EXACT), A, B, C, t, t)
        assert int(got[0, 0, 0]) == f32_bits(-0.875)               # Sec. 5: the CDNA1 entries of the table
        from paper_2511_10909_amd import presets
        kw = presets.PAPER[("cdna1", "fp16" if t == fm.FP16 else "bf16")]
        assert kw["c_mode"] == mm.C_EXACT and kw["group_len"] == L
    # the extremes of the 640-bit accumulator: the largest and the smallest FP32 products in one group
    big, tiny = 0x7F7FFFFF, 0x00000001
    A = np.array([[[big, tiny, big, 0x80000001]]], dtype=np.uint32)
    B = np.array([[[big, tiny, 0xFF7FFFFF, tiny]]], dtype=np.uint32)
    Cz = np.zeros((1, 1, 1), dtype=np.uint32)
    got = gpu_emulate(mm, ModelParams(group_len=4, c_mode=C_EXACT), A, B, Cz, fm.FP32, fm.FP32)
    assert int(got[0, 0, 0]) == 0                                   # everything cancels exactly: +0.0
    got = gpu_emulate(mm, ModelParams(group_len=2, c_mode=C_EXACT), A[:, :, :2], B[:, :, :2], Cz, fm.FP32, fm.FP32)
    assert int(got[0, 0, 0]) == 0x7F800000                          # max * max overflows in the conversion


def test_exact_mode_argument_checks(mm):
    import torch
    z = torch.zeros(64, dtype=torch.int32, device="cuda")
    h = mm.model_create(group_len=4, c_mode=mm.C_EXACT)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, z, z, z, z, 1, 1, 4, 1, (mm.FP16, mm.FP16, mm.FP16, mm.FP16))
    assert ei.value.status == 2
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma_scaled(h, z, z, z, z, z, z, 4, 1, 1, 4, 1, (mm.E4M3, mm.E4M3, mm.FP32, mm.FP32))
    assert ei.value.status == 2
    mm.model_destroy(h)
    with pytest.raises(mm.MmaemuError):
        mm.model_create(group_len=4, c_mode=mm.C_EXACT, frac_bits2=31)


def _exact_cases(rng):
    """(name, params, A, B, C, ta, tb) on whole 16x16 blocks: narrow exponents (the sum stays within the pair of binary64
    numbers the block kernel keeps), whole ranges (BF16 / TF32 groups leave it and take the integer routine), cancelling
    pairs, special values."""
    out = []
    pairs = [p for p in PAIRS if fm.FP32 not in p]
    for idx, (ta, tb) in enumerate(pairs):
        for variant in range(4):
            L = [4, 2, 16, 64][variant]
            k = [12, 6, 48, 64][variant]
            p = ModelParams(group_len=L, c_mode=C_EXACT, out_round=RZ if variant in (1, 3) else RNE, ftz_in=variant == 1, ftz_out=variant == 2,
                            nan_bits=0x7FFFFFFF if variant == 0 else 0x7FC00000, out_mant_bits=13 if variant == 3 else 23)
            nb, m, n = 2, 32, 16
            if variant in (0, 3):
                A = synth.random_bits(rng, (nb, m, k), ta)
                B = synth.random_bits(rng, (nb, n, k), tb)
            else:
                lo_hi = {fm.BF16: (100, 150), fm.TF32: (100, 150), fm.FP16: (1, 30), fm.E4M3: (0, 15), fm.E5M2: (0, 30), fm.E2M3: (0, 3), fm.E3M2: (0, 7), fm.E2M1: (0, 3)}
                A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo_hi[ta])
                B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *lo_hi[tb])
            if variant == 0:
                A[:, :, 1::2] = A[:, :, 0::2] ^ (1 << (synth.WIDTH[ta] - 1) if ta != fm.TF32 else 1 << 31)
                B[:, :, 1::2] = B[:, :, 0::2]
                B[:, ::3, 1] ^= 1
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 90, 160) if variant in (1, 2) else synth.random_bits(rng, (nb, m, n), fm.FP32)
            if variant == 1:
                A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.02)
                C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.03)
                C[0, 0, :4] = [0, 0x80000000, 1, 0x80000001]                  # zeros and subnormal accumulators
            out.append(("types %d x %d, variant %d" % (ta, tb, variant), p, A, B, C, ta, tb))
    return out


def test_exact_mode_in_blocks_matches_the_rational_oracle(mm):
    rng = np.random.default_rng(4343)
    gpu, jobs, names = [], [], []
    for name, p, A, B, C, ta, tb in _exact_cases(rng):
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert gpu_emulate.last_kernel == "e-fdpa, 16x16 blocks through LDS", gpu_emulate.last_kernel
        # the same problem without B's last row (n = 15), in place, runs in the general kernel: the two routes agree
        via_general = gpu_emulate(mm, p, A, B[:, :-1], C[:, :, :-1], ta, tb, in_place=True)
        assert gpu_emulate.last_kernel == "general, exact sum"
        assert_same(got[:, :, :-1], via_general, "block kernel against the general kernel, " + name)
        # in place the block kernel finishes every output itself; elsewhere it marks those it cannot finish for a second
        # launch, with a NaN pattern that moves out of the way of the model's own
        in_place = gpu_emulate(mm, p, A, B, C, ta, tb, in_place=True)
        assert gpu_emulate.last_kernel == "e-fdpa, 16x16 blocks through LDS, in place", gpu_emulate.last_kernel
        assert_same(in_place, got, "in place against out of place, " + name)
        if "variant 0" in name:
            q = dataclasses.replace(p, nan_bits=0x7FEDCBA9)
            other = gpu_emulate(mm, q, A, B, C, ta, tb)
            assert_same(other, np.where(got == p.nan_bits, np.uint32(q.nan_bits), got), "another NaN pattern, " + name)
        keep = slice(0, 1) if "variant 3" in name else slice(0, 2)           # (the oracle on one tile of the longest case)
        gpu.append(got[keep, ::3])
        jobs.append((dataclasses.asdict(p), A[keep, ::3], B[keep], C[keep, ::3], ta, tb, None, None, 0))
        names.append(name)
    want = run_pool(jobs, workers=12)
    bad = []
    for name, g, w in zip(names, gpu, want):
        if not np.array_equal(g, w):
            i = tuple(np.argwhere(g != w)[0])
            bad.append("%s: %d of %d differ, first at %s: gpu %08x, oracle %08x" % (name, int((g != w).sum()), g.size, i, int(g[i]), int(w[i])))
    assert not bad, "\n".join(bad)


def test_exact_mode_blocks_on_ordinary_data_at_size(mm):
    # N(0,1)-like operands on many tiles: every sum stays within the pair of binary64 numbers; against the general kernel
    rng = np.random.default_rng(4344)
    for ta, L, k in ((fm.FP16, 4, 16), (fm.BF16, 2, 16), (fm.E4M3, 16, 32)):
        nb, m, n = 64, 32, 32
        lo_hi = {fm.BF16: (117, 130), fm.FP16: (5, 18), fm.E4M3: (2, 10)}[ta]
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo_hi)
        B = synth.narrow_exponent_bits(rng, (nb, n, k), ta, *lo_hi)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 117, 130)
        for rho in (RNE, RZ):
            p = ModelParams(group_len=L, c_mode=C_EXACT, out_round=rho)
            got = gpu_emulate(mm, p, A, B, C, ta, ta)
            assert gpu_emulate.last_kernel == "e-fdpa, 16x16 blocks through LDS"
            ref = gpu_emulate(mm, p, A, B[:, :-1], C[:, :, :-1], ta, ta, in_place=True)
            assert gpu_emulate.last_kernel == "general, exact sum"
            one = gpu_emulate(mm, p, A, B[:, :-1], C[:, :, :-1], ta, ta)
            assert gpu_emulate.last_kernel == "e-fdpa, one thread per output"
            assert_same(one, ref, "one thread per output, types %d L %d rho %d" % (ta, L, rho))
            assert_same(got[:, :, :-1], ref, "types %d L %d rho %d" % (ta, L, rho))
