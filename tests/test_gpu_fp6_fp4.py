"""GPU parity on FP6 (E2M3, E3M2) and FP4 (E2M1) operands (Require lines of paper Algorithms "T-FDPA" and "ST-FDPA"):
general and tiled kernels, unscaled and block-scaled, against the CPU oracle, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from paper_2511_10909_amd import synth
from test_gpu_parity import mm, assert_same, gpu_emulate  # noqa: F401
from test_gpu_scaled import gpu_emulate_scaled

PAIRS = [(fm.E2M1, fm.E2M1), (fm.E2M3, fm.E2M3), (fm.E3M2, fm.E3M2), (fm.E2M3, fm.E2M1), (fm.E2M1, fm.E3M2),
         (fm.E4M3, fm.E2M1), (fm.E2M3, fm.E5M2), (fm.E3M2, fm.E4M3), (fm.E5M2, fm.E3M2)]


def _params(rng, L, trial):
    mode = [C_IN_GROUP, C_AFTER_RD, C_AFTER_EXACT, C_AFTER_RD][trial % 4]
    p = ModelParams(group_len=L, frac_bits=int(rng.choice([5, 13, 24, 25])), c_mode=mode, out_round=int(rng.integers(0, 2)),
                    ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)))
    if mode == C_AFTER_RD:
        p = p.with_(frac_bits2=31, split=int(rng.integers(0, 4 if L >= 16 else 3)) if L >= 8 else 0, f2_at_leading_bit=bool(rng.integers(0, 2)),
                    acc_special_truncation=bool(rng.integers(0, 2)), skip_zero_terms=bool(rng.integers(0, 2)),
                    zero_result_positive=bool(rng.integers(0, 2)), sum_drop_distance=int(rng.choice([0, 28])))
    return p


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_fp6_fp4_general_kernel(mm, ta, tb):
    rng = np.random.default_rng(3000 + 16 * ta + tb)
    for trial in range(12):
        L = int(rng.choice([2, 3, 6, 0]))
        p = _params(rng, L, trial)
        if p.split:
            p = p.with_(split=0)
        nb, m, n, k = 2, 5, 7, 12
        A, B = synth.random_bits(rng, (nb, m, k), ta), synth.random_bits(rng, (nb, n, k), tb)
        A[0, 0, :] |= 0xC0            # bits above the code are ignored
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 115, 135)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert gpu_emulate.last_kernel.startswith("general")
        assert_same(got, want, "fp6/fp4 general %s" % (p,))


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_fp6_fp4_tiled_kernels(mm, ta, tb):
    rng = np.random.default_rng(4000 + 16 * ta + tb)
    shapes = [(3, 16, 16, 64), (2, 32, 32, 64), (1, 64, 64, 128), (1, 32, 32, 8)]
    for trial in range(12):
        nb, m, n, k = shapes[trial % len(shapes)]
        L = int(rng.choice([x for x in (4, 8, 16, 32) if k % x == 0 and x <= m and x <= k]))
        p = _params(rng, L, trial)
        A, B = synth.random_bits(rng, (nb, m, k), ta), synth.random_bits(rng, (nb, n, k), tb)
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 110, 135)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        print("fp6/fp4 tiled", trial, (nb, m, n, k), p, flush=True)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert gpu_emulate.last_kernel.startswith("tiled"), gpu_emulate.last_kernel
        assert_same(got, want, "fp6/fp4 tiled %s" % (p,))
        if k >= 32 and L <= 32 and 32 % L == 0:            # and with E8M0 block scales (block of 32)
            SA = rng.integers(100, 150, size=(nb, m, k // 32)).astype(np.uint8)
            SB = rng.integers(100, 150, size=(nb, n, k // 32)).astype(np.uint8)
            want, _ = o2lib.emulate_mma_scaled(p, A, B, C, SA, SB, 32, ta, tb)
            got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, 32, ta, tb)
            assert "vm=3" in mm.last_kernel() or p.c_mode != C_AFTER_RD and (p.skip_zero_terms or p.zero_result_positive)
            assert_same(got, want, "fp6/fp4 tiled scaled %s" % (p,))


def test_fp6_fp4_do_not_pair_with_16_bit_types(mm):
    import torch
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    h = mm.model_create(group_len=4, frac_bits=24)
    for dt in ((mm.E2M1, mm.FP16, mm.FP32, mm.FP32), (mm.BF16, mm.E3M2, mm.FP32, mm.FP32)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma(h, z, z, z, z, 4, 4, 8, 1, dt)
        assert ei.value.status == 2
    mm.model_destroy(h)
