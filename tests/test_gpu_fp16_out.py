"""GPU parity of FP16 accumulators and outputs (paper Algorithm "T-FDPA" with F_C = FP16, rho = RNE-FP16): the general
and the tiled kernels against the CPU oracle, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD
from paper_2511_10909_amd import synth
from test_gpu_parity import mm, assert_same, gpu_emulate  # noqa: F401

EXP = {fm.FP16: (3, 22), fm.E4M3: (0, 13), fm.E5M2: (4, 22), fm.BF16: (112, 133)}


def _case(rng, ta, tb, nb, m, n, k, trial):
    if trial % 3 == 0:
        A, B = synth.random_bits(rng, (nb, m, k), ta), synth.random_bits(rng, (nb, n, k), tb)
        C = synth.random_bits(rng, (nb, m, n), fm.FP16, finite=(trial % 2 == 0))
    else:
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *EXP[ta])
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *EXP[tb])
        C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP16, 0, 30)
        if trial % 3 == 2:        # tiny products next to subnormal binary16 accumulators, and cancellation
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, EXP[ta][0], EXP[ta][0] + 4)
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP16, 0, 3)
    return A, B, C


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.E4M3, fm.E5M2), (fm.BF16, fm.BF16), (fm.E5M2, fm.FP16)])
def test_fp16_accumulator_general_kernel(mm, ta, tb):
    rng = np.random.default_rng(900 + ta)
    for trial in range(18):
        L = int(rng.choice([1, 2, 3, 8, 0]))
        k = 24
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([11, 13, 24, 25, 33])), c_mode=int(rng.choice([C_IN_GROUP, C_AFTER_EXACT])),
                        out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)),
                        skip_zero_terms=True, zero_result_positive=bool(rng.integers(0, 2)), nan_bits=0x7FFF)
        nb, m, n = 2, 5, 7
        A, B, C = _case(rng, ta, tb, nb, m, n, k, trial)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb, tc=fm.FP16)
        got = gpu_emulate(mm, p, A, B, C, ta, tb, tc=fm.FP16)
        assert gpu_emulate.last_kernel.startswith("general")
        assert_same(got, want, "fp16 acc general %s" % (p,))


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.E4M3, fm.E5M2), (fm.BF16, fm.BF16)])
def test_fp16_accumulator_tiled_kernels(mm, ta, tb):
    rng = np.random.default_rng(1900 + ta)
    shapes = [(3, 16, 16, 32), (2, 32, 32, 64), (1, 64, 64, 64), (1, 32, 32, 8), (1, 256, 512, 32)]
    for trial in range(20):
        nb, m, n, k = shapes[trial % len(shapes)]
        L = int(rng.choice([x for x in (4, 8, 16, 32, 0) if (x == 0 or (k % x == 0 and x <= m)) and not (k == 8 and x not in (4, 8, 0))]))
        p = ModelParams(group_len=L, frac_bits=int(rng.choice([11, 13, 24, 25, 32])), c_mode=[C_IN_GROUP, C_AFTER_EXACT][trial % 2],
                        out_round=int(rng.integers(0, 2)), ftz_in=bool(rng.integers(0, 2)), ftz_out=bool(rng.integers(0, 2)), nan_bits=0x7FFF)
        A, B, C = _case(rng, ta, tb, nb, m, n, k, trial)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb, tc=fm.FP16)
        print("fp16 acc tiled", trial, (nb, m, n, k), p, flush=True)
        got = gpu_emulate(mm, p, A, B, C, ta, tb, tc=fm.FP16)
        assert gpu_emulate.last_kernel.startswith("tiled"), gpu_emulate.last_kernel
        assert_same(got, want, "fp16 acc tiled %s" % (p,))
        assert trial % 3 == 0 or len(np.unique(want)) > 16


def test_fp16_accumulator_argument_errors(mm):
    import torch
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    for kw, dt, status in ((dict(group_len=8, frac_bits=24, frac_bits2=31, c_mode=mm.C_AFTER_RD), (mm.FP16, mm.FP16, mm.FP16, mm.FP16), 2),
                           (dict(group_len=8, frac_bits=24), (mm.FP16, mm.FP16, mm.FP16, mm.FP32), 2),
                           (dict(group_len=8, frac_bits=24), (mm.FP16, mm.FP16, mm.FP32, mm.FP16), 2),
                           (dict(group_len=8, frac_bits=13, out_round=mm.RZ, out_mant_bits=13), (mm.E4M3, mm.E4M3, mm.FP16, mm.FP16), 2),
                           (dict(group_len=4, family=mm.FAMILY_FTZ_ADDMUL), (mm.FP16, mm.FP16, mm.FP16, mm.FP16), 2)):
        h = mm.model_create(**kw)
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma(h, z, z, z, z, 4, 4, 8, 1, dt)
        assert ei.value.status == status
        mm.model_destroy(h)
