"""GPU parity of the Phi_FTZ-AddMul family (paper Sec. 4.1.1) against the CPU oracle, bit for bit, and its printed values
through the library."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_mma as o1_emulate, FAMILY_FTZ_ADDMUL
from paper_2511_10909_amd import synth
from helpers import f32_bits, bf16_bits, fp16_bits
from test_gpu_parity import mm, gpu_emulate, assert_same, PAIRS  # noqa: F401


@pytest.mark.parametrize("ta,tb", PAIRS)
def test_addmul_random(mm, ta, tb):
    rng = np.random.default_rng(2100 + 8 * ta + tb)
    for trial in range(10):
        p = ModelParams(group_len=2 if trial % 2 else 4, family=FAMILY_FTZ_ADDMUL, nan_bits=0x7FC00000 if trial % 3 else 0xFFC00000)
        k = 4 * int(rng.integers(1, 9))
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        if trial % 3 == 0:
            A = synth.random_bits(rng, (nb, m, k), ta)
            B = synth.random_bits(rng, (nb, n, k), tb)
            C = synth.random_bits(rng, (nb, m, n), fm.FP32)
        else:     # products and sums around the flush threshold
            lo = {fm.BF16: (50, 80), fm.FP16: (0, 6), fm.E5M2: (0, 6), fm.E4M3: (0, 4)}
            A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo[ta])
            B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *lo[tb])
            C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 0, 6 if (ta == fm.BF16 and tb == fm.BF16) else 110)
        if trial % 4 == 0:
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[ta], 0.02)
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.02)
            C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.05)
        want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert_same(got, want, "%s %s" % (p, gpu_emulate.last_kernel))
        assert gpu_emulate.last_kernel.startswith("ftz-addmul")
        assert_same(got[:1, :2, :2], o1_emulate(p, A[:1, :2], B[:1, :2], C[:1, :2, :2], ta, tb), "rational form")


@pytest.mark.parametrize("ta,tb", [(fm.BF16, fm.BF16), (fm.FP16, fm.FP16), (fm.E5M2, fm.FP16), (fm.E4M3, fm.BF16)])
def test_addmul_blocks_through_lds(mm, ta, tb):
    # shapes that take the kernels with operand sharing: 16 x 16 and 32 x 32 blocks of D, k above and below the staged
    # chunk of 64, both P; all bit patterns (NaN and infinities included) and values around the flush threshold
    rng = np.random.default_rng(2300 + 8 * ta + tb)
    for (nb, m, n, k, P, kernel) in ((5, 32, 32, 8, 2, "32x32"), (3, 16, 16, 16, 4, "16x16"), (2, 48, 16, 12, 2, "16x16"),
                                     (1, 64, 32, 72, 4, "32x32"), (2, 32, 64, 130, 2, "32x32")):
        p = ModelParams(group_len=P, family=FAMILY_FTZ_ADDMUL, nan_bits=0xFFC00000 if P == 2 else 0x7FC00000)
        for trial in range(2):
            if trial == 0:
                A = synth.random_bits(rng, (nb, m, k), ta, finite=False)
                B = synth.random_bits(rng, (nb, n, k), tb, finite=False)
                C = synth.random_bits(rng, (nb, m, n), fm.FP32, finite=False)
            else:
                lo = {fm.BF16: (50, 80), fm.FP16: (0, 6), fm.E5M2: (0, 6), fm.E4M3: (0, 4)}
                A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, *lo[ta])
                B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, *lo[tb])
                C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, 0, 6 if (ta == fm.BF16 and tb == fm.BF16) else 110)
            want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
            got = gpu_emulate(mm, p, A, B, C, ta, tb)
            assert gpu_emulate.last_kernel == "ftz-addmul P=%d, %s blocks through LDS" % (P, kernel), gpu_emulate.last_kernel
            assert_same(got, want, "%s %s" % (p, gpu_emulate.last_kernel))
            assert_same(got[:1, :2, :4], o1_emulate(p, A[:1, :2], B[:1, :4], C[:1, :2, :4], ta, tb), "rational form")


def test_addmul_printed_values(mm):
    # Table "divergent results ...", CDNA2 row: 0.0 (P = 4) and -0.375 (P = 2)
    a = [bf16_bits(x) for x in (-2.0 ** 13, -0.5, -0.25, -0.125)]
    b = [bf16_bits(x) for x in (2.0 ** 10, 1.0, 1.0, 1.0)]
    A, B, C = np.array([[a]], dtype=np.uint16), np.array([[b]], dtype=np.uint16), np.array([[[f32_bits(2.0 ** 23)]]], dtype=np.uint32)
    for P, want in ((4, 0.0), (2, -0.375)):
        got = gpu_emulate(mm, ModelParams(group_len=P, family=FAMILY_FTZ_ADDMUL), A, B, C, fm.BF16, fm.BF16)
        assert got.view(np.float32)[0, 0, 0] == want


def test_addmul_rejects_bad_k(mm):
    import torch
    z = torch.zeros(64, dtype=torch.int32, device="cuda")
    h = mm.model_create(group_len=4, family=mm.FAMILY_FTZ_ADDMUL)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, z, z, z, z, 1, 1, 6, 1, (mm.FP16, mm.FP16, mm.FP32, mm.FP32))
    assert ei.value.status == 3
    mm.model_destroy(h)
