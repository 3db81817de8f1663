"""GPU parity of GST-FDPA (paper Algorithm "GST-FDPA"): the library against the CPU oracle, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import o2lib
from gpu_utils import to_dev, dev_empty, to_host
from test_gpu_parity import mm, assert_same  # noqa: F401


def gpu_gst(mm, A, B, C, SA, SB, L, G, kb, F, rho, fmt, nan_bits=0x7FFFFFFF):
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(family=mm.FAMILY_GST_FDPA, group_len=L, gst_group=G, frac_bits=F, out_round=rho, nan_bits=nan_bits, scale_format=fmt)
    try:
        dD = dev_empty((nb, m, n), np.uint32)
        mm.emulate_mma_scaled(h, to_dev(A), to_dev(B), to_dev(C), dD, to_dev(SA), to_dev(SB), kb, m, n, k, nb, (mm.E2M1, mm.E2M1, mm.FP32, mm.FP32))
        want_kernel = "gst-fdpa, 16x16 blocks through LDS" if (m % 16 == 0 and n % 16 == 0 and G % 4 == 0 and (L or k) <= 256) else "gst-fdpa"
        assert mm.last_kernel() == want_kernel, mm.last_kernel()
        return to_host(dD, np.uint32)
    finally:
        mm.model_destroy(h)


@pytest.mark.parametrize("fmt,kb", [(1, 16), (0, 32), (1, 32), (0, 16)])
def test_gst_matches_oracle(mm, fmt, kb):
    rng = np.random.default_rng(60 + 2 * kb + fmt)
    for trial in range(12):
        L, G = [(64, 16), (32, 8), (0, 16), (128, 4)][trial % 4]
        k = 128
        F = int(rng.choice([6, 20, 35, 40]))
        rho = int(rng.integers(0, 2))
        nb, m, n = int(rng.integers(1, 4)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        A = rng.integers(0, 256, (nb, m, k)).astype(np.uint8)          # (bits above the FP4 code are ignored)
        B = rng.integers(0, 16, (nb, n, k)).astype(np.uint8)
        lo, hi = ((0x08, 0x7F) if trial % 3 else (0x00, 0x100)) if fmt == 1 else ((100, 150) if trial % 3 else (0, 256))
        SA = rng.integers(lo, hi, (nb, m, k // kb)).astype(np.uint8)
        SB = rng.integers(lo, hi, (nb, n, k // kb)).astype(np.uint8)
        C = (rng.standard_normal((nb, m, n)) * 2.0 ** rng.integers(-30, 30, (nb, m, n))).astype(np.float32).view(np.uint32)
        C.flat[0] = 0x7F800000
        C.flat[-1] = 0xFFC00000
        want = o2lib.emulate_gst(A, B, C, SA, SB, L, G, kb, F, rho, fmt)
        got = gpu_gst(mm, A, B, C, SA, SB, L, G, kb, F, rho, fmt)
        assert_same(got, want, "gst L=%d G=%d kb=%d F=%d" % (L, G, kb, F))


@pytest.mark.parametrize("fmt,kb", [(1, 16), (0, 32), (1, 32), (0, 16)])
def test_gst_blocks_through_lds(mm, fmt, kb):
    # shapes that take the kernel with operand sharing (16 x 16 blocks of D, dot products by v_dot4_i32_i8): every output
    # against the C form of the oracle, a sample against the rational form
    from oracle import gst as ogst
    rng = np.random.default_rng(160 + 2 * kb + fmt)
    for trial in range(8):
        L, G = [(64, 16), (32, 8), (0, 16), (128, 4), (256, 16), (64, 32)][trial % 6]
        if G > kb:
            G = kb
        k = 256 if L == 256 else 128
        F = int(rng.choice([6, 20, 35, 40]))
        rho = int(rng.integers(0, 2))
        nb, m, n = [(3, 16, 16), (2, 32, 48), (1, 48, 16)][trial % 3]
        A = rng.integers(0, 256, (nb, m, k)).astype(np.uint8)
        B = rng.integers(0, 16, (nb, n, k)).astype(np.uint8)
        lo, hi = ((0x08, 0x7F) if trial % 3 else (0x00, 0x100)) if fmt == 1 else ((100, 150) if trial % 3 else (0, 256))
        SA = rng.integers(lo, hi, (nb, m, k // kb)).astype(np.uint8)
        SB = rng.integers(lo, hi, (nb, n, k // kb)).astype(np.uint8)
        C = (rng.standard_normal((nb, m, n)) * 2.0 ** rng.integers(-30, 30, (nb, m, n))).astype(np.float32).view(np.uint32)
        C.flat[0] = 0x7F800000
        C.flat[-1] = 0xFFC00000
        want = o2lib.emulate_gst(A, B, C, SA, SB, L, G, kb, F, rho, fmt)
        got = gpu_gst(mm, A, B, C, SA, SB, L, G, kb, F, rho, fmt)
        assert mm.last_kernel() == "gst-fdpa, 16x16 blocks through LDS"
        assert_same(got, want, "gst blocks L=%d G=%d kb=%d F=%d" % (L, G, kb, F))
        for (ti, ii, jj) in ((0, 0, 0), (0, 1, 2), (nb - 1, m - 1, n - 1), (0, 5, 15)):
            w1 = ogst.emulate_element(A[ti, ii].tolist(), B[ti, jj].tolist(), int(C[ti, ii, jj]), SA[ti, ii].tolist(), SB[ti, jj].tolist(),
                                      L or k, G, kb, F, rho, fmt)
            assert int(got[ti, ii, jj]) == w1, ("rational form", ti, ii, jj)


def test_gst_presets_and_errors(mm):
    import torch
    from paper_2511_10909_amd import presets
    rng = np.random.default_rng(3)
    for (key, kb) in ((("blackwell", "mxfp4"), 32), (("blackwell", "nvfp4"), 16)):
        kw = presets.PAPER_GST[key]
        A = rng.integers(0, 16, (2, 16, 128)).astype(np.uint8)
        B = rng.integers(0, 16, (2, 16, 128)).astype(np.uint8)
        SA = rng.integers(0x20, 0x60, (2, 16, 128 // kb)).astype(np.uint8) if kb == 16 else rng.integers(115, 140, (2, 16, 4)).astype(np.uint8)
        SB = rng.integers(0x20, 0x60, (2, 16, 128 // kb)).astype(np.uint8) if kb == 16 else rng.integers(115, 140, (2, 16, 4)).astype(np.uint8)
        C = rng.standard_normal((2, 16, 16)).astype(np.float32).view(np.uint32)
        want = o2lib.emulate_gst(A, B, C, SA, SB, 64, 16, kb, 35, 1, kw["scale_format"])
        got = gpu_gst(mm, A, B, C, SA, SB, 64, 16, kb, 35, 1, kw["scale_format"])
        assert_same(got, want, "gst preset %s" % (key,))
    z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    h = mm.model_create(**presets.PAPER_GST[("blackwell", "nvfp4")])
    for args, status in (((h, z, z, z, z, z, z, 16, 4, 4, 96, 1, (mm.E2M1, mm.E2M1, mm.FP32, mm.FP32)), 3),        # k % L
                         ((h, z, z, z, z, z, z, 8, 4, 4, 64, 1, (mm.E2M1, mm.E2M1, mm.FP32, mm.FP32)), 3),         # block % G
                         ((h, z, z, z, z, z, z, 16, 4, 4, 64, 1, (mm.E4M3, mm.E2M1, mm.FP32, mm.FP32)), 2)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma_scaled(*args)
        assert ei.value.status == status
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, z, z, z, z, 4, 4, 64, 1, (mm.E2M1, mm.E2M1, mm.FP32, mm.FP32))
    assert ei.value.status == 2
    mm.model_destroy(h)
    for kw in (dict(family=mm.FAMILY_GST_FDPA, group_len=64, gst_group=0), dict(family=mm.FAMILY_GST_FDPA, group_len=64, gst_group=24),
               dict(family=mm.FAMILY_GST_FDPA, group_len=64, gst_group=16, skip_zero_terms=True), dict(gst_group=16)):
        with pytest.raises(mm.MmaemuError):
            mm.model_create(**kw)
