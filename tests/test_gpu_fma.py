"""GPU parity for the FMA family (Phi_FMA, Sec. 4.1.2): the chain of standard fused multiply-adds on FP32 operands,
element by element against oracle/fma.py, every launch variant of the kernel (16 x 16 blocks or row-major order, 128-bit
or single loads), every input family including zeros of both signs, and both NaN rules."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, fma as ofma
from oracle.fdpa import ModelParams, C_AFTER_EXACT
from oracle.rounding import RNE
from paper_2511_10909_amd import synth
from gpu_utils import to_dev, dev_empty, to_host
from test_gpu_parity import gpu_emulate, assert_same, mm                                     # noqa: F401  (mm is a fixture)
from test_gpu_fp32_operands import fp32_case

ZEROS = np.array([0, 0x80000000, 0, 0x80000000, 0x3F800000, 0xBF800000, 0x00000001, 0x80000001], dtype=np.uint32)


def gpu_fma(mm, A, B, C, nan_bits=0x7FC00000, nan_propagate=False, offset_words=0):
    """Runs the FMA family; offset_words shifts A and B off their 16-byte alignment (single-load variant)."""
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(family=mm.FAMILY_FMA, nan_bits=nan_bits, nan_propagate=nan_propagate)
    try:
        def shifted(x):
            buf = np.zeros(x.size + offset_words, dtype=np.uint32)
            buf[offset_words:] = x.reshape(-1)
            return to_dev(buf)
        bA, bB = shifted(A.astype(np.uint32)), shifted(B.astype(np.uint32))
        dC = to_dev(C.astype(np.uint32))
        dD = dev_empty((nb, m, n), np.uint32)
        mm.emulate_mma(h, bA.data_ptr() + 4 * offset_words, bB.data_ptr() + 4 * offset_words, dC, dD, m, n, k, nb,
                       (mm.FP32, mm.FP32, mm.FP32, mm.FP32))
        gpu_fma.last_kernel = mm.last_kernel()
        return to_host(dD, np.uint32)
    finally:
        mm.model_destroy(h)


def zero_case(rng, nb, m, n, k):
    return ZEROS[rng.integers(0, len(ZEROS), (nb, m, k))], ZEROS[rng.integers(0, len(ZEROS), (nb, n, k))], ZEROS[rng.integers(0, len(ZEROS), (nb, m, n))]


SHAPES = [  # (tiles, m, n, k, offset_words, expected kernel variant)
    (6, 16, 16, 4, 0, "fma chain, 16x16 blocks, 128-bit loads, 4 blocks in flight"),
    (2, 32, 32, 2, 0, "fma chain, 16x16 blocks, 64-bit loads, 4 blocks in flight"),
    (3, 32, 32, 1, 0, "fma chain, 16x16 blocks"),
    (40, 4, 4, 1, 0, "fma chain"),
    (3, 5, 7, 3, 0, "fma chain"),
    (2, 9, 13, 8, 0, "fma chain, 128-bit loads"),
    (2, 16, 16, 8, 1, "fma chain, 16x16 blocks"),            # rows off the 8-byte alignment
    (2, 16, 16, 8, 2, "fma chain, 16x16 blocks, 64-bit loads"),      # rows 8-byte but not 16-byte aligned
    (5, 3, 6, 6, 0, "fma chain, 64-bit loads"),
    (1, 48, 32, 20, 0, "fma chain, 16x16 blocks, 128-bit loads"),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_fma_family_matches_the_oracle(mm, shape):
    nb, m, n, k, off, kernel = shape
    rng = np.random.default_rng(5200 + 7 * m + k)
    for trial in range(5):
        print("case", shape, trial, flush=True)
        A, B, C = zero_case(rng, nb, m, n, k) if trial == 4 else fp32_case(rng, nb, m, n, k, trial)
        for propagate, nan_bits in ((False, 0x7FC00000), (True, 0xFFC00000), (False, 0x7FFFFFFF)):
            want = ofma.emulate_mma(A, B, C, nan_bits=nan_bits, nan_propagate=propagate)
            got = gpu_fma(mm, A, B, C, nan_bits=nan_bits, nan_propagate=propagate, offset_words=off)
            assert gpu_fma.last_kernel == (kernel.replace("fma chain", "fma chain, payloads") if propagate else kernel), gpu_fma.last_kernel
            assert_same(got, want, "fma family %s trial %d propagate %d" % (shape, trial, propagate))
        if trial == 4:
            assert np.count_nonzero(want == 0x80000000) > 0       # the case does reach the sign rule


def test_fma_family_kernel_names(mm):
    rng = np.random.default_rng(1)
    A, B, C = fp32_case(rng, 1, 16, 16, 4, 1)
    gpu_fma(mm, A, B, C, nan_propagate=True)
    assert gpu_fma.last_kernel == "fma chain, payloads, 16x16 blocks, 128-bit loads, 4 blocks in flight"
    gpu_fma(mm, A, B, C)
    assert gpu_fma.last_kernel == "fma chain, 16x16 blocks, 128-bit loads, 4 blocks in flight"


def test_fma_family_differs_from_the_fdpa_chain_only_in_the_sign_of_zero(mm):
    chain = ModelParams(group_len=1, frac_bits=46, c_mode=C_AFTER_EXACT, out_round=RNE)
    rng = np.random.default_rng(5300)
    seen = 0
    for trial in range(5):
        A, B, C = zero_case(rng, 4, 16, 16, 4) if trial == 4 else fp32_case(rng, 4, 16, 16, 4, trial)
        x, y = gpu_fma(mm, A, B, C), gpu_emulate(mm, chain, A, B, C, fm.FP32, fm.FP32)
        d = x != y
        assert np.all(x[d] == 0x80000000) and np.all(y[d] == 0)
        seen += int(np.count_nonzero(d))
    assert seen > 0


def test_fma_family_on_a_gemm_shape_sampled(mm):
    # a larger problem in the blocked order: sampled outputs against the oracle, the rest against the chain of the
    # FDPA family (the general kernel), which may differ only in a zero's sign
    rng = np.random.default_rng(5400)
    m, n, k = 128, 96, 64
    A = rng.standard_normal((1, m, k)).astype(np.float32).view(np.uint32)
    B = rng.standard_normal((1, n, k)).astype(np.float32).view(np.uint32)
    C = rng.standard_normal((1, m, n)).astype(np.float32).view(np.uint32)
    got = gpu_fma(mm, A, B, C)
    for _ in range(200):
        i, j = int(rng.integers(0, m)), int(rng.integers(0, n))
        assert int(got[0, i, j]) == ofma.emulate_element(A[0, i].tolist(), B[0, j].tolist(), int(C[0, i, j])), (i, j)
    chain = ModelParams(group_len=1, frac_bits=46, c_mode=C_AFTER_EXACT, out_round=RNE)
    assert_same(got, gpu_emulate(mm, chain, A, B, C, fm.FP32, fm.FP32), "gemm shape")


@pytest.mark.parametrize("shape", [(1, 64, 64, 64), (2, 128, 64, 80), (1, 64, 192, 128), (512, 128, 128, 64), (130, 256, 128, 80)])
def test_fma_family_lds_tiled_kernel(mm, shape):
    # large shapes go through LDS in 64 x 64 blocks: equal, element by element, to the simple kernel (taken when the
    # operands are off their 16-byte alignment), and to the oracle on sampled outputs and on every NaN output
    nb, m, n, k = shape
    rng = np.random.default_rng(5500 + m + n + k)
    big = m % 128 == 0 and n % 128 == 0 and nb * (m // 128) * (n // 128) >= 512          # 128 x 128 blocks
    for trial in ((1, 4) if big else range(5)):
        print("case", shape, trial, flush=True)
        A, B, C = zero_case(rng, nb, m, n, k) if trial == 4 else fp32_case(rng, nb, m, n, k, trial)
        if trial == 1:          # a few NaN / infinite operands only: most outputs stay finite, some chains meet a NaN late
            A, B, C = fp32_case(rng, nb, m, n, k, 2)
            A = synth.sprinkle(rng, A, synth.SPECIAL_CODES[fm.FP32], 0.002)
            B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[fm.FP32], 0.002)
        for propagate, nan_bits in ((False, 0x7FC00000), (True, 0xFFC00000)):
            got = gpu_fma(mm, A, B, C, nan_bits=nan_bits, nan_propagate=propagate)
            assert gpu_fma.last_kernel == "fma chain%s, %s blocks through LDS" % (", payloads" if propagate else "", "128x128" if big else "64x64"), gpu_fma.last_kernel
            simple = gpu_fma(mm, A, B, C, nan_bits=nan_bits, nan_propagate=propagate, offset_words=1)
            assert "16x16 blocks" in gpu_fma.last_kernel
            assert_same(got, simple, "tiled against simple %s trial %d propagate %d" % (shape, trial, propagate))
            nan = np.argwhere((got & 0x7FFFFFFF) > 0x7F800000)[:150]
            picks = [tuple(x) for x in nan] + [(int(rng.integers(0, nb)), int(rng.integers(0, m)), int(rng.integers(0, n))) for _ in range(60)]
            for t, i, j in picks:
                want = ofma.emulate_element(A[t, i].tolist(), B[t, j].tolist(), int(C[t, i, j]), nan_bits=nan_bits, nan_propagate=propagate)
                assert int(got[t, i, j]) == want, (shape, trial, propagate, (t, i, j), hex(int(got[t, i, j])), hex(want))


def test_fma_family_lds_tiled_kernel_in_place(mm):
    # D may alias C
    rng = np.random.default_rng(5600)
    nb, m, n, k = 1, 64, 128, 64
    A, B, C = fp32_case(rng, nb, m, n, k, 1)
    want = gpu_fma(mm, A, B, C, nan_bits=0xFFC00000, nan_propagate=True)
    h = mm.model_create(family=mm.FAMILY_FMA, nan_bits=0xFFC00000, nan_propagate=True)
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C)
    mm.emulate_mma(h, dA, dB, dC, dC, m, n, k, nb, (mm.FP32,) * 4)
    assert "through LDS" in mm.last_kernel()
    mm.model_destroy(h)
    assert_same(to_host(dC, np.uint32), want, "in place")
