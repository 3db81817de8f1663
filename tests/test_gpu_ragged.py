"""GPU parity of the tiled kernels on ragged shapes (m or n not a multiple of the 32 x 32 block, more than one block each
way): edge blocks stage the tile's last row again and store only what lies inside D.  Every output against the C form of
the oracle, a sample against the rational form; the words around D must stay untouched."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, SPLIT_HALVES, SPLIT_QUARTERS
from oracle.fdpa import emulate_mma as o1_emulate
from gpu_utils import to_dev, to_host
from test_gpu_parity import assert_same, mm, NP  # noqa: F401  (fixture)
from test_gpu_tiled import operands
from test_gpu_tiled_rd import random_rd_params

GUARD = 64                       # words before and after D
FILL = 0x5EAFBEEF


def emulate_guarded(mm, p, A, B, C, ta, tb):
    """The emulation with D inside a larger buffer whose other words are checked afterwards."""
    nb, m, k = A.shape
    n = B.shape[1]
    h = mm.model_create(group_len=p.group_len, frac_bits=p.frac_bits, frac_bits2=p.frac_bits2, c_mode=p.c_mode, out_round=p.out_round,
                        ftz_in=p.ftz_in, ftz_out=p.ftz_out, nan_bits=p.nan_bits, split=p.split,
                        acc_special_truncation=p.acc_special_truncation, frac_bits_merge=p.frac_bits_merge,
                        frac_bits_acc=p.frac_bits_acc, f2_at_leading_bit=p.f2_at_leading_bit,
                        skip_zero_terms=p.skip_zero_terms, zero_result_positive=p.zero_result_positive,
                        sum_drop_distance=p.sum_drop_distance, family=p.family, out_mant_bits=p.out_mant_bits,
                        wide_products=p.wide_products, nan_propagate=p.nan_propagate, rd_toward_zero=p.rd_toward_zero)
    try:
        dA, dB, dC = to_dev(A.astype(NP[ta])), to_dev(B.astype(NP[tb])), to_dev(C.astype(np.uint32))
        count = nb * m * n
        buf = torch.full((count + 2 * GUARD,), FILL, dtype=torch.int32, device="cuda")
        dD = buf[GUARD:GUARD + count]
        mm.emulate_mma(h, dA, dB, dC, dD, m, n, k, nb, (ta, tb, fm.FP32, fm.FP32))
        kernel = mm.last_kernel()
        whole = to_host(buf, np.uint32)
        assert (whole[:GUARD] == FILL).all() and (whole[GUARD + count:] == FILL).all(), "words outside D were written (%s)" % kernel
        return whole[GUARD:GUARD + count].reshape(nb, m, n), kernel
    finally:
        mm.model_destroy(h)


def check_sample_against_rational_form(rng, p, A, B, C, ta, tb, got, what, count=24):
    nb, m, k = A.shape
    n = B.shape[1]
    # the outputs of the last row and column (edge blocks) and a few anywhere
    places = [(nb - 1, m - 1, n - 1), (0, m - 1, 0), (0, 0, n - 1)]
    places += [(int(rng.integers(nb)), int(rng.integers(m)), int(rng.integers(n))) for _ in range(count)]
    for (t, i, j) in places:
        want = o1_emulate(p, A[t:t + 1, i:i + 1, :], B[t:t + 1, j:j + 1, :], C[t:t + 1, i:i + 1, j:j + 1], ta, tb)[0, 0, 0]
        assert got[t, i, j] == want, "%s: output %s: got %08x, the rational form gives %08x" % (what, (t, i, j), got[t, i, j], want)


SHAPES = [(33, 47, 32, 2), (70, 100, 64, 1), (45, 33, 24, 3), (95, 129, 32, 1), (64, 40, 8, 2), (34, 64, 32, 1),
          (20, 20, 16, 5), (32, 33, 32, 2), (17, 31, 8, 3), (33, 17, 64, 2)]       # (the last four: one block one way or both)


@pytest.mark.parametrize("ta,tb", [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.FP16)])
def test_ragged_shapes_in_the_tiled_kernels(mm, ta, tb):
    rng = np.random.default_rng(8800 + 8 * ta + tb)
    rd_cases = rd_tiled = 0
    for (m, n, k, nb) in SHAPES:
        Ls = [L for L in (4, 8, 16, 32) if k % L == 0 and (k % 32 == 0 or L <= 8)]
        for mode in ("narrow", "full", "special"):
            for cm in (C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD):
                L = int(rng.choice(Ls))
                if cm == C_AFTER_RD:
                    p = random_rd_params(rng, k).with_(group_len=L)
                else:
                    F = int(rng.choice([3, 13, 16, 24, 25, 27, 28, 30, 32, 35]))
                    if cm == C_AFTER_EXACT:
                        F = min(F, 30)
                    p = ModelParams(group_len=L, frac_bits=F, c_mode=cm, out_round=int(rng.integers(0, 2)),
                                    ftz_in=bool(rng.integers(0, 4) == 0), ftz_out=bool(rng.integers(0, 4) == 0))
                A, B, C = operands(rng, ta, tb, nb, m, n, k, mode)
                print("ragged", ta, tb, (m, n, k, nb), mode, p, flush=True)
                want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
                got, kernel = emulate_guarded(mm, p, A, B, C, ta, tb)
                what = "ragged %s %s %s %s" % ((m, n, k, nb), mode, p, kernel)
                assert_same(got, want, what)
                if cm == C_AFTER_RD:         # (some of the random variations run in the general kernel for any shape)
                    rd_cases += 1
                    rd_tiled += kernel.startswith("tiled 32x32")
                else:
                    assert kernel.startswith("tiled 32x32"), what
                if mode != "narrow":
                    check_sample_against_rational_form(rng, p, A, B, C, ta, tb, got, what, count=6)
    assert rd_tiled >= 0.6 * rd_cases, (rd_tiled, rd_cases)


def test_ragged_shapes_split_groups(mm):
    # even / odd, halves and quarters (binary32 values only: FP8 and FP16 operands)
    rng = np.random.default_rng(8900)
    base = ModelParams(group_len=16, frac_bits=13, frac_bits2=31, c_mode=C_AFTER_RD, nan_bits=0xFFC00000)
    cases = [(base.with_(c_mode=C_AFTER_RD_EVEN_ODD), fm.E5M2, fm.E4M3), (base.with_(split=SPLIT_HALVES, frac_bits_merge=24, frac_bits_acc=24), fm.E4M3, fm.E4M3),
             (base.with_(split=SPLIT_QUARTERS, group_len=32), fm.E4M3, fm.E5M2), (base.with_(split=SPLIT_HALVES, group_len=8, frac_bits=20), fm.FP16, fm.FP16)]
    for p, ta, tb in cases:
        for (m, n, k, nb) in ((33, 47, 32, 2), (70, 41, 64, 1)):
            for mode in ("narrow", "special"):
                A, B, C = operands(rng, ta, tb, nb, m, n, k, mode)
                want, _ = o2lib.emulate_mma(p, A, B, C, ta, tb)
                got, kernel = emulate_guarded(mm, p, A, B, C, ta, tb)
                what = "ragged split %s %s %s %s" % ((m, n, k, nb), mode, p, kernel)
                assert_same(got, want, what)
                assert kernel.startswith("tiled 32x32"), what


def test_narrow_ragged_tiles_and_long_groups_keep_the_general_kernel(mm):
    # at most 16 rows or columns (and no multiple of 16 both ways), or groups that span several staged chunks
    rng = np.random.default_rng(8901)
    for (m, n, k, nb, L) in ((12, 12, 16, 3, 8), (16, 33, 32, 2, 8), (40, 9, 32, 2, 8), (70, 100, 128, 1, 64), (70, 100, 64, 1, 0)):
        p = ModelParams(group_len=L, frac_bits=24)
        A, B, C = operands(rng, fm.FP16, fm.FP16, nb, m, n, k, "special")
        want, _ = o2lib.emulate_mma(p, A, B, C, fm.FP16, fm.FP16)
        got, kernel = emulate_guarded(mm, p, A, B, C, fm.FP16, fm.FP16)
        assert_same(got, want, "general %s" % ((m, n, k, nb, L),))
        assert kernel == "general", kernel


def test_ragged_shapes_tf32(mm):
    # operands in 32-bit words (four to a 128-bit load): edge blocks of one block and of several, three modes
    from test_gpu_tf32 import tf32_case
    rng = np.random.default_rng(8902)
    trial = 0
    for (m, n, k, nb) in ((20, 20, 16, 5), (33, 47, 32, 2), (17, 31, 8, 3), (70, 41, 64, 1)):
        for cm in (C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD):
            trial += 1
            L = int(rng.choice([L for L in (4, 8, 16, 32) if k % L == 0 and (k % 32 == 0 or L <= 8)]))
            p = ModelParams(group_len=L, frac_bits=int(rng.choice([13, 24, 25, 27])), c_mode=cm, out_round=int(rng.integers(0, 2)),
                            ftz_in=bool(rng.integers(0, 4) == 0), ftz_out=bool(rng.integers(0, 4) == 0))
            if cm == C_AFTER_RD:
                p = p.with_(frac_bits2=31)
            A, B, C = tf32_case(rng, nb, m, n, k, trial)
            print("ragged tf32", (m, n, k, nb), p, flush=True)
            want, _ = o2lib.emulate_mma(p, A, B, C, fm.TF32, fm.TF32)
            got, kernel = emulate_guarded(mm, p, A, B, C, fm.TF32, fm.TF32)
            what = "ragged tf32 %s %s %s" % ((m, n, k, nb), p, kernel)
            assert_same(got, want, what)
            assert kernel.startswith("tiled 32x32") and "vm=4" in kernel, what
            check_sample_against_rational_form(rng, p, A, B, C, fm.TF32, fm.TF32, got, what, count=4)
