"""The general (one thread per output, integer arithmetic) kernel against the RATIONAL-ARITHMETIC form of the oracle,
directly: every accumulation mode, every split, every variation switch on its own, block-scaled and not, at least a
thousand outputs per case, on shapes that the tiled kernels do not take.

Why this file exists: the C form of the oracle and the device's integer routine are both written as sequences of
shifts on wide integers, so agreement between those two says less than agreement with the form that evaluates the
algorithms on exact fractions, step by step in the paper's notation.  Here nothing but that form is the reference.
"""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm
from oracle.fdpa import (ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, SPLIT_NONE, SPLIT_EVEN_ODD,
                         SPLIT_HALVES, SPLIT_QUARTERS)
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import synth
from o1_jobs import run_pool
from test_gpu_parity import mm, gpu_emulate, assert_same  # noqa: F401
from test_gpu_scaled import gpu_emulate_scaled

RD = dict(c_mode=C_AFTER_RD, frac_bits=24, frac_bits2=31)
# (name, parameters): one switch at a time on top of each mode's plain form
CASES = [
    ("in-group plain", dict(c_mode=C_IN_GROUP, frac_bits=24)),
    ("in-group narrow F", dict(c_mode=C_IN_GROUP, frac_bits=9)),
    ("in-group wide F", dict(c_mode=C_IN_GROUP, frac_bits=40)),
    ("in-group ftz_in", dict(c_mode=C_IN_GROUP, frac_bits=24, ftz_in=True)),
    ("in-group ftz_out", dict(c_mode=C_IN_GROUP, frac_bits=24, ftz_out=True)),
    ("in-group RZ", dict(c_mode=C_IN_GROUP, frac_bits=24, out_round=RZ)),
    ("in-group RZ-E8M13", dict(c_mode=C_IN_GROUP, frac_bits=13, out_round=RZ, out_mant_bits=13)),
    ("in-group skip_zero_terms", dict(c_mode=C_IN_GROUP, frac_bits=24, skip_zero_terms=True)),
    ("in-group zero_result_positive", dict(c_mode=C_IN_GROUP, frac_bits=24, zero_result_positive=True)),
    ("after-exact plain", dict(c_mode=C_AFTER_EXACT, frac_bits=24)),
    ("after-exact flushes RZ", dict(c_mode=C_AFTER_EXACT, frac_bits=20, ftz_in=True, ftz_out=True, out_round=RZ)),
    ("after-exact skip_zero_terms", dict(c_mode=C_AFTER_EXACT, frac_bits=24, skip_zero_terms=True)),
    ("after-exact zero_result_positive", dict(c_mode=C_AFTER_EXACT, frac_bits=24, zero_result_positive=True)),
    ("TR-FDPA plain", dict(RD)),
    ("TR-FDPA F2 < F", dict(RD, frac_bits2=20)),
    ("TR-FDPA flushes RZ", dict(RD, ftz_in=True, ftz_out=True, out_round=RZ)),
    ("TR-FDPA acc_special_truncation", dict(RD, acc_special_truncation=True)),
    ("TR-FDPA frac_bits_acc", dict(RD, frac_bits_acc=13)),
    ("TR-FDPA f2_at_leading_bit", dict(RD, f2_at_leading_bit=True)),
    ("TR-FDPA sum_drop_distance", dict(RD, sum_drop_distance=12)),
    ("TR-FDPA wide_products", dict(RD, wide_products=True)),
    ("TR-FDPA skip_zero_terms", dict(RD, skip_zero_terms=True)),
    ("TR-FDPA zero_result_positive", dict(RD, zero_result_positive=True)),
    ("GTR-FDPA (the paper's mode)", dict(c_mode=C_AFTER_RD_EVEN_ODD, frac_bits=24, frac_bits2=31)),
    ("even/odd split, merge bits", dict(RD, split=SPLIT_EVEN_ODD, frac_bits_merge=13)),
    ("even/odd split, leading bit + skip zeros", dict(RD, split=SPLIT_EVEN_ODD, f2_at_leading_bit=True, skip_zero_terms=True)),
    ("halves split", dict(RD, split=SPLIT_HALVES)),
    ("halves split, F 13 merge 24 (the fitted FP8 shape)", dict(RD, frac_bits=13, split=SPLIT_HALVES, frac_bits_merge=24, frac_bits_acc=24,
                                                                 acc_special_truncation=True, f2_at_leading_bit=True, skip_zero_terms=True,
                                                                 zero_result_positive=True, sum_drop_distance=28)),
    ("quarters split", dict(RD, split=SPLIT_QUARTERS)),
    ("quarters split, merge bits + special truncation", dict(RD, frac_bits=13, split=SPLIT_QUARTERS, frac_bits_merge=24, acc_special_truncation=True)),
]
PAIRS = [(fm.FP16, fm.FP16), (fm.BF16, fm.BF16), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3), (fm.E5M2, fm.E5M2), (fm.FP16, fm.BF16)]
WORD_CASES = (0, 1, 9, 13, 16, 18, 19, 23, 26)      # indices into CASES that also run with TF32 and FP32 operands
SCALED_PAIRS = [(fm.E4M3, fm.E4M3), (fm.E5M2, fm.E4M3), (fm.E2M3, fm.E3M2), (fm.E2M1, fm.E5M2), (fm.FP16, fm.FP16), (fm.E3M2, fm.E2M1)]


def _inputs(rng, ta, tb, nb, m, n, k, idx):
    """Operands with a fifth of the elements zero (either sign), exponents mostly near each other so that alignment,
    the round-downs and the thresholds all come into play; every fourth case over the whole exponent range."""
    if ta == fm.BF16:
        A = synth.narrow_exponent_bits(rng, (nb, m, k), ta, 110, 140) if idx % 4 else synth.random_bits(rng, (nb, m, k), ta)
    else:
        A = synth.random_bits(rng, (nb, m, k), ta)
    if tb == fm.BF16:
        B = synth.narrow_exponent_bits(rng, (nb, n, k), tb, 110, 140) if idx % 4 else synth.random_bits(rng, (nb, n, k), tb)
    else:
        B = synth.random_bits(rng, (nb, n, k), tb)
    A = synth.sprinkle(rng, A, np.array([0, 1 << (synth.WIDTH[ta] - 1)], dtype=A.dtype), 0.2)
    lo, hi = (1, 254) if idx % 4 == 0 else (95, 160)
    C = synth.narrow_exponent_bits(rng, (nb, m, n), fm.FP32, lo, hi)
    C = synth.sprinkle(rng, C, np.array([0, 0x80000000, 1, 0x007FFFFF], dtype=np.uint32), 0.05)
    if idx % 3 == 0:        # special values of Sec. 4.2 in a few places
        B = synth.sprinkle(rng, B, synth.SPECIAL_CODES[tb], 0.01)
        C = synth.sprinkle(rng, C, synth.SPECIAL_CODES[fm.FP32], 0.01)
    return A, B, C


def _group_shape(kw, idx):
    """Group length and k that every mode of the case accepts; tiles of 15 x 27 (no tiled kernel takes tiles of fewer than 16 rows)."""
    L = [8, 16, 4, 32][idx % 4]
    if kw.get("split") == SPLIT_QUARTERS:
        L = max(L, 16) if idx % 2 else 32
    k = L * (1 + idx % 2)
    return L, k


@pytest.fixture(scope="module")
def results(mm):
    """All GPU outputs first, then the rational oracle for every case in a process pool."""
    rng = np.random.default_rng(2511)
    gpu, jobs, names = [], [], []
    for idx, (name, kw) in enumerate(CASES):
        L, k = _group_shape(kw, idx)
        p = ModelParams(group_len=L, **kw)
        # not block-scaled: 3 tiles of 15 x 27 (1215 outputs)
        ta, tb = PAIRS[idx % len(PAIRS)]
        A, B, C = _inputs(rng, ta, tb, 3, 15, 27, k, idx)
        got = gpu_emulate(mm, p, A, B, C, ta, tb)
        assert gpu_emulate.last_kernel == "general", (name, gpu_emulate.last_kernel)
        gpu.append(got)
        jobs.append((dataclasses.asdict(p), A, B, C, ta, tb, None, None, 0))
        names.append(name + " [operand types %d x %d]" % (ta, tb))
        # block-scaled (Algorithm "ST-FDPA"): blocks of 8 or 32 products, scales around 1 and far from it
        ta, tb = SCALED_PAIRS[idx % len(SCALED_PAIRS)]
        block = 8 if idx % 2 else 32
        ks = max(k, block)
        ks += (-ks) % L
        A, B, C = _inputs(rng, ta, tb, 3, 15, 27, ks, idx + 1)
        lo, hi = [(100, 150), (40, 215)][idx % 2]
        SA = rng.integers(lo, hi, size=(3, 15, ks // block)).astype(np.uint8)
        SB = rng.integers(lo, hi, size=(3, 27, ks // block)).astype(np.uint8)
        if idx % 5 == 0:
            SA[0, 0, 0] = 0xFF          # a NaN scale
        got = gpu_emulate_scaled(mm, p, A, B, C, SA, SB, block, ta, tb)
        assert mm.last_kernel().startswith("general"), (name, mm.last_kernel())
        gpu.append(got)
        jobs.append((dataclasses.asdict(p), A, B, C, ta, tb, SA, SB, block))
        names.append(name + ", block-scaled")
        # operands held in 32-bit words (TF32: 10 mantissa bits count; FP32: whole 48-bit products), for some of the cases
        if idx in WORD_CASES:
            for tw in (fm.TF32, fm.FP32):
                A, B, C = _inputs(rng, tw, tw, 3, 15, 27, k, idx + 2)
                if idx % 2:         # exponents close together: alignment matters
                    A = synth.narrow_exponent_bits(rng, A.shape, tw, 118, 136)
                    B = synth.narrow_exponent_bits(rng, B.shape, tw, 118, 136)
                got = gpu_emulate(mm, p, A, B, C, tw, tw)
                assert gpu_emulate.last_kernel == "general", (name, gpu_emulate.last_kernel)
                gpu.append(got)
                jobs.append((dataclasses.asdict(p), A, B, C, tw, tw, None, None, 0))
                names.append(name + " [operand type %d]" % tw)
    want = run_pool(jobs, workers=12)
    return names, gpu, want


def test_every_path_of_the_general_kernel_matches_the_rational_oracle(results):
    names, gpu, want = results
    assert len(names) == 2 * len(CASES) + 2 * len(WORD_CASES)
    bad = []
    for name, g, w in zip(names, gpu, want):
        assert g.size >= 1000
        if not np.array_equal(g, w):
            i = np.argwhere(g != w)[0]
            bad.append("%s: %d of %d differ, first at %s: gpu %08x, oracle %08x" % (name, int((g != w).sum()), g.size, tuple(i), int(g[tuple(i)]), int(w[tuple(i)])))
    assert not bad, "\n".join(bad)


def test_the_cases_are_not_degenerate(results):
    """Sanity of the inputs: the outputs of every case take many values, and special values occur."""
    names, gpu, want = results
    for name, w in zip(names, want):
        assert len(np.unique(w)) > 100, name
    assert any(((w & 0x7FFFFFFF) > 0x7F800000).any() for w in want)            # NaN results occur somewhere
    assert any(((w & 0x7FFFFFFF) == 0x7F800000).any() for w in want)           # and infinities
