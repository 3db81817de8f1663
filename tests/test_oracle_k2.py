"""Brute force over ALL FP8 operand tuples for k = 2 (the second term of Algorithm "T-FDPA": alignment and truncation of
the smaller product), for the four type pairings: the oracle against closed forms evaluated in binary64.

All 2^32 (a0, b0, a1, b1) tuples reduce to all ordered pairs of product classes (tests/k2_sweep.py).  Here:
  * the reduction itself is checked on the oracle: every one of the 65536 first pairs, against several second pairs,
    gives what its class gives;
  * the C form of the oracle equals the closed form on EVERY pair of classes, with nothing cut (exact sum rounded once),
    with F = 13 (the paper's FP8 setting) and with F = 4 (even the larger product loses bits);
  * the rational form equals the C form on a stratified sample: every class, as first and as second product, against
    sixteen random partners (the complete set of class pairs would take the rational form an hour).
"""
import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, emulate_element
from k2_sweep import PAIRINGS, product_classes, class_pair_operands, closed_form_table

WIDE = 40      # wide enough that nothing is cut: FP8 products span 2^-32 .. 2^32 with 8-bit significands (see below)


def _o2_table(ta, tb, reps, F):
    A, B = class_pair_operands(reps)
    C = np.zeros((A.shape[0], 1, 1), dtype=np.uint32)
    D, _ = o2lib.emulate_mma(ModelParams(group_len=2, frac_bits=F), A, B, C, ta, tb)
    return D.reshape(-1)


@pytest.mark.parametrize("ta,tb", PAIRINGS)
def test_class_reduction_is_complete(ta, tb):
    cls, reps, info = product_classes(ta, tb)
    n = len(reps)
    assert 1500 < n < 4000 and cls.max() == n - 1
    rng = np.random.default_rng(ta * 8 + tb)
    for F in (WIDE, 13, 4):
        table = _o2_table(ta, tb, reps, F).reshape(n, n)
        # all 65536 first pairs against 12 second pairs (and the other way round): the oracle on the codes themselves
        pairs = np.arange(65536)
        a0, b0 = (pairs & 255).astype(np.uint8), (pairs >> 8).astype(np.uint8)
        for second in rng.integers(0, 65536, size=12):
            a1, b1 = np.uint8(second & 255), np.uint8(second >> 8)
            for order in (0, 1):
                A = np.stack([a0, np.full(65536, a1, np.uint8)][:: 1 - 2 * order or 1], axis=1).reshape(65536, 1, 2)
                B = np.stack([b0, np.full(65536, b1, np.uint8)][:: 1 - 2 * order or 1], axis=1).reshape(65536, 1, 2)
                D, _ = o2lib.emulate_mma(ModelParams(group_len=2, frac_bits=F), A, B, np.zeros((65536, 1, 1), np.uint32), ta, tb)
                want = table[cls[pairs], cls[second]] if order == 0 else table[cls[second], cls[pairs]]
                assert np.array_equal(D.reshape(-1), want), (F, int(second), order)


@pytest.mark.parametrize("ta,tb", PAIRINGS)
def test_every_class_pair_against_the_closed_forms(ta, tb):
    cls, reps, info = product_classes(ta, tb)
    # with F = 40 nothing is cut unless the products lie more than 40 - 7 places apart; the closed form with F = 40 says
    # exactly what is cut, and the exact-sum form agrees wherever the exponents are closer than that
    for F in (WIDE, 13, 4):
        got = _o2_table(ta, tb, reps, F)
        want = closed_form_table(ta, tb, reps, info, F)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (F, bad.size, [(info[i // len(reps)], info[i % len(reps)], hex(got[i]), hex(want[i])) for i in bad[:3]])
    exact = closed_form_table(ta, tb, reps, info, None)
    wide = _o2_table(ta, tb, reps, WIDE)
    n = len(reps)
    e = np.array([k[2] if k[0] == "fin" else 0 for k in info])
    s = np.array([k[3] if k[0] == "fin" else 1 for k in info])
    close = (np.abs(e[:, None] - e[None, :]) <= WIDE - 8) | (s[:, None] == 0) | (s[None, :] == 0)
    assert np.array_equal(wide.reshape(n, n)[close], exact.reshape(n, n)[close])
    assert close.mean() > 0.8


@pytest.mark.parametrize("ta,tb", PAIRINGS)
def test_rational_form_on_a_stratified_sample_of_class_pairs(ta, tb):
    cls, reps, info = product_classes(ta, tb)
    n = len(reps)
    rng = np.random.default_rng(77 + ta * 8 + tb)
    for F in (13, 4, WIDE):
        table = _o2_table(ta, tb, reps, F).reshape(n, n)
        p = ModelParams(group_len=2, frac_bits=F)
        partners = 6 if F != 13 else 10
        for c0 in range(0, n, 3 if F != 13 else 1):              # every class (every third one for two of the widths)
            for c1 in rng.integers(0, n, size=partners):
                for x, y in ((c0, int(c1)), (int(c1), c0)):
                    a = [int(reps[x, 0]), int(reps[y, 0])]
                    b = [int(reps[x, 1]), int(reps[y, 1])]
                    assert emulate_element(p, a, b, 0, ta, tb) == int(table[x, y]), (F, info[x], info[y])
