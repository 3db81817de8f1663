"""CPU tests of the probing steps (paper Sec. 3.1, Steps 1 to 3) in paper_2511_10909_amd/probes.py: the tree
realisation against the four tables the paper prints (Figure "Examples of summation trees ..."), round trips over
random trees, and the whole probes driven against the CPU oracle's models, whose structure is known."""
import os

import numpy as np
import pytest

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams, C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, SPLIT_HALVES
from oracle.rounding import RNE, RZ
from paper_2511_10909_amd import probes
from test_oracle_model import _trees


class OracleInterface:
    def __init__(self, p, m, n, k, ta, tb):
        self.p, self.m, self.n, self.k, self.ta, self.tb = p, m, n, k, ta, tb

    def __call__(self, A, B, C):
        return o2lib.emulate_mma(self.p, A, B, C, self.ta, self.tb)[0]


def full_table(rows, n=5):
    t = [[None] * n for _ in range(n)]
    for i, r in enumerate(rows):
        for q, v in enumerate(r):
            t[i][i + 1 + q] = v
    return t


PAPER_TREES = {
    "a_chain_of_binary_sums": "((((p0 + p4) + p1) + p2) + p3)",
    "b_pairwise_then_accumulate": "(((p0 + p1) + (p2 + p3)) + p4)",
    "c_nonswamped_3term_fused": "Fx[Fx[p0, p1, p4], p2, p3]",
    "d_swamped_5term_fused": "F[p0, p1, p2, p3, p4]",
}


@pytest.mark.parametrize("name", sorted(PAPER_TREES))
def test_tree_realisation_of_the_papers_tables(name):
    rows = _trees()[name]
    tree = probes.infer_tree(full_table(rows))
    assert probes.tree_to_string(tree) == PAPER_TREES[name]
    assert probes.table_from_tree(tree, 5) == full_table(rows)


def random_tree(rng, leaves):
    if len(leaves) == 1:
        return ("leaf", leaves[0])
    arity = int(rng.integers(2, min(len(leaves), 5) + 1))
    cuts = sorted(rng.choice(np.arange(1, len(leaves)), size=arity - 1, replace=False).tolist())
    parts = [leaves[a:b] for a, b in zip([0] + cuts, cuts + [len(leaves)])]
    kind = None if arity == 2 else bool(rng.integers(0, 2))
    kids = sorted((random_tree(rng, p) for p in parts), key=lambda t: min(_leaves(t)))
    return ("sum", kind, kids)


def _leaves(t):
    return [t[1]] if t[0] == "leaf" else [x for ch in t[2] for x in _leaves(ch)]


def test_tree_round_trip_on_random_trees():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n = int(rng.integers(2, 20))
        leaves = rng.permutation(n).tolist()
        tree = random_tree(rng, leaves)
        table = probes.table_from_tree(tree, n)
        got = probes.infer_tree(table)
        # a non-swamped fused sum can admit more than one grouping of the same table (two leaves next to a pair
        # read the same as a pair next to two leaves): the realisation must reproduce the table, and the tree
        # itself wherever no such node occurs
        assert probes.table_from_tree(got, n) == table, trial
        if "Fx[" not in probes.tree_to_string(tree):
            assert probes.tree_to_string(got) == probes.tree_to_string(tree), (trial, table)


def test_inconsistent_table_is_rejected():
    t = full_table([[2, 1, 0, 3], [1, 0, 2], [0, 1], [0]])
    t[0][1] = 1
    with pytest.raises(ValueError):
        probes.infer_tree(t)


def test_encode_round_trips():
    import torch
    for t, tdt in ((probes.E4M3, torch.float8_e4m3fn), (probes.E5M2, torch.float8_e5m2), (probes.FP16, torch.float16), (probes.BF16, torch.bfloat16)):
        lo, hi = probes.exponent_range(t)
        for e in range(lo, hi + 1):
            for sig in (1, 3):
                try:
                    code = probes.encode(t, 1, sig, e - (1 if sig == 3 else 0))
                except ValueError:
                    continue
                w = 8 if t < 2 else 16
                raw = torch.from_numpy(np.array([code], dtype=np.uint8 if w == 8 else np.uint16).view(np.uint8 if w == 8 else np.int16))
                val = float(raw.view(tdt).to(torch.float64)[0])
                assert val == -sig * 2.0 ** (e - (1 if sig == 3 else 0)), (t, e, sig, code, val)
    with pytest.raises(ValueError):
        probes.encode(probes.E4M3, 0, 1, 9)
    with pytest.raises(ValueError):
        probes.encode(probes.FP16, 0, 1, -25)


def test_step1_independence_on_the_oracle():
    iface = OracleInterface(ModelParams(group_len=8, frac_bits=24), 4, 4, 16, fm.FP16, fm.FP16)
    assert probes.independence(iface, trials=8)

    class Coupled(OracleInterface):          # an interface whose outputs depend on the column index
        def __call__(self, A, B, C):
            D = super().__call__(A, B, C)
            D[:, :, 1] ^= 1
            return D
    assert not probes.independence(Coupled(iface.p, 4, 4, 16, fm.FP16, fm.FP16), trials=4)


@pytest.mark.parametrize("p,k,t,want", [
    # T-FDPA with the accumulator inside, one group: a single swamped fused sum of K + 1 terms (Fig. (d))
    (ModelParams(group_len=4, frac_bits=24), 4, fm.FP16, "F[p0, p1, p2, p3, p4]"),
    # chained groups of 4 with the accumulator inside each group
    (ModelParams(group_len=4, frac_bits=24), 8, fm.FP16, "F[F[p0, p1, p2, p3, p8], p4, p5, p6, p7]"),
    # wide F: nothing is swamped inside a group (Fig. (c) generalised)
    (ModelParams(group_len=4, frac_bits=60), 8, fm.FP16, "Fx[Fx[p0, p1, p2, p3, p8], p4, p5, p6, p7]"),
    # the accumulator added exactly after the fused sum of the products: a binary sum above each fused group
    (ModelParams(group_len=4, frac_bits=24, c_mode=C_AFTER_EXACT), 8, fm.FP16, "((F[p0, p1, p2, p3] + p8) + F[p4, p5, p6, p7])"),
    # TR-FDPA: the accumulator is aligned at E = max(e_max, e_c) and rounded down to F bits even when the products
    # cancel, so a small accumulator is lost next to +-U products: the group reads as a swamped (L+1)-term fused sum
    (ModelParams(group_len=4, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD), 8, fm.BF16, "F[F[p0, p1, p2, p3, p8], p4, p5, p6, p7]"),
    # two sub-groups merged with RD at 24 bits at their common maximum: small sums of the other half are lost
    # too, and Step 2 sees one flat fused sum (the halves only show in Step 3, as two different precisions)
    (ModelParams(group_len=8, frac_bits=13, frac_bits_merge=24, frac_bits_acc=24, frac_bits2=31, c_mode=C_AFTER_RD, split=SPLIT_HALVES),
     8, fm.E5M2, "F[p0, p1, p2, p3, p4, p5, p6, p7, p8]"),
])
def test_step2_tree_of_oracle_models(p, k, t, want):
    iface = OracleInterface(p, 2, 2, k, t, t)
    table = probes.summation_table(iface)
    assert probes.tree_to_string(probes.infer_tree(table)) == want


def test_step2_reproduces_the_papers_walkthrough():
    # the footnote of Step 2: chain ((((c + p0) + p1) + p2) + p3), i = 0, j = 1 gives d / v = 2
    iface = OracleInterface(ModelParams(group_len=1, frac_bits=60), 1, 1, 4, fm.FP16, fm.FP16)
    table = probes.summation_table(iface)
    assert table[0][1] == 2
    assert [r[i + 1:] for i, r in enumerate(table[:4])] == _trees()["a_chain_of_binary_sums"]


def test_step3_precision_and_rounding_on_oracle_models():
    for F in (13, 24, 27):
        iface = OracleInterface(ModelParams(group_len=8, frac_bits=F), 1, 1, 8, fm.BF16, fm.BF16)
        assert probes.fused_precision(iface, 0, 1, 2) == F
    # the RD mode: products keep F bits among themselves
    iface = OracleInterface(ModelParams(group_len=8, frac_bits=13, frac_bits2=31, frac_bits_acc=24, c_mode=C_AFTER_RD), 1, 1, 8, fm.E5M2, fm.E5M2)
    assert probes.fused_precision(iface, 0, 1, 2) == 13
    # exact as far as an E5M2 product can go down (62 binary places below the largest)
    iface = OracleInterface(ModelParams(group_len=8, frac_bits=64), 1, 1, 8, fm.E5M2, fm.E5M2)
    assert probes.fused_precision(iface, 0, 1, 2) is None
    # output conversion seen through a wide fused sum
    for rho, name in ((RNE, "RNE"), (RZ, "RZ")):
        iface = OracleInterface(ModelParams(group_len=8, frac_bits=60, out_round=rho), 1, 1, 8, fm.BF16, fm.BF16)
        assert probes.rounding_mode(iface, 0, 1, 23) == name
    # the accumulator's round-down in the RD mode: c small and negative / positive against a product of U
    iface = OracleInterface(ModelParams(group_len=8, frac_bits=24, frac_bits2=31, c_mode=C_AFTER_RD), 1, 1, 8, fm.BF16, fm.BF16)
    # RD to 24 bits (half a binary32 place) followed by RNE: +0.75 -> +0.5 -> tie to even (down), -0.75 -> -1 (away),
    # +-0.25 -> 0 / -0.5 -> tie to even (toward zero)
    assert probes.rounding_mode(iface, 0, 8, 23) == "composite ZZAZ"
    # with a coarser round-down (F_c = 20) the binary32 output no longer hides it
    iface = OracleInterface(ModelParams(group_len=8, frac_bits=24, frac_bits2=31, frac_bits_acc=20, c_mode=C_AFTER_RD), 1, 1, 8, fm.BF16, fm.BF16)
    assert probes.rounding_mode(iface, 0, 8, 20) == "RD"
