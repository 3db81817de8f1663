"""Exhaustive k = 2 sweep on the GPU: ALL 2^32 (a0, b0, a1, b1) code tuples of each of the four FP8 type pairings, as
1 x 1 x 2 tiles through mmaemu_emulate_mma, for three internal widths (nothing cut that 40 bits hold; F = 13, the
paper's FP8 setting; F = 4).  Expected values: the oracle's outputs for every ordered pair of product classes
(tests/k2_sweep.py; tests/test_oracle_k2.py proves those tables equal to binary64 closed forms and shows that the class
of a code pair is all the model sees), looked up per tuple.  torch does the bookkeeping (code tuples, table lookups,
the count of differing words); every output comes from the library, every expected value from the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import formats as fm, o2lib
from oracle.fdpa import ModelParams
from k2_sweep import PAIRINGS, product_classes, class_pair_operands
from test_gpu_parity import mm  # noqa: F401


@pytest.mark.parametrize("ta,tb", PAIRINGS)
def test_all_fp8_tuples_k2(mm, ta, tb):
    import torch
    cls, reps, info = product_classes(ta, tb)
    n = len(reps)
    A2, B2 = class_pair_operands(reps)
    dev = "cuda"
    cls_d = torch.from_numpy(cls.astype(np.int64)).to(dev)
    chunk = 1 << 28
    A = torch.empty((chunk, 1, 2), dtype=torch.uint8, device=dev)
    B = torch.empty((chunk, 1, 2), dtype=torch.uint8, device=dev)
    C = torch.zeros((chunk, 1, 1), dtype=torch.int32, device=dev)
    D = torch.empty((chunk, 1, 1), dtype=torch.int32, device=dev)
    dt = (ta, tb, mm.FP32, mm.FP32)
    for F in (40, 13, 4):
        table, _ = o2lib.emulate_mma(ModelParams(group_len=2, frac_bits=F), A2, B2, np.zeros((n * n, 1, 1), np.uint32), ta, tb)
        table_d = torch.from_numpy(table.reshape(-1).view(np.int32)).to(dev)
        h = mm.model_create(group_len=2, frac_bits=F)
        total_bad = 0
        for c in range((1 << 32) // chunk):
            t = torch.arange(c * chunk, (c + 1) * chunk, dtype=torch.int64, device=dev)      # tuple = a0 | b0 << 8 | a1 << 16 | b1 << 24
            A[:, 0, 0] = (t & 255).to(torch.uint8)
            B[:, 0, 0] = ((t >> 8) & 255).to(torch.uint8)
            A[:, 0, 1] = ((t >> 16) & 255).to(torch.uint8)
            B[:, 0, 1] = ((t >> 24) & 255).to(torch.uint8)
            mm.emulate_mma(h, A, B, C, D, 1, 1, 2, chunk, dt)
            assert mm.last_kernel() == "general"
            want = table_d[cls_d[t & 0xFFFF] * n + cls_d[t >> 16]]
            bad = int((D.view(-1) != want).sum().item())
            if bad:
                i = int(torch.nonzero(D.view(-1) != want)[0].item())
                pytest.fail("F=%d: %d of 2^28 tuples differ in chunk %d, first tuple %#x: gpu %#x, oracle %#x"
                            % (F, bad, c, c * chunk + i, int(D.view(-1)[i].item()) & 0xFFFFFFFF, int(want[i].item()) & 0xFFFFFFFF))
            total_bad += bad
            del t, want
        mm.model_destroy(h)
        assert total_bad == 0
