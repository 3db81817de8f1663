"""mmaemu_generate_noalloc (the entry point for callers that cannot allocate) against mmaemu_generate, bit for bit.

Two calls in a row through the C-ABI, the second smaller than the first, so that what the first call left in the
library's static device array cannot leak into the second; then every scale scope and an unscaled family.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from gpu_utils import to_host


@pytest.fixture(scope="module")
def mm():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2511_10909_amd import binding
    return binding


def _both(mm, dtype, np_dtype, ept, first_tile, n_tiles, **kw):
    import torch
    tdt = {np.uint8: torch.uint8, np.uint16: torch.int16, np.uint32: torch.int32}[np_dtype]
    ref = torch.zeros(n_tiles * ept, dtype=tdt, device="cuda")
    got = torch.zeros(n_tiles * ept, dtype=tdt, device="cuda")
    ws = torch.zeros(8, dtype=torch.uint8, device="cuda")
    mm.generate(ref, dtype, ept, first_tile, n_tiles, workspace=ws, **kw)
    mm.generate_noalloc(got, dtype, ept, first_tile, n_tiles, **kw)
    return to_host(ref, np_dtype), to_host(got, np_dtype)


def test_noalloc_matches_generate_on_two_calls_in_a_row(mm):
    kw = dict(family=mm.GEN_NORMAL, seed=7, operand=0, scale_scope=mm.SCALE_TENSOR, scale_target=448.0)
    # first call: 3000 tiles of 300 elements (ragged against the 4-element random blocks and the 256-thread workgroups)
    ref, got = _both(mm, mm.E4M3, np.uint8, 300, 5, 3000, **kw)
    assert np.array_equal(ref, got)
    assert (got & 0x7F).max() == 0x7E                       # scaled so that the largest magnitude is 448
    # second call, smaller, other seed and target: a maximum left over from the first call would change the scale
    kw2 = dict(family=mm.GEN_NORMAL, seed=8, operand=1, scale_scope=mm.SCALE_TENSOR, scale_target=57344.0)
    ref2, got2 = _both(mm, mm.E5M2, np.uint8, 64, 0, 17, **kw2)
    assert np.array_equal(ref2, got2)
    assert (got2 & 0x7F).max() == 0x7B


@pytest.mark.parametrize("scope", ["none", "tile", "tensor"])
def test_noalloc_matches_generate_every_scope(mm, scope):
    sc = dict(none=mm.SCALE_NONE, tile=mm.SCALE_TILE, tensor=mm.SCALE_TENSOR)[scope]
    for fam in (mm.GEN_NORMAL, mm.GEN_UNIFORM, mm.GEN_NORMAL_OUTLIERS):
        ref, got = _both(mm, mm.BF16, np.uint16, 256, 3, 129, family=fam, seed=3, operand=2, scale_scope=sc, scale_target=2.0)
        assert np.array_equal(ref, got), (scope, fam)
    ref, got = _both(mm, mm.FP32, np.uint32, 1000, 0, 33, family=mm.GEN_UNIFORM_EXP, seed=1, operand=0, exp_lo=1, exp_hi=254)
    assert np.array_equal(ref, got)


def test_noalloc_rejects_calls_over_its_limit(mm):
    with pytest.raises(mm.MmaemuError) as ei:
        mm.generate_noalloc(0x1000, mm.FP16, 1 << 20, 0, (1 << 20) + 1, family=mm.GEN_NORMAL, scale_scope=mm.SCALE_TENSOR, stream=0)
    assert ei.value.status == 3 and "2^40" in mm.last_error()
    mm.generate_noalloc(None, mm.FP16, 256, 0, 0, family=mm.GEN_NORMAL, stream=0)        # no tiles: nothing to do
