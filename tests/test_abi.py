"""The C-ABI library loads without a GPU and exports every function the public header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mmaemu.h")
LIB = os.path.join(ROOT, "paper_2511_10909_amd", "libmmaemu.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2511_10909_amd.build import build_library
        build_library(verbose=False)
    return ctypes.CDLL(LIB)


def declared_functions():
    with open(HEADER) as fh:
        text = fh.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmaemu_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for required in ("mmaemu_model_create", "mmaemu_model_destroy", "mmaemu_emulate_mma", "mmaemu_compare",
                     "mmaemu_stats_reset", "mmaemu_generate", "mmaemu_mfma_probe", "mmaemu_exact_dot_sample",
                     "mmaemu_status_string", "mmaemu_last_error"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_struct_sizes_match_binding():
    from paper_2511_10909_amd import binding as mm
    assert ctypes.sizeof(mm.ModelParams) == 96
    assert ctypes.sizeof(mm.Stats) == 8 * 39
    assert ctypes.sizeof(mm.ErrStats) == 8 * 44
    assert ctypes.sizeof(mm.GenParams) == 48


def test_host_side_validation_needs_no_gpu():
    from paper_2511_10909_amd import binding as mm
    h = mm.model_create(group_len=8, frac_bits=24)
    assert mm.model_get_params(h)["group_len"] == 8
    mm.model_destroy(h)
    mm.model_destroy(None)
    for kw, status in ((dict(frac_bits=49), 2), (dict(frac_bits=41, frac_bits2=31, c_mode=2), 2), (dict(out_round=2), 1), (dict(c_mode=5), 1), (dict(align_round=1), 2),
                       (dict(out_mant_bits=13), 2), (dict(out_mant_bits=10, out_round=1), 2), (dict(frac_bits2=31), 2), (dict(c_mode=2, frac_bits2=49), 2), (dict(split=1), 2), (dict(c_mode=2, split=4), 1),
                       (dict(c_mode=3, frac_bits2=31, frac_bits_acc=24), 2), (dict(c_mode=2, frac_bits_merge=24), 2), (dict(skip_zero_terms=2), 1), (dict(family=3), 1), (dict(family=2), 2), (dict(family=1, group_len=8), 2), (dict(family=1, group_len=4, ftz_out=True), 2), (dict(struct_size=40), 1), (dict(group_len=(1 << 20) + 1), 2)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.model_create(**kw)
        assert ei.value.status == status, kw
    assert "frac_bits" in mm.last_error() or "group_len" in mm.last_error()
    mm.model_destroy(mm.model_create(group_len=16, frac_bits=13, out_round=mm.RZ, out_mant_bits=13))
    for mode in (mm.C_AFTER_RD, mm.C_AFTER_RD_EVEN_ODD):
        h = mm.model_create(group_len=8, frac_bits=24, frac_bits2=31, c_mode=mode)
        assert mm.model_get_params(h)["frac_bits2"] == 31
        mm.model_destroy(h)
    info = mm.mfma_info(mm.MFMA_F32_16X16X32_FP8_BF8)
    assert info == dict(m=16, n=16, k=32, a=mm.E4M3, b=mm.E5M2)
    with pytest.raises(mm.MmaemuError):
        mm.mfma_info(99)
