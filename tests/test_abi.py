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
    assert ctypes.sizeof(mm.ModelParams) == 100
    assert ctypes.sizeof(mm.DeviationHist) == 8 * 72
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
                       (dict(c_mode=3, frac_bits2=31, frac_bits_acc=24), 2), (dict(c_mode=2, frac_bits_merge=24), 2), (dict(skip_zero_terms=2), 1), (dict(family=4), 1), (dict(family=2), 2), (dict(family=1, group_len=8), 2), (dict(family=1, group_len=4, ftz_out=True), 2), (dict(struct_size=40), 1),
                       (dict(rd_toward_zero=True), 2), (dict(c_mode=2, frac_bits2=31, rd_toward_zero=2), 2), (dict(group_len=(1 << 20) + 1), 2)):
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


def test_emulate_rejects_bad_arguments_before_any_gpu_call():
    """Every check of mmaemu_emulate_mma's arguments runs on the host: fake addresses never reach a kernel."""
    from paper_2511_10909_amd import binding as mm
    h = mm.model_create(group_len=8, frac_bits=24)
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    ok = 0x1000
    cases = [
        (dict(A=ok + 1), 1),          # FP16 operand at an odd address
        (dict(C=ok + 2), 1),          # FP32 accumulator off a 4-byte boundary
        (dict(D=ok + 1), 1),
        (dict(A=None), 1),
        (dict(k=12), 3),              # k is not a multiple of the group length
        (dict(m=0), 3),
        (dict(k=(1 << 20) + 8), 3),
    ]
    for change, status in cases:
        a = dict(A=ok, B=ok, C=ok, D=ok, m=16, n=16, k=16, batch=1)
        a.update(change)
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma(h, a["A"], a["B"], a["C"], a["D"], a["m"], a["n"], a["k"], a["batch"], dt, stream=0)
        assert ei.value.status == status, (change, mm.last_error())
    # batch = 0 is a no-op whatever the pointers are
    mm.emulate_mma(h, None, None, None, None, 16, 16, 16, 0, dt, stream=0)
    with pytest.raises(mm.MmaemuError) as ei:
        mm.emulate_mma(h, ok, ok, ok, ok, 16, 16, 16, 1, (mm.TF32, mm.FP16, mm.FP32, mm.FP32), stream=0)
    assert ei.value.status == 2
    mm.model_destroy(h)


def test_fma_family_argument_checks():
    from paper_2511_10909_amd import binding as mm
    for kw in (dict(group_len=2), dict(ftz_in=True), dict(out_round=mm.RZ), dict(c_mode=mm.C_AFTER_EXACT), dict(out_mant_bits=13, out_round=mm.RZ)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.model_create(family=mm.FAMILY_FMA, **kw)
        assert ei.value.status == 2, kw
    h = mm.model_create(family=mm.FAMILY_FMA, group_len=1)
    ok = 0x1000
    for dt in ((mm.BF16, mm.BF16, mm.FP32, mm.FP32), (mm.TF32, mm.TF32, mm.FP32, mm.FP32), (mm.FP32, mm.FP32, mm.FP16, mm.FP16)):
        with pytest.raises(mm.MmaemuError) as ei:
            mm.emulate_mma(h, ok, ok, ok, ok, 16, 16, 4, 1, dt, stream=0)
        assert ei.value.status == 2, dt
    with pytest.raises(mm.MmaemuError):
        mm.emulate_mma_scaled(h, ok, ok, ok, ok, ok, ok, 4, 16, 16, 4, 1, (mm.FP32,) * 4, stream=0)
    mm.emulate_mma(h, None, None, None, None, 16, 16, 4, 0, (mm.FP32,) * 4, stream=0)     # batch = 0: no-op
    mm.model_destroy(h)


def test_compare_many_classes_is_a_host_side_query():
    """Which models mmaemu_emulate_compare_many runs in common launches: decided on the host, no GPU needed."""
    from paper_2511_10909_amd import binding as mm
    rd = dict(group_len=8, frac_bits=24, frac_bits2=31, c_mode=mm.C_AFTER_RD)
    sets = [dict(group_len=8, frac_bits=24), dict(group_len=16, frac_bits=32, out_round=mm.RZ, ftz_in=True),      # T-FDPA: class 0
            rd, dict(rd, f2_at_leading_bit=True, sum_drop_distance=28, acc_special_truncation=True),               # TR-FDPA: class 1
            dict(rd, skip_zero_terms=True), dict(rd, skip_zero_terms=True, ftz_in=True),                           # zero terms out of the maxima: 2, 3
            dict(rd, split=mm.SPLIT_HALVES),                                                                       # halves / quarters: 4 to 6
            dict(group_len=8, frac_bits=24, c_mode=mm.C_AFTER_EXACT), dict(rd, split=mm.SPLIT_EVEN_ODD),           # not in the scan kernel; even / odd: 7 to 9
            dict(group_len=2, frac_bits=24), dict(group_len=8, frac_bits=44)]
    hs = [mm.model_create(**kw) for kw in sets]
    dt = (mm.FP16, mm.FP16, mm.FP32, mm.FP32)
    assert mm.compare_many_classes(hs, 16, 16, 16, dt) == [0, 0, 1, 1, 2, 3, 4, -1, 7, -1, -1]
    assert mm.compare_many_classes(hs[:6], 32, 32, 16, dt) == [0, 0, 1, 1, 2, 3]
    assert mm.compare_many_classes(hs[:6], 16, 16, 32, (mm.BF16, mm.BF16, mm.FP32, mm.FP32)) == [0, 0, 1, 1, 2, 3]
    assert mm.compare_many_classes(hs[:3], 16, 16, 64, dt) == [-1, -1, -1]          # shapes the kernel does not stage whole
    assert mm.compare_many_classes(hs[:3], 20, 20, 16, dt) == [-1, -1, -1]
    assert mm.compare_many_classes(hs[:3], 16, 16, 16, (mm.TF32, mm.TF32, mm.FP32, mm.FP32)) == [-1, -1, -1]
    wide = mm.model_create(**dict(rd, wide_products=True))
    assert mm.compare_many_classes([wide], 16, 16, 16, (mm.BF16, mm.BF16, mm.FP32, mm.FP32)) == [-1]
    assert mm.compare_many_classes([wide], 16, 16, 16, dt) == [1]
    quarters = [mm.model_create(**dict(rd, group_len=16, frac_bits=13, split=mm.SPLIT_QUARTERS, skip_zero_terms=True, ftz_in=f)) for f in (False, True)]
    assert mm.compare_many_classes(quarters, 16, 16, 32, (mm.E4M3, mm.E5M2, mm.FP32, mm.FP32)) == [5, 6]
    assert mm.compare_many_classes(quarters, 16, 16, 32, (mm.BF16, mm.BF16, mm.FP32, mm.FP32)) == [-1, -1]     # (binary32 values only)
    assert mm.compare_many_classes(quarters, 32, 32, 8, dt) == [-1, -1]                                         # (the group is the whole k = 8: no quarters of four)
    for h in quarters:
        mm.model_destroy(h)
    for h in hs + [wide]:
        mm.model_destroy(h)
