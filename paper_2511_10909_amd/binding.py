"""ctypes binding of libmmaemu: same names as the C entry points, argument marshalling only.

Device memory and streams come from PyTorch (tensors are passed as their data_ptr(), the
stream as torch's current HIP stream handle); every computation happens inside the library.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmmaemu.so")

E4M3, E5M2, FP16, BF16, FP32, E8M0 = 0, 1, 2, 3, 4, 5
E2M3, E3M2, E2M1 = 6, 7, 8                      # FP6 and FP4 operands, one code per byte
TF32 = 9                                        # binary32 words whose low 13 mantissa bits are ignored
FP64 = 10                                       # binary64: the FMA family, the generators, the comparison, two MFMA forms
C_IN_GROUP, C_AFTER_EXACT, C_AFTER_RD, C_AFTER_RD_EVEN_ODD, C_EXACT = 0, 1, 2, 3, 4
RNE, RZ = 0, 1
SPLIT_NONE, SPLIT_EVEN_ODD, SPLIT_HALVES, SPLIT_QUARTERS = 0, 1, 2, 3
FAMILY_FDPA, FAMILY_FTZ_ADDMUL, FAMILY_GST_FDPA, FAMILY_FMA = 0, 1, 2, 3
SCALE_FORMAT_E8M0, SCALE_FORMAT_UE4M3 = 0, 1
GEN_ZERO, GEN_FINITE_BITS, GEN_UNIFORM_EXP, GEN_RANDOM_BITS, GEN_NORMAL = 0, 1, 2, 3, 4
GEN_UNIFORM, GEN_NORMAL_OUTLIERS, GEN_CANCELLING, GEN_SIGNED_ZEROS = 5, 6, 7, 8
SCALE_NONE, SCALE_TENSOR, SCALE_TILE, SCALE_FACTOR = 0, 1, 2, 3
(MFMA_F32_16X16X16_F16, MFMA_F32_16X16X16_BF16, MFMA_F32_32X32X8_F16, MFMA_F32_32X32X8_BF16,
 MFMA_F32_16X16X32_F16, MFMA_F32_16X16X32_BF16, MFMA_F32_16X16X32_FP8_FP8, MFMA_F32_16X16X32_FP8_BF8,
 MFMA_F32_16X16X32_BF8_FP8, MFMA_F32_16X16X32_BF8_BF8) = range(10)
# v_mfma_scale_f32_16x16x128_f8f6f4: id = base + 5 fa + fb, formats numbered 0 E4M3, 1 E5M2, 2 E2M3, 3 E3M2, 4 E2M1
MFMA_SCALE_BASE = 10
MFMA_SCALE_FORMATS = (0, 1, 6, 7, 8)            # dtype ids in the instruction's numbering


MFMA_SCALE32_BASE = 43                          # v_mfma_scale_f32_32x32x64_f8f6f4, numbered the same way


def mfma_scale_id(ta, tb, m=16):
    """Instruction id of the block-scaled MFMA (m = 16: 16x16x128, m = 32: 32x32x64) with operand types ta (A) and tb (B)."""
    return (MFMA_SCALE_BASE if m == 16 else MFMA_SCALE32_BASE) + 5 * MFMA_SCALE_FORMATS.index(ta) + MFMA_SCALE_FORMATS.index(tb)


MFMA_SCALE_F32_16X16X128_FP8_FP8, MFMA_SCALE_F32_16X16X128_FP8_BF8 = 10, 11
MFMA_SCALE_F32_16X16X128_BF8_FP8, MFMA_SCALE_F32_16X16X128_BF8_BF8 = 15, 16
MFMA_SCALE_FP8_IDS = (10, 11, 15, 16)
MFMA_SCALE_IDS = tuple(range(10, 35))
MFMA_SCALE32_IDS = tuple(range(43, 68))
(MFMA_F32_32X32X16_F16, MFMA_F32_32X32X16_BF16, MFMA_F32_32X32X16_FP8_FP8, MFMA_F32_32X32X16_FP8_BF8,
 MFMA_F32_32X32X16_BF8_FP8, MFMA_F32_32X32X16_BF8_BF8) = range(35, 41)
MFMA_F32_16X16X4_F32, MFMA_F32_32X32X2_F32 = 41, 42
# multi-block forms (one issue = 64 / m tiles): 32x32x4_2b, 16x16x4_4b, 4x4x4_16b for FP16 and BF16; 32x32x1_2b, 16x16x1_4b, 4x4x1_16b for FP32
MFMA_MULTIBLOCK_F16_IDS, MFMA_MULTIBLOCK_BF16_IDS, MFMA_MULTIBLOCK_F32_IDS = (68, 69, 70), (71, 72, 73), (74, 75, 76)
MFMA_F64_16X16X4_F64, MFMA_F64_4X4X4_4B_F64 = 77, 78
MFMA_UNSCALED_IDS = tuple(range(10)) + tuple(range(35, 43)) + tuple(range(68, 79))
ELEM_BYTES = {E4M3: 1, E5M2: 1, FP16: 2, BF16: 2, FP32: 4, E8M0: 1, E2M3: 1, E3M2: 1, E2M1: 1, TF32: 4, FP64: 8}
NO_MISMATCH = (1 << 64) - 1


class MmaemuError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libmmaemu: %s (status %d): %s" % (_status_string(status), status, text))
        self.status = status


class ModelParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("struct_size", "group_len", "frac_bits", "align_round", "c_mode", "frac_bits2", "out_round",
                 "out_mant_bits", "ftz_in", "ftz_out", "nan_bits", "split", "acc_special_truncation",
                 "frac_bits_merge", "frac_bits_acc", "f2_at_leading_bit", "skip_zero_terms", "zero_result_positive",
                 "sum_drop_distance", "family", "wide_products", "gst_group", "scale_format", "nan_propagate", "rd_toward_zero")]


class Dtypes(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("a", "b", "c", "d")]


class GenParams(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("family", ctypes.c_uint32), ("seed", ctypes.c_uint64),
                ("operand", ctypes.c_uint32), ("exp_lo", ctypes.c_uint32), ("exp_hi", ctypes.c_uint32),
                ("exp_zero", ctypes.c_uint32), ("scale_scope", ctypes.c_uint32), ("scale_target", ctypes.c_double)]


class Stats(ctypes.Structure):
    _fields_ = [("n_compared", ctypes.c_uint64), ("n_mismatch_bits", ctypes.c_uint64),
                ("n_mismatch_nan_equiv", ctypes.c_uint64), ("first_mismatch_index", ctypes.c_uint64),
                ("max_ulp_dist", ctypes.c_uint64), ("ulp_hist", ctypes.c_uint64 * 34)]


class ErrStats(ctypes.Structure):
    _fields_ = [("n_samples", ctypes.c_uint64), ("n_equal_rne", ctypes.c_uint64), ("n_above", ctypes.c_uint64),
                ("n_below", ctypes.c_uint64), ("n_skipped", ctypes.c_uint64), ("ulp_hist", ctypes.c_uint64 * 34),
                ("sum_abs_err", ctypes.c_double), ("max_abs_err", ctypes.c_double), ("sum_rel_err", ctypes.c_double),
                ("max_rel_err", ctypes.c_double), ("sum_signed_err", ctypes.c_double)]


DEVIATION_BINS = 64


class DeviationHist(ctypes.Structure):
    _fields_ = [("n_samples", ctypes.c_uint64), ("n_skipped", ctypes.c_uint64), ("n_negative", ctypes.c_uint64),
                ("n_zero", ctypes.c_uint64), ("n_positive", ctypes.c_uint64), ("bins", ctypes.c_uint64 * DEVIATION_BINS),
                ("sum", ctypes.c_double), ("sum_abs", ctypes.c_double), ("sum_sq", ctypes.c_double)]


STATS_BYTES = ctypes.sizeof(Stats)
ERR_STATS_BYTES = ctypes.sizeof(ErrStats)
DEVIATION_HIST_BYTES = ctypes.sizeof(DeviationHist)

if not os.path.exists(LIB_PATH):
    raise ImportError("libmmaemu.so is not built (%s); run `python -m paper_2511_10909_amd.build` or "
                      "__graft_entry__.build() first -- there is no fallback path" % LIB_PATH)
# PyTorch first: it ships its own HIP runtime, and the library must bind to that same copy (tensors and streams
# come from it).  Loaded the other way round, the library's runtime is a second one that sees no device.
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(LIB_PATH)

_vp, _u32, _u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
_lib.mmaemu_status_string.restype = ctypes.c_char_p
_lib.mmaemu_status_string.argtypes = [ctypes.c_int]
_lib.mmaemu_last_error.restype = ctypes.c_char_p
_lib.mmaemu_last_kernel.restype = ctypes.c_char_p
_lib.mmaemu_version.restype = _u32
_lib.mmaemu_model_create.argtypes = [ctypes.POINTER(ModelParams), ctypes.POINTER(_vp)]
_lib.mmaemu_model_destroy.argtypes = [_vp]
_lib.mmaemu_model_get_params.argtypes = [_vp, ctypes.POINTER(ModelParams)]
_lib.mmaemu_emulate_mma.argtypes = [_vp, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _u64, Dtypes, _vp]
_lib.mmaemu_emulate_mma_scaled.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _u32, _u64, Dtypes, _vp]
_lib.mmaemu_emulate_compare_many.argtypes = [ctypes.POINTER(_vp), _u32, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _u64, Dtypes, _u64, _vp, _vp]
_lib.mmaemu_compare_many_classes.argtypes = [ctypes.POINTER(_vp), _u32, _u32, _u32, _u32, Dtypes, ctypes.POINTER(ctypes.c_int32)]
_lib.mmaemu_stats_reset.argtypes = [_vp, _vp]
_lib.mmaemu_compare.argtypes = [_vp, _vp, _u64, _u64, ctypes.c_int, _vp, _vp]
_lib.mmaemu_generate.argtypes = [ctypes.POINTER(GenParams), _vp, ctypes.c_int, _u64, _u64, _u64, _vp, _vp]
_lib.mmaemu_generate_noalloc.argtypes = [ctypes.POINTER(GenParams), _vp, ctypes.c_int, _u64, _u64, _u64, _vp]
_lib.mmaemu_mfma_info.argtypes = [ctypes.c_int] + [ctypes.POINTER(_u32)] * 3 + [ctypes.POINTER(ctypes.c_int)] * 2
_lib.mmaemu_mfma_probe.argtypes = [ctypes.c_int, _vp, _vp, _vp, _vp, _u32, _u64, _vp]
_lib.mmaemu_mfma_probe_scaled.argtypes = [ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _u64, _vp]
_lib.mmaemu_issue_probe_count.restype = _u32
_lib.mmaemu_issue_probe_name.restype = ctypes.c_char_p
_lib.mmaemu_issue_probe_name.argtypes = [_u32]
_lib.mmaemu_issue_probe.argtypes = [_u32, _u32, _u32, _vp, _vp]
_lib.mmaemu_err_stats_reset.argtypes = [_vp, _vp]
_lib.mmaemu_exact_dot_sample.argtypes = [_vp, _vp, _vp, _u32, _u32, _u32, Dtypes, _u64, _vp, _vp]
_lib.mmaemu_deviation_hist_reset.argtypes = [_vp, _vp]
_lib.mmaemu_deviation_sample.argtypes = [_vp, _vp, _vp, _vp, _u32, _u32, _u32, _u64, Dtypes, _u64, ctypes.c_int32, _vp, _vp]


def _status_string(s):
    return _lib.mmaemu_status_string(int(s)).decode()


def _check(status):
    if status != 0:
        raise MmaemuError(status, _lib.mmaemu_last_error().decode())


def _ptr(x):
    """Device pointer of a torch tensor (or a raw integer address / None)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def version():
    return int(_lib.mmaemu_version())


def last_kernel():
    return _lib.mmaemu_last_kernel().decode()


def last_error():
    return _lib.mmaemu_last_error().decode()


def model_create(group_len=0, frac_bits=24, c_mode=C_IN_GROUP, out_round=RNE, ftz_in=False, ftz_out=False,
                 nan_bits=0x7FC00000, align_round=0, frac_bits2=0, out_mant_bits=23, struct_size=None,
                 split=SPLIT_NONE, acc_special_truncation=False, frac_bits_merge=0, frac_bits_acc=0,
                 f2_at_leading_bit=False, skip_zero_terms=False, zero_result_positive=False, sum_drop_distance=0,
                 family=FAMILY_FDPA, wide_products=False, gst_group=0, scale_format=0, nan_propagate=False, rd_toward_zero=False):
    p = ModelParams(ctypes.sizeof(ModelParams) if struct_size is None else struct_size, group_len, frac_bits,
                    align_round, c_mode, frac_bits2, out_round, out_mant_bits, int(ftz_in), int(ftz_out), nan_bits,
                    split, int(acc_special_truncation), frac_bits_merge, frac_bits_acc, int(f2_at_leading_bit),
                    int(skip_zero_terms), int(zero_result_positive), sum_drop_distance, family, int(wide_products), gst_group, scale_format,
                    int(nan_propagate), int(rd_toward_zero))
    h = _vp()
    _check(_lib.mmaemu_model_create(ctypes.byref(p), ctypes.byref(h)))
    return h


def model_destroy(model):
    _check(_lib.mmaemu_model_destroy(model))


def model_get_params(model):
    p = ModelParams()
    _check(_lib.mmaemu_model_get_params(model, ctypes.byref(p)))
    return {n: getattr(p, n) for n, _ in ModelParams._fields_}


def emulate_mma(model, A, B, C, D, m, n, k, batch, dtypes, stream=None):
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    _check(_lib.mmaemu_emulate_mma(model, _ptr(A), _ptr(B), _ptr(C), _ptr(D), m, n, k, batch, dt, _stream(stream)))


def emulate_mma_scaled(model, A, B, C, D, SA, SB, block, m, n, k, batch, dtypes, stream=None):
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    _check(_lib.mmaemu_emulate_mma_scaled(model, _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(SA), _ptr(SB), block, m, n, k, batch, dt,
                                          _stream(stream)))


def emulate_compare_many(models, A, B, C, Dref, D_out, m, n, k, batch, dtypes, dev_stats, index_base=0, stream=None):
    """dev_stats: device memory for len(models) statistics structs (a uint8 tensor of len(models) * STATS_BYTES)."""
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    arr = (_vp * len(models))(*[h if isinstance(h, _vp) else _vp(h) for h in models])
    _check(_lib.mmaemu_emulate_compare_many(arr, len(models), _ptr(A), _ptr(B), _ptr(C), _ptr(Dref), _ptr(D_out), m, n, k, batch, dt,
                                            index_base, _ptr(dev_stats), _stream(stream)))


def compare_many_classes(models, m, n, k, dtypes):
    """Per model, the class under which emulate_compare_many launches it (equal numbers share launches), -1 if it runs unfused."""
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    arr = (_vp * len(models))(*[h if isinstance(h, _vp) else _vp(h) for h in models])
    out = (ctypes.c_int32 * len(models))()
    _check(_lib.mmaemu_compare_many_classes(arr, len(models), m, n, k, dt, out))
    return list(out)


def stats_reset(dev_stats, stream=None):
    _check(_lib.mmaemu_stats_reset(_ptr(dev_stats), _stream(stream)))


def compare(D0, D1, count, dev_stats, index_base=0, d=FP32, stream=None):
    _check(_lib.mmaemu_compare(_ptr(D0), _ptr(D1), count, index_base, d, _ptr(dev_stats), _stream(stream)))


def generate(out, dtype, elems_per_tile, first_tile, n_tiles, family, seed=0, operand=0, exp_lo=0, exp_hi=0,
             exp_zero=False, scale_scope=SCALE_NONE, scale_target=1.0, workspace=None, stream=None, struct_size=None):
    g = GenParams(ctypes.sizeof(GenParams) if struct_size is None else struct_size, family, seed, operand,
                  exp_lo, exp_hi, int(exp_zero), scale_scope, scale_target)
    _check(_lib.mmaemu_generate(ctypes.byref(g), _ptr(out), dtype, elems_per_tile, first_tile, n_tiles,
                                _ptr(workspace), _stream(stream)))


def generate_noalloc(out, dtype, elems_per_tile, first_tile, n_tiles, family, seed=0, operand=0, exp_lo=0, exp_hi=0,
                     exp_zero=False, scale_scope=SCALE_NONE, scale_target=1.0, stream=None):
    g = GenParams(ctypes.sizeof(GenParams), family, seed, operand, exp_lo, exp_hi, int(exp_zero), scale_scope, scale_target)
    _check(_lib.mmaemu_generate_noalloc(ctypes.byref(g), _ptr(out), dtype, elems_per_tile, first_tile, n_tiles, _stream(stream)))


def mfma_info(instr):
    m, n, k = _u32(), _u32(), _u32()
    a, b = ctypes.c_int(), ctypes.c_int()
    _check(_lib.mmaemu_mfma_info(instr, ctypes.byref(m), ctypes.byref(n), ctypes.byref(k), ctypes.byref(a), ctypes.byref(b)))
    return dict(m=m.value, n=n.value, k=k.value, a=a.value, b=b.value)


def mfma_probe(instr, A, B, C, D, k, batch, stream=None):
    _check(_lib.mmaemu_mfma_probe(instr, _ptr(A), _ptr(B), _ptr(C), _ptr(D), k, batch, _stream(stream)))


def mfma_probe_scaled(instr, A, B, C, D, SA, SB, k, batch, stream=None):
    _check(_lib.mmaemu_mfma_probe_scaled(instr, _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(SA), _ptr(SB), k, batch, _stream(stream)))


def issue_probe_names():
    return [_lib.mmaemu_issue_probe_name(i).decode() for i in range(_lib.mmaemu_issue_probe_count())]


def issue_probe(op, iterations, workgroups, out, stream=None):
    _check(_lib.mmaemu_issue_probe(op, iterations, workgroups, _ptr(out), _stream(stream)))


def err_stats_reset(dev_err, stream=None):
    _check(_lib.mmaemu_err_stats_reset(_ptr(dev_err), _stream(stream)))


def exact_dot_sample(A, B, D, m, n, k, dtypes, stride, dev_err, stream=None):
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    _check(_lib.mmaemu_exact_dot_sample(_ptr(A), _ptr(B), _ptr(D), m, n, k, dt, stride, _ptr(dev_err), _stream(stream)))


def deviation_hist_reset(dev_hist, stream=None):
    _check(_lib.mmaemu_deviation_hist_reset(_ptr(dev_hist), _stream(stream)))


def deviation_sample(A, B, C, D, m, n, k, batch, dtypes, stride, bin_exp, dev_hist, stream=None):
    dt = dtypes if isinstance(dtypes, Dtypes) else Dtypes(*dtypes)
    _check(_lib.mmaemu_deviation_sample(_ptr(A), _ptr(B), _ptr(C) if C is not None else None, _ptr(D), m, n, k, batch, dt, stride,
                                        bin_exp, _ptr(dev_hist), _stream(stream)))


# ---- unpacking of the device-side result structs (host copies; no arithmetic) -----------

def _unpack(struct_type, dev_tensor):
    raw = bytes(dev_tensor.cpu().numpy().tobytes())
    st = struct_type.from_buffer_copy(raw[:ctypes.sizeof(struct_type)])
    out = {}
    for name, typ in struct_type._fields_:
        v = getattr(st, name)
        out[name] = list(v) if hasattr(v, "__len__") else v
    return out


def read_stats(dev_stats):
    """Synchronising copy of a device mmaemu_stats (a uint8 tensor of STATS_BYTES) to a dict."""
    return _unpack(Stats, dev_stats)


def read_stats_array(dev_stats, count):
    """The same for an array of `count` structs (a uint8 tensor of count * STATS_BYTES): a list of dicts."""
    flat = dev_stats.reshape(-1)
    return [_unpack(Stats, flat[i * STATS_BYTES:(i + 1) * STATS_BYTES]) for i in range(count)]


def read_err_stats(dev_err):
    return _unpack(ErrStats, dev_err)


def read_deviation_hist(dev_hist):
    return _unpack(DeviationHist, dev_hist)
