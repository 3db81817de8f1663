"""ctypes loader for oracle/o2/oracle2.c.  Test infrastructure: see oracle/__init__.py."""
import ctypes
import os
import subprocess

import numpy as np

from . import formats as fm

_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "o2")
_SO = os.path.join(_DIR, "liboracle2.so")
_lib = None


def build(force=False):
    src = os.path.join(_DIR, "oracle2.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _SO, src, "-lm"])
    return _SO


class O2Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("group_len", "frac_bits", "align_round", "c_mode", "out_round", "ftz_in", "ftz_out", "nan_bits", "frac_bits2", "split", "acc_special_truncation",
                 "frac_bits_merge", "frac_bits_acc", "skip_zero_terms", "f2_at_leading_bit", "zero_result_positive",
                 "sum_drop_distance", "family", "out_mant_bits", "wide_products", "acc_fp16", "nan_propagate", "rd_toward_zero")]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
    return _lib


def _params(p, tc=fm.FP32):
    return O2Params(p.group_len, p.frac_bits, p.align_round, p.c_mode, p.out_round,
                    int(p.ftz_in), int(p.ftz_out), p.nan_bits, p.frac_bits2, p.split, int(p.acc_special_truncation),
                    p.frac_bits_merge, p.frac_bits_acc, int(p.skip_zero_terms), int(p.f2_at_leading_bit),
                    int(p.zero_result_positive), p.sum_drop_distance, p.family, p.out_mant_bits, int(p.wide_products),
                    1 if tc == fm.FP16 else 0, int(p.nan_propagate), int(p.rd_toward_zero))


_NP = {fm.E4M3: np.uint8, fm.E5M2: np.uint8, fm.FP16: np.uint16, fm.BF16: np.uint16, fm.FP32: np.uint32,
       fm.E2M3: np.uint8, fm.E3M2: np.uint8, fm.E2M1: np.uint8, fm.TF32: np.uint32}


def _prep(A, B, C, ta, tb):
    A = np.ascontiguousarray(np.asarray(A).astype(_NP[ta], copy=False))
    B = np.ascontiguousarray(np.asarray(B).astype(_NP[tb], copy=False))
    C = np.ascontiguousarray(np.asarray(C).astype(np.uint32, copy=False))
    if A.ndim == 2:
        A, B, C = A[None], B[None], C[None]
    nb, m, k = A.shape
    n = B.shape[1]
    assert B.shape == (nb, n, k) and C.shape == (nb, m, n), (A.shape, B.shape, C.shape)
    return A, B, C, nb, m, n, k


def _vp(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def emulate_mma(p, A, B, C, ta, tb, nthreads=0, tc=fm.FP32):
    """Same contract as oracle.fdpa.emulate_mma (tc = FP16: C and D hold binary16 patterns); returns (D, threads_used)."""
    A, B, C, nb, m, n, k = _prep(A, B, C, ta, tb)
    D = np.empty((nb, m, n), dtype=np.uint32)
    used = ctypes.c_int(0)
    pp = _params(p, tc)
    rc = _load().o2_emulate_mma(ctypes.byref(pp), _vp(A), _vp(B), _vp(C), _vp(D),
                                ctypes.c_uint32(m), ctypes.c_uint32(n), ctypes.c_uint32(k),
                                ctypes.c_uint64(nb), ta, tb, nthreads, ctypes.byref(used))
    if rc:
        raise ValueError("o2_emulate_mma failed: %d" % rc)
    return D, used.value


def emulate_mma_scaled(p, A, B, C, SA, SB, block, ta, tb, nthreads=0, tc=fm.FP32):
    """Algorithm "ST-FDPA": as emulate_mma with E8M0 block scales SA[batch][m][k/block], SB[batch][n][k/block]."""
    A, B, C, nb, m, n, k = _prep(A, B, C, ta, tb)
    SA = np.ascontiguousarray(np.asarray(SA).astype(np.uint8, copy=False)).reshape(nb, m, k // block)
    SB = np.ascontiguousarray(np.asarray(SB).astype(np.uint8, copy=False)).reshape(nb, n, k // block)
    D = np.empty((nb, m, n), dtype=np.uint32)
    used = ctypes.c_int(0)
    pp = _params(p, tc)
    rc = _load().o2_emulate_mma_scaled(ctypes.byref(pp), _vp(A), _vp(B), _vp(C), _vp(D), _vp(SA), _vp(SB), ctypes.c_uint32(block),
                                       ctypes.c_uint32(m), ctypes.c_uint32(n), ctypes.c_uint32(k),
                                       ctypes.c_uint64(nb), ta, tb, nthreads, ctypes.byref(used))
    if rc:
        raise ValueError("o2_emulate_mma_scaled failed: %d" % rc)
    return D, used.value


def emulate_sample(p, A, B, C, idx, ta, tb, nthreads=0):
    """D at flattened indices idx (index = (b*m + i)*n + j)."""
    A, B, C, nb, m, n, k = _prep(A, B, C, ta, tb)
    idx = np.ascontiguousarray(idx, dtype=np.uint64)
    out = np.empty(idx.shape, dtype=np.uint32)
    used = ctypes.c_int(0)
    pp = _params(p)
    rc = _load().o2_emulate_sample(ctypes.byref(pp), _vp(A), _vp(B), _vp(C), _vp(idx),
                                   ctypes.c_uint64(idx.size), _vp(out),
                                   ctypes.c_uint32(m), ctypes.c_uint32(n), ctypes.c_uint32(k),
                                   ctypes.c_uint64(nb), ta, tb, nthreads, ctypes.byref(used))
    if rc:
        raise ValueError("o2_emulate_sample failed: %d" % rc)
    return out


def exact_dot_stats(A, B, D, ta, tb, stride):
    A = np.ascontiguousarray(np.asarray(A).astype(_NP[ta], copy=False))
    B = np.ascontiguousarray(np.asarray(B).astype(_NP[tb], copy=False))
    D = np.ascontiguousarray(D, dtype=np.uint32)
    m, k = A.shape
    n = B.shape[0]
    assert D.shape == (m, n)
    io = np.zeros(38, dtype=np.uint64)
    do = np.zeros(5, dtype=np.float64)
    rc = _load().o2_exact_dot_stats(_vp(A), _vp(B), _vp(D), ctypes.c_uint32(m), ctypes.c_uint32(n),
                                    ctypes.c_uint32(k), ta, tb, ctypes.c_uint64(stride), _vp(io), _vp(do))
    if rc:
        raise ValueError("o2_exact_dot_stats failed: %d" % rc)
    return dict(n_samples=int(io[0]), n_equal_rne=int(io[1]), n_above=int(io[2]), n_below=int(io[3]),
                ulp_hist=[int(x) for x in io[4:38]], sum_abs_err=float(do[0]), max_abs_err=float(do[1]),
                sum_rel_err=float(do[2]), max_rel_err=float(do[3]), sum_signed_err=float(do[4]))


class GstParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("L", "G", "k_block", "F", "out_round", "scale_format", "nan_bits")]


def emulate_gst(A, B, C, SA, SB, L, G, k_block, F, out_round, scale_format, nan_bits=0x7FFFFFFF, nthreads=0):
    """Algorithm "GST-FDPA" chained over K / L operations: FP4 codes A[batch][m][k], B[batch][n][k] (one per byte),
    scale codes SA[batch][m][k / k_block], SB[batch][n][k / k_block]; returns D as uint32 FP32 bits."""
    A = np.ascontiguousarray(np.asarray(A).astype(np.uint8, copy=False))
    B = np.ascontiguousarray(np.asarray(B).astype(np.uint8, copy=False))
    C = np.ascontiguousarray(np.asarray(C).astype(np.uint32, copy=False))
    if A.ndim == 2:
        A, B, C = A[None], B[None], C[None]
    nb, m, k = A.shape
    n = B.shape[1]
    SA = np.ascontiguousarray(np.asarray(SA).astype(np.uint8, copy=False)).reshape(nb, m, k // k_block)
    SB = np.ascontiguousarray(np.asarray(SB).astype(np.uint8, copy=False)).reshape(nb, n, k // k_block)
    D = np.empty((nb, m, n), dtype=np.uint32)
    g = GstParams(L, G, k_block, F, out_round, scale_format, nan_bits)
    rc = _load().o2_emulate_gst(ctypes.byref(g), _vp(A), _vp(B), _vp(C), _vp(D), _vp(SA), _vp(SB), ctypes.c_uint32(m), ctypes.c_uint32(n),
                                ctypes.c_uint32(k), ctypes.c_uint64(nb), nthreads)
    if rc:
        raise ValueError("o2_emulate_gst failed: %d" % rc)
    return D
