"""Exact dot products and error statistics of an emulated D against them.
Test infrastructure: see oracle/__init__.py.

Methodology after the paper's accuracy study (Sec. 6.2.4: deviation
delta = D_model - D_real of a model's output from the real result), with the real
result taken as the exact rational c + sum_k a_k b_k rather than an FP64 product.

Sampling rule (this library's definition): flattened output index i*n + j is sampled
when it is a multiple of `stride`.

Per sample, with R = RNE-FP32(exact):
  integer part : n_samples; n_equal_rne (D bits == R bits); n_above / n_below
                 (ordered key of D greater / less than that of R);
                 ulp_hist[34] of |key(D) - key(R)| bucketed as in oracle/stats.py
  float64 part : sum and max of |D - exact|, sum and max of |D - exact| / |exact|
                 (samples with exact == 0 skipped for the relative figures),
                 sum of (D - exact)
"""
from fractions import Fraction

import numpy as np

from . import formats as fm
from .rounding import rne_fp32
from .stats import ordered_key, N_BUCKETS


def exact_dot(a_bits, b_bits, ta, tb, c_bits=0):
    v = fm.decode(c_bits, fm.FP32).value
    for x, y in zip(a_bits, b_bits):
        v += fm.decode(int(x), ta).value * fm.decode(int(y), tb).value
    return v


def fp32_value(bits):
    d = fm.decode(bits, fm.FP32)
    assert d.finite
    return d.value


def empty_err_stats():
    return dict(n_samples=0, n_equal_rne=0, n_above=0, n_below=0, ulp_hist=[0] * N_BUCKETS,
                sum_abs_err=0.0, max_abs_err=0.0, sum_rel_err=0.0, max_rel_err=0.0, sum_signed_err=0.0)


def sample_indices(m, n, stride):
    return range(0, m * n, stride)


def error_stats(A, B, D, ta, tb, stride, stats=None, indices=None):
    """A[m][k], B[n][k] raw bits, D[m][n] FP32 bits (C is zero)."""
    st = empty_err_stats() if stats is None else stats
    A = np.asarray(A); B = np.asarray(B); D = np.asarray(D, dtype=np.uint32)
    m, n = D.shape
    sums = dict(abs=Fraction(0), rel=Fraction(0), sgn=Fraction(0))
    for idx in (sample_indices(m, n, stride) if indices is None else indices):
        i, j = divmod(idx, n)
        ex = exact_dot(A[i].tolist(), B[j].tolist(), ta, tb)
        r = rne_fp32(ex)
        dbits = int(D[i, j])
        st["n_samples"] += 1
        kd, kr = int(ordered_key(dbits)), int(ordered_key(r))
        if dbits == r:
            st["n_equal_rne"] += 1
        if kd > kr:
            st["n_above"] += 1
        elif kd < kr:
            st["n_below"] += 1
        st["ulp_hist"][abs(kd - kr).bit_length()] += 1
        err = fp32_value(dbits) - ex
        sums["abs"] += abs(err)
        sums["sgn"] += err
        st["max_abs_err"] = max(st["max_abs_err"], float(abs(err)))
        if ex != 0:
            rel = abs(err) / abs(ex)
            sums["rel"] += rel
            st["max_rel_err"] = max(st["max_rel_err"], float(rel))
    st["sum_abs_err"] += float(sums["abs"])
    st["sum_rel_err"] += float(sums["rel"])
    st["sum_signed_err"] += float(sums["sgn"])
    return st


DEVIATION_BINS = 64


def empty_deviation_hist():
    return dict(n_samples=0, n_skipped=0, n_negative=0, n_zero=0, n_positive=0, bins=[0] * DEVIATION_BINS,
                sum=0.0, sum_abs=0.0, sum_sq=0.0)


def deviation_hist(A, B, C, D, ta, tb, stride, bin_exp, hist=None):
    """Sec. 6.2.4: distribution of delta = D - D_real over sampled outputs, D_real = c + sum_k a_k b_k as an exact
    rational.  A[batch][m][k], B[batch][n][k], C (None: zero) and D[batch][m][n] FP32 bits; the flattened index over
    the whole batch is sampled when it is a multiple of `stride`.  Bin i holds delta in [(i - 32) w, (i - 31) w),
    w = 2^bin_exp; the outermost bins take everything beyond.  Samples with a NaN or an infinity anywhere are skipped."""
    h = empty_deviation_hist() if hist is None else hist
    A = np.asarray(A); B = np.asarray(B); D = np.asarray(D, dtype=np.uint32)
    nb, m, n = D.shape
    w = Fraction(2) ** bin_exp
    s1 = s2 = s3 = Fraction(0)
    for idx in range(0, nb * m * n, stride):
        t, rem = divmod(idx, m * n)
        i, j = divmod(rem, n)
        da = [fm.decode(int(x), ta) for x in A[t, i].tolist()]
        db = [fm.decode(int(x), tb) for x in B[t, j].tolist()]
        dc = fm.decode(int(C[t, i, j]) if C is not None else 0, fm.FP32)
        dd = fm.decode(int(D[t, i, j]), fm.FP32)
        if not (all(x.finite for x in da) and all(x.finite for x in db) and dc.finite and dd.finite):
            h["n_skipped"] += 1
            continue
        real = dc.value + sum((x.value * y.value for x, y in zip(da, db)), Fraction(0))
        delta = dd.value - real
        h["n_samples"] += 1
        h["n_negative" if delta < 0 else ("n_zero" if delta == 0 else "n_positive")] += 1
        q = delta / w
        fi = q.numerator // q.denominator                       # floor
        h["bins"][min(max(fi + DEVIATION_BINS // 2, 0), DEVIATION_BINS - 1)] += 1
        s1 += delta
        s2 += abs(delta)
        s3 += delta * delta
    h["sum"] += float(s1)
    h["sum_abs"] += float(s2)
    h["sum_sq"] += float(s3)
    return h
