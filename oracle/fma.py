"""The model built from the standard fused multiply-add.  Test infrastructure: see oracle/__init__.py.

Follows the paper's Sec. 4.1.2:
  * Algorithm "FMA": d = F(a x b + c), the sum as if to infinite precision, rounded once to the format F to nearest,
    ties to even.  F is binary32 (fmt = FP32, the default) or binary64 (fmt = FP64), the two formats the algorithm
    names.
  * Algorithm "Phi_FMA": d <- c; for k = 0 .. K - 1 in order: d <- FMA(a_k, b_k, d).
  * Sec. 4.2: a NaN operand, infinity times zero and infinities of both signs give NaN; otherwise infinities
    propagate with the usual signs.

Values are exact rationals; one rounding per step by oracle.rounding.  Readings:
  * the paper calls the operation the one IEEE-754 defines, so what the algorithm's one line leaves open is taken from
    the standard: subnormal inputs and results are kept; overflow gives infinity; an exact zero result is +0.0 unless
    the product and the addend are zeros of the same sign, which keep it (round-to-nearest rule for sums of zeros; a
    zero product carries the XOR of its factors' signs);
  * every NaN result is the model's nan_bits; with nan_propagate the payload variation instead (per step, in this
    order: a NaN a made quiet; a NaN b made quiet; nan_bits for infinity times zero; a NaN addend made quiet; nan_bits
    for infinities of both signs), the same rule oracle.fdpa applies to a group of one product;
  * the model's NaN pattern is a binary32 word; for binary64 it is widened as a conversion between the two formats
    widens a NaN: sign kept, exponent field all ones, the 23 mantissa bits at the top of the 52.
"""
import numpy as np

from . import formats as fm
from .rounding import to_fp32, to_fp64, RNE

QUIET = 0x00400000


def widen_nan(nan_bits):
    """The binary64 pattern of a binary32 NaN pattern (see the head of this file)."""
    return ((nan_bits >> 31) << 63) | 0x7FF0000000000000 | ((nan_bits & 0x7FFFFF) << 29)


def fma(a_bits, b_bits, c_bits, nan_bits=0x7FC00000, nan_propagate=False, fmt=fm.FP32):
    """Algorithm "FMA" on binary32 (binary64) patterns; returns the pattern of the result."""
    if fmt == fm.FP64:
        return _fma64(int(a_bits), int(b_bits), int(c_bits), widen_nan(nan_bits), nan_propagate)
    a, b, c = fm.decode(a_bits, fm.FP32), fm.decode(b_bits, fm.FP32), fm.decode(c_bits, fm.FP32)
    invalid_product = (a.cls == fm.INF and b.cls == fm.ZERO) or (b.cls == fm.INF and a.cls == fm.ZERO)
    if nan_propagate:
        if a.cls == fm.NAN:
            return int(a_bits) | QUIET
        if b.cls == fm.NAN:
            return int(b_bits) | QUIET
        if invalid_product:
            return nan_bits
        if c.cls == fm.NAN:
            return int(c_bits) | QUIET
    elif fm.NAN in (a.cls, b.cls, c.cls) or invalid_product:
        return nan_bits
    psign = a.sign ^ b.sign
    if a.cls == fm.INF or b.cls == fm.INF:
        if c.cls == fm.INF and c.sign != psign:
            return nan_bits                                     # inf - inf
        return (psign << 31) | 0x7F800000
    if c.cls == fm.INF:
        return int(c_bits)
    product = a.value * b.value
    total = product + c.value
    if total == 0:
        if product == 0 and c.value == 0 and psign == c.sign:
            return psign << 31                                  # zeros of one sign keep it
        return 0                                                # every other exact zero is +0.0
    return to_fp32(total, RNE)


def _fma64(a_bits, b_bits, c_bits, nan64, nan_propagate):
    """The same steps on binary64 patterns (quiet bit 51)."""
    quiet = 1 << 51
    a, b, c = fm.decode(a_bits, fm.FP64), fm.decode(b_bits, fm.FP64), fm.decode(c_bits, fm.FP64)
    invalid_product = (a.cls == fm.INF and b.cls == fm.ZERO) or (b.cls == fm.INF and a.cls == fm.ZERO)
    if nan_propagate:
        if a.cls == fm.NAN:
            return a_bits | quiet
        if b.cls == fm.NAN:
            return b_bits | quiet
        if invalid_product:
            return nan64
        if c.cls == fm.NAN:
            return c_bits | quiet
    elif fm.NAN in (a.cls, b.cls, c.cls) or invalid_product:
        return nan64
    psign = a.sign ^ b.sign
    if a.cls == fm.INF or b.cls == fm.INF:
        if c.cls == fm.INF and c.sign != psign:
            return nan64
        return (psign << 63) | 0x7FF0000000000000
    if c.cls == fm.INF:
        return c_bits
    product = a.value * b.value
    total = product + c.value
    if total == 0:
        if product == 0 and c.value == 0 and psign == c.sign:
            return psign << 63
        return 0
    return to_fp64(total, RNE)


def emulate_element(a_bits, b_bits, c_bits, nan_bits=0x7FC00000, nan_propagate=False, fmt=fm.FP32):
    """Algorithm "Phi_FMA" for one output element: the chain over k."""
    d = int(c_bits)
    for x, y in zip(a_bits, b_bits):
        d = fma(int(x), int(y), d, nan_bits, nan_propagate, fmt)
    return d


def emulate_mma(A, B, C, nan_bits=0x7FC00000, nan_propagate=False, fmt=fm.FP32):
    """A[batch, m, k], B[batch, n, k] (row j of B is column j of the mathematical B), C[batch, m, n]: binary32 patterns
    (binary64 patterns in uint64 arrays for fmt = FP64)."""
    A, B, C = np.asarray(A), np.asarray(B), np.asarray(C)
    batch, m, k = A.shape
    n = B.shape[1]
    D = np.zeros((batch, m, n), dtype=np.uint64 if fmt == fm.FP64 else np.uint32)
    for t in range(batch):
        for i in range(m):
            row = A[t, i].tolist()
            for j in range(n):
                D[t, i, j] = emulate_element(row, B[t, j].tolist(), int(C[t, i, j]), nan_bits, nan_propagate, fmt)
    return D
