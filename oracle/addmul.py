"""The model built from binary flush-to-zero operations.  Test infrastructure: see oracle/__init__.py.

Follows the paper's Sec. 4.1.1:
  * Algorithm "FTZ-Add and FTZ-Mul": z = RNE-FP32(x + y) or RNE-FP32(x * y) (as if to infinite precision, rounded
    once); then |z| < 2^-126 becomes zero with z's sign.
  * Algorithm "Phi_FTZ-AddMul": subnormal A, B, C inputs are replaced by +0.0; d <- c; for every P consecutive
    products (P in {2, 4}): p_l = FTZ-Mul(a_l, b_l); s = FTZ-Add(p_0, p_1); for P = 4 also s' = FTZ-Add(p_2, p_3),
    s = FTZ-Add(s, s'); d <- FTZ-Add(d, s).
  * Sec. 4.2: NaN + x = NaN, NaN * x = NaN, inf - inf = NaN, inf * 0 = NaN, otherwise infinities propagate with
    the usual signs.

Values are exact rationals (or the tags "nan", "+inf", "-inf"), one operation per function, each rounded by
oracle.rounding.  Readings: the sign of an exact zero sum is that of IEEE-754 round-to-nearest (+0 unless both
addends are -0); a product's zero carries the XOR of the signs; every NaN result is the model's nan_bits; K must
be a multiple of P.
"""
from fractions import Fraction

from . import formats as fm
from .rounding import to_fp32, RNE

NAN, PINF, NINF = "nan", "+inf", "-inf"


def _val(bits, t):
    """FP bits -> exact value: Fraction, or a tag; zeros keep their sign as (Fraction(0), sign)."""
    d = fm.decode(bits, t)
    if d.cls == fm.NAN:
        return NAN
    if d.cls == fm.INF:
        return NINF if d.sign else PINF
    return (d.value, d.sign)


def _from_fp32(bits):
    return _val(bits, fm.FP32)


def _round_flush(exact, sign_if_zero):
    """RNE-FP32 of a rational (sign_if_zero tells the sign of an exact zero), then the flush; returns FP32 bits."""
    if exact == 0:
        return sign_if_zero << 31
    z = to_fp32(exact, RNE)
    if (z & 0x7F800000) == 0:            # |z| < 2^-126 after rounding: zero of the same sign
        z &= 0x80000000
    return z


def ftz_mul(x_bits, tx, y_bits, ty, nan_bits):
    x, y = _val(x_bits, tx), _val(y_bits, ty)
    if x == NAN or y == NAN:
        return nan_bits
    xinf, yinf = x in (PINF, NINF), y in (PINF, NINF)
    sx = (x == NINF) if xinf else x[1]
    sy = (y == NINF) if yinf else y[1]
    if xinf or yinf:
        if (not xinf and x[0] == 0) or (not yinf and y[0] == 0):
            return nan_bits                                   # inf * 0
        return 0xFF800000 if (sx ^ sy) else 0x7F800000
    return _round_flush(x[0] * y[0], int(sx) ^ int(sy))


def ftz_add(x_bits, y_bits, nan_bits):
    x, y = _from_fp32(x_bits), _from_fp32(y_bits)
    if x == NAN or y == NAN:
        return nan_bits
    if x in (PINF, NINF) or y in (PINF, NINF):
        if x in (PINF, NINF) and y in (PINF, NINF) and x != y:
            return nan_bits                                   # inf - inf
        inf = x if x in (PINF, NINF) else y
        return 0xFF800000 if inf == NINF else 0x7F800000
    total = x[0] + y[0]
    if total == 0:
        both_zero = x[0] == 0 and y[0] == 0
        return _round_flush(Fraction(0), int(both_zero and x[1] and y[1]))   # -0 only for (-0) + (-0)
    return _round_flush(total, 0)


def emulate_element(P, a_bits, b_bits, c_bits, ta, tb, nan_bits=0x7FC00000):
    """Algorithm "Phi_FTZ-AddMul" for one output element."""
    K = len(a_bits)
    if P not in (2, 4):
        raise ValueError("P must be 2 or 4")
    if K % P:
        raise ValueError("K=%d is not a multiple of P=%d" % (K, P))
    a = [fm.flush_subnormal(int(x), ta) for x in a_bits]
    b = [fm.flush_subnormal(int(x), tb) for x in b_bits]
    d = fm.flush_subnormal(int(c_bits), fm.FP32)
    for k in range(0, K, P):
        p = [ftz_mul(a[k + l], ta, b[k + l], tb, nan_bits) for l in range(P)]
        s = ftz_add(p[0], p[1], nan_bits)
        if P == 4:
            s2 = ftz_add(p[2], p[3], nan_bits)
            s = ftz_add(s, s2, nan_bits)
        d = ftz_add(d, s, nan_bits)
    return d
