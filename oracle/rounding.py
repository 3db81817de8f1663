"""Conversion functions rho of the paper's Table "Conversion functions", on exact
rationals.  Test infrastructure: see oracle/__init__.py.

RNE-FP32: IEEE-754 round-to-nearest-even to binary32, gradual underflow,
          overflow to infinity.
RZ-FP32 : truncate the magnitude to the binary32 grid (gradual underflow);
          a magnitude beyond the largest finite value gives the largest finite
          value (IEEE-754 roundTowardZero; the paper is silent on overflow).

An exactly-zero value converts to +0.0 (the paper does not state the sign of an
exact-zero fused sum; this reading is fixed for the whole build).  A non-zero
value that rounds to zero keeps its sign.
"""
from fractions import Fraction

FP32_MBITS = 23
FP32_EMIN = -126
FP32_EMAX = 127
FP32_INF = 0x7F800000
FP32_MAXFINITE = 0x7F7FFFFF

RNE, RZ = 0, 1


def floor_log2(q):
    """floor(log2(q)) for a positive Fraction, exactly."""
    assert q > 0
    e = q.numerator.bit_length() - q.denominator.bit_length()
    # 2^(e-1) < q < 2^(e+1)
    if Fraction(2) ** e > q:
        e -= 1
    assert Fraction(2) ** e <= q < Fraction(2) ** (e + 1)
    return e


def to_fp32(v, mode):
    """Round the exact rational v to binary32 bits under `mode` (RNE or RZ)."""
    v = Fraction(v)
    if v == 0:
        return 0
    sign = 1 if v < 0 else 0
    a = -v if sign else v
    e = max(floor_log2(a), FP32_EMIN)          # exponent of the grid the value falls in
    quantum = Fraction(2) ** (e - FP32_MBITS)  # spacing of binary32 numbers there
    q = a / quantum
    n = q.numerator // q.denominator           # floor
    rem = q - n
    if mode == RNE:
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
            n += 1
    elif mode != RZ:
        raise ValueError(mode)
    # n is in [0, 2^24]; n == 2^24 means the rounding carried into the next binade
    if n == (1 << (FP32_MBITS + 1)):
        n >>= 1
        e += 1
    if e > FP32_EMAX:
        mag = FP32_INF if mode == RNE else FP32_MAXFINITE
    elif n < (1 << FP32_MBITS):
        assert e == FP32_EMIN                   # subnormal or zero
        mag = n
    else:
        mag = ((e + 127) << FP32_MBITS) | (n - (1 << FP32_MBITS))
    return (sign << 31) | mag


def to_fp16(v, mode):
    """Round the exact rational v to binary16 bits under `mode`: RNE-FP16 of the paper's table (RZ likewise, by
    analogy with RZ-FP32).  Same rules as to_fp32 on the binary16 grid: 10 mantissa bits, exponents -14 .. 15,
    gradual underflow, overflow to infinity (RNE) or to the largest finite value (RZ), exact zero -> +0.0."""
    v = Fraction(v)
    if v == 0:
        return 0
    sign = 1 if v < 0 else 0
    a = -v if sign else v
    e = max(floor_log2(a), -14)
    q = a / Fraction(2) ** (e - 10)
    n = q.numerator // q.denominator
    rem = q - n
    if mode == RNE:
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
            n += 1
    elif mode != RZ:
        raise ValueError(mode)
    if n == (1 << 11):
        n >>= 1
        e += 1
    if e > 15:
        mag = 0x7C00 if mode == RNE else 0x7BFF
    elif n < (1 << 10):
        assert e == -14
        mag = n
    else:
        mag = ((e + 15) << 10) | (n - (1 << 10))
    return (sign << 15) | mag


def to_fp64(v, mode):
    """Round the exact rational v to binary64 bits: the rules of to_fp32 on the binary64 grid (52 mantissa bits,
    exponents -1022 .. 1023, gradual underflow, overflow to infinity under RNE, exact zero -> +0.0)."""
    v = Fraction(v)
    if v == 0:
        return 0
    sign = 1 if v < 0 else 0
    a = -v if sign else v
    e = max(floor_log2(a), -1022)
    q = a / Fraction(2) ** (e - 52)
    n = q.numerator // q.denominator
    rem = q - n
    if mode == RNE:
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
            n += 1
    elif mode != RZ:
        raise ValueError(mode)
    if n == (1 << 53):
        n >>= 1
        e += 1
    if e > 1023:
        mag = 0x7FF0000000000000 if mode == RNE else 0x7FEFFFFFFFFFFFFF
    elif n < (1 << 52):
        assert e == -1022
        mag = n
    else:
        mag = ((e + 1023) << 52) | (n - (1 << 52))
    return (sign << 63) | mag


def rne_fp32(v):
    return to_fp32(v, RNE)


def rz_fp32(v):
    return to_fp32(v, RZ)
