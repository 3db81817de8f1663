"""Phi_FMA on binary64 (Algorithms "FMA" / "Phi_FMA" with F = FP64) and the binary64 plumbing of the oracle, pinned to
things outside it: the C library's fma() (an independent correctly rounded implementation, through ctypes), numpy's
binary64 arithmetic, Python's float <-> bits conversions, and the worked example of Sec. 5."""
import ctypes
import ctypes.util
import itertools
import struct
from fractions import Fraction

import numpy as np

from oracle import formats as fm, gen as ogen, stats as ostats
from oracle.fma import fma, emulate_element, emulate_mma, widen_nan
from oracle.rounding import to_fp64, RNE, RZ

libm = ctypes.CDLL(ctypes.util.find_library("m"))
libm.fma.restype = ctypes.c_double
libm.fma.argtypes = [ctypes.c_double] * 3


def bits(x):
    return struct.unpack("<Q", struct.pack("<d", x))[0]


def val(b):
    return struct.unpack("<d", struct.pack("<Q", b))[0]


def c_fma(a, b, c):
    return bits(libm.fma(val(a), val(b), val(c)))


CRITICAL = [0x0, 1 << 63, 1, (1 << 52) - 1, 1 << 52, bits(1.0), bits(-1.0), bits(1.5), bits(1.0 + 2.0 ** -52),
            0x7FEFFFFFFFFFFFFF, 0xFFEFFFFFFFFFFFFF, 0x7FF0000000000000, 0xFFF0000000000000, bits(2.0 ** -53), bits(-2.0 ** -53),
            bits(2.0 ** 511), bits(2.0 ** -537)]


def test_decode_and_rounder_against_python_floats():
    rng = np.random.default_rng(1)
    for b in list(rng.integers(0, 1 << 63, size=300, dtype=np.uint64)) + CRITICAL:
        b = int(b)
        d = fm.decode(b, fm.FP64)
        if d.finite:
            assert d.value == Fraction(val(b))                       # Fraction(float) is exact
            assert to_fp64(d.value, RNE) == (b if d.value != 0 else 0)   # representable values round to themselves
    # the rounder on values that are not representable: against Python's correctly rounded int / int division
    for _ in range(300):
        n, dn = int(rng.integers(1, 1 << 62)), int(rng.integers(1, 1 << 62))
        e = int(rng.integers(-1100, 1000))
        v = Fraction(n, dn) * Fraction(2) ** e
        want = (n / dn) * 2.0 ** e if -1000 < e < 900 else None     # (scaling by a power of two is exact away from the ends)
        if want is not None:
            assert to_fp64(v, RNE) == bits(want)
    assert to_fp64(Fraction(2) ** 1024, RNE) == 0x7FF0000000000000 and to_fp64(Fraction(2) ** 1024, RZ) == 0x7FEFFFFFFFFFFFFF
    assert to_fp64(Fraction(1, 2) * Fraction(2) ** -1074, RNE) == 0 and to_fp64(Fraction(3, 2) * Fraction(2) ** -1074, RNE) == 2   # ties to even
    assert to_fp64(-Fraction(2) ** -1074, RNE) == (1 << 63) | 1


def test_one_step_against_libm_on_critical_triples():
    for a, b, c in itertools.product(CRITICAL, repeat=3):
        want = c_fma(a, b, c)
        got = fma(a, b, c, fmt=fm.FP64)
        if (want & 0x7FFFFFFFFFFFFFFF) > 0x7FF0000000000000:
            assert got == 0x7FF8000000000000, (hex(a), hex(b), hex(c))
        else:
            assert got == want, (hex(a), hex(b), hex(c), hex(got), hex(want))


def test_chains_against_libm():
    rng = np.random.default_rng(2)
    for family in range(4):
        for _ in range(60):
            k = 8
            if family == 0:      # ordinary values
                a = rng.standard_normal(k); b = rng.standard_normal(k); c = rng.standard_normal()
            elif family == 1:    # c ~ -a0 b0: the low product bits decide
                a = rng.standard_normal(k); b = rng.standard_normal(k); c = -(a[0] * b[0])
            elif family == 2:    # around the bottom of the range
                a = rng.standard_normal(k) * 2.0 ** -520; b = rng.standard_normal(k) * 2.0 ** -520; c = rng.standard_normal() * 2.0 ** -1060
            else:                # all finite bit patterns (overflow and underflow everywhere)
                a = np.array([val(int(x)) for x in rng.integers(0, 0x7FF0000000000000, size=k, dtype=np.uint64)])
                b = np.array([val(int(x)) for x in rng.integers(0, 0x7FF0000000000000, size=k, dtype=np.uint64)]) * rng.choice([-1.0, 1.0], size=k)
                c = float(rng.standard_normal())
            ab, bb = [bits(float(x)) for x in a], [bits(float(x)) for x in b]
            want = bits(float(c))
            for x, y in zip(ab, bb):
                want = c_fma(x, y, want)
                if (want & 0x7FFFFFFFFFFFFFFF) > 0x7FF0000000000000:
                    want = 0x7FF8000000000000
            assert emulate_element(ab, bb, bits(float(c)), fmt=fm.FP64) == want


def test_worked_example_and_nan_rules():
    # Sec. 5: every FP64 / FP32 instruction gives -0.875 on the worked example
    a = [-2.0 ** 13, -0.5, -0.25, -0.125]
    b = [2.0 ** 10, 1.0, 1.0, 1.0]
    assert emulate_element([bits(x) for x in a], [bits(x) for x in b], bits(2.0 ** 23), fmt=fm.FP64) == bits(-0.875)
    assert widen_nan(0x7FC00000) == 0x7FF8000000000000 and widen_nan(0xFFC00000) == 0xFFF8000000000000
    assert widen_nan(0x7FFFFFFF) == 0x7FFFFFFFE0000000
    assert val(widen_nan(0x7FC00001)) != val(widen_nan(0x7FC00001))          # still a NaN
    assert struct.unpack("<d", struct.pack("<d", struct.unpack("<f", struct.pack("<I", 0x7FC12345))[0]))[0] != 0    # (python widens NaNs too)
    assert bits(struct.unpack("<f", struct.pack("<I", 0x7FC12345))[0]) == widen_nan(0x7FC12345)   # the C conversion keeps the payload at the top
    one, inf, nan_p, zero = bits(1.0), 0x7FF0000000000000, 0x7FF0000000012345, 0
    assert fma(nan_p, one, one, nan_bits=0xFFC00000, fmt=fm.FP64) == 0xFFF8000000000000
    assert fma(nan_p, one, one, nan_propagate=True, fmt=fm.FP64) == nan_p | (1 << 51)
    assert fma(one, nan_p, one, nan_propagate=True, fmt=fm.FP64) == nan_p | (1 << 51)
    assert fma(inf, zero, nan_p, nan_propagate=True, fmt=fm.FP64) == 0x7FF8000000000000      # the invalid product goes first
    assert fma(one, one, nan_p, nan_propagate=True, fmt=fm.FP64) == nan_p | (1 << 51)
    assert fma(inf, one, inf | (1 << 63), fmt=fm.FP64) == 0x7FF8000000000000
    assert fma(inf, bits(-1.0), one, fmt=fm.FP64) == inf | (1 << 63)
    # signs of exact zeros
    mz = 1 << 63
    assert fma(mz, one, mz, fmt=fm.FP64) == mz and fma(zero, bits(-1.0), mz, fmt=fm.FP64) == mz
    assert fma(zero, one, mz, fmt=fm.FP64) == 0 and fma(one, one, bits(-1.0), fmt=fm.FP64) == 0


def test_matrix_form_is_the_chain_per_element():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((2, 3, 5)).view(np.uint64); B = rng.standard_normal((2, 4, 5)).view(np.uint64)
    C = rng.standard_normal((2, 3, 4)).view(np.uint64)
    D = emulate_mma(A, B, C, fmt=fm.FP64)
    d = C.view(np.float64)[1, 2, 3]
    for kk in range(5):
        d = libm.fma(A.view(np.float64)[1, 2, kk], B.view(np.float64)[1, 3, kk], d)
    assert D.dtype == np.uint64 and int(D[1, 2, 3]) == bits(d)


def test_binary64_generators():
    gp = lambda fam, **kw: ogen.GenParams(family=fam, seed=5, operand=1, **kw)
    # value family: the binary64 value itself; rounding it to binary32 gives the FP32 stream of the same call
    z = ogen.generate(gp(ogen.GEN_NORMAL), fm.FP64, 64, 2, 50)
    f = ogen.generate(gp(ogen.GEN_NORMAL), fm.FP32, 64, 2, 50)
    assert z.dtype == np.uint64 and np.array_equal(z.view(np.float64).astype(np.float32).view(np.uint32), f)
    zs = ogen.generate(gp(ogen.GEN_NORMAL, scale_scope=ogen.SCALE_FACTOR, scale_target=1000.0), fm.FP64, 64, 2, 50)
    assert np.array_equal(zs.view(np.float64), z.view(np.float64) * 1000.0)
    v = z.view(np.float64)
    assert abs(v.mean()) < 0.1 and 0.9 < v.std() < 1.1
    # bit families
    r = ogen.generate(gp(ogen.GEN_RANDOM_BITS), fm.FP64, 256, 0, 64)
    ones = np.unpackbits(r.view(np.uint8)).mean()
    assert 0.49 < ones < 0.51
    fb = ogen.generate(gp(ogen.GEN_FINITE_BITS), fm.FP64, 256, 0, 64)
    E = (fb >> np.uint64(52)) & np.uint64(0x7FF)
    assert E.max() <= 2046 and E.min() <= 5 and E.max() >= 2040 and 0.45 < (fb >> np.uint64(63)).mean() < 0.55
    # the arithmetic of FINITE_BITS against Python integers
    from oracle.gen import _words
    g = np.arange(0, 8, dtype=np.uint64)
    lo, hi = _words(5, 1, g * np.uint64(2)), _words(5, 1, g * np.uint64(2) + np.uint64(1))
    for i in range(8):
        v = (((int(hi[i]) << 32) | int(lo[i])) * (2 * (2047 << 52))) >> 64
        want = v if v < (2047 << 52) else (1 << 63) | (v - (2047 << 52))
        assert int(fb.ravel()[i]) == want
    ue = ogen.generate(gp(ogen.GEN_UNIFORM_EXP, exp_lo=1000, exp_hi=1040, exp_zero=True), fm.FP64, 256, 0, 64)
    E = (ue >> np.uint64(52)) & np.uint64(0x7FF)
    assert set(np.unique(E).tolist()) == {0} | set(range(1000, 1041))
    assert np.all((ue[E == 0] & np.uint64(0x7FFFFFFFFFFFFFFF)) < np.uint64(1 << 52))
    sz = ogen.generate(gp(ogen.GEN_SIGNED_ZEROS), fm.FP64, 256, 0, 16)
    assert set(np.unique(sz).tolist()) == {0, 1 << 63, 1, (1 << 63) | 1, bits(1.0), bits(-1.0)}
    # any chunk independently
    whole = ogen.generate(gp(ogen.GEN_FINITE_BITS), fm.FP64, 10, 0, 7)
    assert np.array_equal(whole[3:5], ogen.generate(gp(ogen.GEN_FINITE_BITS), fm.FP64, 10, 3, 2))


def test_compare_on_64_bit_patterns():
    x = np.array([0, 1, (1 << 63) | 1, 0x7FF0000000000000, 0x7FF8000000000000, 0x7FF8000000000001, bits(1.0), 5], dtype=np.uint64)
    y = np.array([1 << 63, 3, 1, 0xFFF0000000000000, 0, 0x7FF8000000000000, bits(1.0), 5 + (1 << 40)], dtype=np.uint64)
    st = ostats.compare(x, y, width=64, index_base=100)
    assert st["n_compared"] == 8 and st["n_mismatch_bits"] == 7 and st["n_mismatch_nan_equiv"] == 1
    assert st["first_mismatch_index"] == 100
    h = st["ulp_hist"]
    # +0 / -0: bucket 0; 1 vs 3: distance 2 -> bucket 2; -1ulp vs +1ulp: distance 2; +inf vs -inf and 2^40: bucket 32;
    # NaN vs number: 33; NaN vs NaN: 0; equal: 0
    assert h[0] == 3 and h[2] == 2 and h[32] == 2 and h[33] == 1 and sum(h) == 8
    assert st["max_ulp_dist"] == 2 * 0x7FF0000000000000
