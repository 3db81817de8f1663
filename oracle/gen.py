"""Synthetic tile generators (CPU twins of the on-device generators).
Test infrastructure: see oracle/__init__.py.

The paper's randomized validation (Sec. 3.1, Step 4) draws inputs from common
distributions and from random bit streams; it fixes no generator.  This file is
this library's definition, stated so that an integer-exact twin can exist on the
device:

Random words.  Element with global index g = (first_tile + t) * elems_per_tile + e
of operand `operand` (0 = A, 1 = B, 2 = C) owns `wpe` consecutive words starting at
word index w = g * wpe of the stream
    word(w) = Philox4x32-10(counter = (lo32(w >> 2), hi32(w >> 2), operand, 0),
                            key = (lo32(seed), hi32(seed)))[w & 3].
wpe is 2 for FP32 output of the UNIFORM_EXP family and 1 otherwise.

Families (r = first word, r1 = second word):
  ZERO          all bits zero.
  FINITE_BITS   uniform over all finite bit patterns: v = (r * ncodes) >> 32 with
                ncodes = 2 * nmag (nmag = number of finite magnitudes of the format);
                sign = v >= nmag; magnitude code = v - sign * nmag.
  UNIFORM_EXP   sign = r >> 31; exponent field uniform over `exp_lo..exp_hi`
                (plus the value 0 as one extra, equally likely, choice when
                `exp_zero`), drawn as idx = (sel * nchoices) >> nsel with
                sel = bits m..30 of r (nsel = 31 - m) -- for FP32: sel = r & 0x7FFFFFFF,
                nsel = 31 and the mantissa comes from r1; mantissa = low m bits.
  RANDOM_BITS   the low `width` bits of r (NaN and infinities included).
  SIGNED_ZEROS  one of eight equally likely values picked by the top three bits of r: sign = bit 29, magnitude by
                bits 31..30: 0 and 1 -> zero, 2 -> 1.0 (exponent field = bias, mantissa 0), 3 -> the smallest
                subnormal (code 1).  Exact zeros of both signs next to the values that produce them.
  NORMAL        Box-Muller on word pairs (elements 2i, 2i+1 of the flattened
                operand share (r_2i, r_2i+1)):  u1 = (r_2i + 0.5) / 2^32,
                phi = 2 pi r_2i+1 / 2^32 (+ half a step), radius = sqrt(-2 ln u1);
                element 2i gets radius*cos(phi), element 2i+1 radius*sin(phi).
                ln, sin and cos are evaluated in binary64 with +, *, / only
                (series below, fixed operation order, no fused multiply-add), and the
                square root is IEEE-754's own correctly rounded operation, so
                that any IEEE-754 machine produces the same bits.  The value is
                optionally multiplied by scale_target / absmax (absmax over the
                whole call, or over each tile), rounded to binary32 (RNE), then to
                the output format (RNE, saturating at the largest finite value).
  UNIFORM       uniform on [-1, 1): (r + 0.5) * 2^-31 - 1 (exact in binary64); scaling and casts as NORMAL.
  NORMAL_OUTLIERS  the DNN-like family of Sec. 3.1 Step 4, N(0,1) + Bernoulli(0.001) * N(0,100), with the
                variance 100 read as standard deviation 10: z + h * 10 * z', z as NORMAL, z' the same
                construction on word stream `operand + 256`, h = 1 where the word of stream
                `operand + 512` is below floor(0.001 * 2^32) = 4294967.  Scaling and casts as NORMAL.
  CANCELLING    adversarial sums with large condition numbers (Sec. 3.1 Step 4): an element of even index
                is drawn as UNIFORM_EXP; the odd element after it repeats that draw -- with the sign
                flipped for operand 0, and for the other operands with the last mantissa bit flipped
                where the low 4 bits of the odd element's own word are zero.  Not defined for FP32.
"""
import math
from dataclasses import dataclass

import numpy as np

from . import formats as fm
from .philox import philox4x32_10

GEN_ZERO, GEN_FINITE_BITS, GEN_UNIFORM_EXP, GEN_RANDOM_BITS, GEN_NORMAL = 0, 1, 2, 3, 4
GEN_UNIFORM, GEN_NORMAL_OUTLIERS, GEN_CANCELLING, GEN_SIGNED_ZEROS = 5, 6, 7, 8
VALUE_FAMILIES = (GEN_NORMAL, GEN_UNIFORM, GEN_NORMAL_OUTLIERS)
SCALE_NONE, SCALE_TENSOR, SCALE_TILE, SCALE_FACTOR = 0, 1, 2, 3


@dataclass(frozen=True)
class GenParams:
    family: int
    seed: int = 0
    operand: int = 0
    exp_lo: int = 0
    exp_hi: int = 0
    exp_zero: bool = False
    scale_scope: int = SCALE_NONE
    scale_target: float = 1.0


def _words(seed, operand, w):
    """word(w) for an array of word indices."""
    w = np.asarray(w, dtype=np.uint64)
    blk = w >> np.uint64(2)
    out = philox4x32_10(blk & np.uint64(0xFFFFFFFF), blk >> np.uint64(32), operand, 0,
                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    lane = (w & np.uint64(3)).astype(np.int64)
    return np.choose(lane, out)


def _n_finite_magnitudes(f):
    if f.no_specials:
        return (f.emax_field + 1) << f.mbits
    return (f.emax_field << f.mbits) if f.ieee_specials else ((f.emax_field + 1) << f.mbits) - 1


def max_finite_code(f):
    return _n_finite_magnitudes(f) - 1


def cast_from_fp32(bits32, fmt_id):
    """RNE conversion of finite binary32 bit patterns to `fmt_id`, saturating at the
    largest finite magnitude.  Integer arithmetic only."""
    f = fm.FORMATS[fmt_id]
    b = np.asarray(bits32, dtype=np.uint32).astype(np.uint64)
    if fmt_id == fm.FP32:
        return b.astype(np.uint32)
    sign = b >> np.uint64(31)
    E32 = (b >> np.uint64(23)) & np.uint64(0xFF)
    sig = (b & np.uint64(0x7FFFFF)) | np.where(E32 > 0, np.uint64(1 << 23), np.uint64(0))
    exp = np.maximum(E32, 1).astype(np.int64) - 127              # value = sig * 2^(exp-23)
    q = np.maximum(exp, 1 - f.bias) - f.mbits                    # exponent of the target's last place
    shift = np.minimum(q - (exp - 23), 40).astype(np.uint64)     # >= 23 - m > 0
    n = sig >> shift
    rem = sig & ((np.uint64(1) << shift) - np.uint64(1))
    half = np.uint64(1) << (shift - np.uint64(1))
    n = n + ((rem > half) | ((rem == half) & ((n & np.uint64(1)) == 1))).astype(np.uint64)
    Et = np.maximum(exp + f.bias, 1).astype(np.uint64)
    code = ((Et - np.uint64(1)) << np.uint64(f.mbits)) + n
    code = np.minimum(code, np.uint64(max_finite_code(f)))
    return ((sign << np.uint64(f.width - 1)) | code).astype(np.uint32)


# ---- binary64 elementary functions from +, *, / only (fixed order) -------------------

LN2 = float.fromhex("0x1.62e42fefa39efp-1")
HALF_PI = float.fromhex("0x1.921fb54442d18p+0")
LOG_TERMS = 12     # ln m = 2 s (1 + s^2/3 + ... + s^(2*12)/(2*12+1)),  s = (m-1)/(m+1)
SIN_TERMS = 10     # through theta^19
COS_TERMS = 11     # through theta^20


def _ln_unit(r):
    """ln((r + 0.5) / 2^32) for uint32 r."""
    t = 2.0 * r.astype(np.float64) + 1.0                  # odd integer < 2^33, exact
    mant, ex = np.frexp(t)                                # t = mant * 2^ex, mant in [0.5, 1)
    m = mant * 2.0                                        # [1, 2)
    s = (m - 1.0) / (m + 1.0)
    s2 = s * s
    poly = np.full_like(s, 1.0 / (2 * LOG_TERMS + 1))
    for n in range(LOG_TERMS - 1, 0, -1):
        poly = poly * s2 + 1.0 / (2 * n + 1)
    poly = poly * s2 + 1.0
    lnm = (2.0 * s) * poly
    return lnm + (ex - 1 - 33).astype(np.float64) * LN2


def _sqrt(x):
    return np.sqrt(x)                                     # correctly rounded (IEEE-754 squareRoot)


def _sincos_quarter(theta):
    t2 = theta * theta
    ps = np.full_like(theta, (-1.0) ** (SIN_TERMS - 1) / math.factorial(2 * SIN_TERMS - 1))
    for n in range(SIN_TERMS - 2, -1, -1):
        ps = ps * t2 + (-1.0) ** n / math.factorial(2 * n + 1)
    pc = np.full_like(theta, (-1.0) ** (COS_TERMS - 1) / math.factorial(2 * COS_TERMS - 2))
    for n in range(COS_TERMS - 2, -1, -1):
        pc = pc * t2 + (-1.0) ** n / math.factorial(2 * n)
    return theta * ps, pc


def normal_pairs(r_even, r_odd):
    """Box-Muller: two uint32 arrays -> (z_even, z_odd) binary64."""
    radius = _sqrt(-2.0 * _ln_unit(r_even))
    quad = (r_odd >> np.uint32(30)).astype(np.int64)
    frac = ((r_odd & np.uint32(0x3FFFFFFF)).astype(np.float64) + 0.5) * (1.0 / (1 << 30))
    s, c = _sincos_quarter(frac * HALF_PI)
    cosphi = np.choose(quad, [c, -s, -c, s])
    sinphi = np.choose(quad, [s, c, -s, -c])
    return radius * cosphi, radius * sinphi


# ---- the generators ------------------------------------------------------------------

def words_per_elem(gp, fmt_id):
    return 2 if (gp.family == GEN_UNIFORM_EXP and fmt_id == fm.FP32) else 1


def _normal_range(gp, g0, count):
    p0, p1 = g0 >> 1, (g0 + count + 1) >> 1                       # pairs covering elements g0 .. g0+count-1
    pair = np.arange(p0, p1, dtype=np.uint64)
    ze, zo = normal_pairs(_words(gp.seed, gp.operand, pair * np.uint64(2)),
                          _words(gp.seed, gp.operand, pair * np.uint64(2) + np.uint64(1)))
    z = np.stack([ze, zo], axis=1).ravel()                         # element 2i from the cosine, 2i+1 from the sine
    off = g0 - 2 * p0
    return z[off:off + count]


def _value_range(gp, g0, count):
    """Unscaled binary64 values of elements g0 .. g0+count-1 for the three value families."""
    if gp.family == GEN_UNIFORM:
        g = np.arange(g0, g0 + count, dtype=np.uint64)
        r = _words(gp.seed, gp.operand, g).astype(np.float64)
        return (r + 0.5) * (1.0 / 2147483648.0) - 1.0
    z = _normal_range(gp, g0, count)
    if gp.family == GEN_NORMAL_OUTLIERS:
        from dataclasses import replace
        z2 = _normal_range(replace(gp, operand=gp.operand + 256), g0, count)
        g = np.arange(g0, g0 + count, dtype=np.uint64)
        hit = _words(gp.seed, gp.operand + 512, g).astype(np.uint64) < np.uint64(4294967)
        z = np.where(hit, z + 10.0 * z2, z)
    return z


def normal_values(gp, elems_per_tile, first_tile, n_tiles, threads=1):
    """Unscaled binary64 values of the value families (NORMAL, UNIFORM, NORMAL_OUTLIERS), shape (n_tiles, elems_per_tile).
    `threads` > 1 only splits the element range over a thread pool (numpy releases the GIL);
    every element is computed by the same operations either way."""
    g0 = first_tile * elems_per_tile
    total = n_tiles * elems_per_tile
    step = 1 << 18                                                 # cache-sized pieces
    if total <= step:
        return _value_range(gp, g0, total).reshape(n_tiles, elems_per_tile)
    from concurrent.futures import ThreadPoolExecutor
    starts = list(range(0, total, step))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        parts = list(ex.map(lambda s0: _value_range(gp, g0 + s0, min(step, total - s0)), starts))
    return np.concatenate(parts).reshape(n_tiles, elems_per_tile)


E8M0 = 5       # block-scale codes: one byte, 2^(code - 127), no sign and no mantissa


def _generate_scale_codes(gp, elems_per_tile, first_tile, n_tiles):
    """E8M0 codes from the bit-pattern families: all zero, the low byte of the element's word, or a code drawn
    uniformly from exp_lo .. exp_hi (plus code 0 with exp_zero) with the word's low 31 bits as the selector."""
    total = n_tiles * elems_per_tile
    if gp.family == GEN_ZERO:
        return np.zeros((n_tiles, elems_per_tile), dtype=np.uint32)
    g = np.arange(first_tile * elems_per_tile, first_tile * elems_per_tile + total, dtype=np.uint64)
    r = _words(gp.seed, gp.operand, g).astype(np.uint64)
    if gp.family == GEN_RANDOM_BITS:
        out = r & np.uint64(0xFF)
    elif gp.family == GEN_UNIFORM_EXP:
        nch = gp.exp_hi - gp.exp_lo + 1 + (1 if gp.exp_zero else 0)
        idx = ((r & np.uint64(0x7FFFFFFF)) * np.uint64(nch)) >> np.uint64(31)
        if gp.exp_zero:
            out = np.where(idx == 0, np.uint64(0), np.uint64(gp.exp_lo) + idx - np.uint64(1))
        else:
            out = np.uint64(gp.exp_lo) + idx
    else:
        raise ValueError("scale codes come from ZERO, RANDOM_BITS and UNIFORM_EXP only")
    return out.astype(np.uint32).reshape(n_tiles, elems_per_tile)


def _generate_fp64(gp, elems_per_tile, first_tile, n_tiles, threads=1):
    """binary64 output (uint64 patterns).  Value families: the binary64 value itself (times scale_target under
    SCALE_FACTOR; the other scale scopes are not defined here), one word per element as for every other format.  Bit
    families: element g owns the two words 2g (low half, lo) and 2g + 1 (high half, hi):
      RANDOM_BITS   hi:lo
      FINITE_BITS   v = floor(hi:lo * 2 * nmag / 2^64) with nmag = 2047 * 2^52 finite magnitudes; sign = v >= nmag
      UNIFORM_EXP   sign = hi bit 31; exponent field chosen by the low 31 bits of hi exactly as for FP32; mantissa =
                    (hi's low 20 bits):lo
      SIGNED_ZEROS  as for the other formats, decided by hi
    """
    total = n_tiles * elems_per_tile
    if gp.family == GEN_ZERO:
        return np.zeros((n_tiles, elems_per_tile), dtype=np.uint64)
    if gp.family in VALUE_FAMILIES:
        z = normal_values(gp, elems_per_tile, first_tile, n_tiles, threads)
        if gp.scale_scope == SCALE_FACTOR:
            z = z * np.float64(gp.scale_target)
        elif gp.scale_scope != SCALE_NONE:
            raise ValueError("binary64 output: no scaling, or a constant factor")
        return np.ascontiguousarray(z, dtype=np.float64).view(np.uint64).reshape(n_tiles, elems_per_tile)
    g = np.arange(first_tile * elems_per_tile, first_tile * elems_per_tile + total, dtype=np.uint64)
    lo = _words(gp.seed, gp.operand, g * np.uint64(2)).astype(np.uint64)
    hi = _words(gp.seed, gp.operand, g * np.uint64(2) + np.uint64(1)).astype(np.uint64)
    if gp.family == GEN_RANDOM_BITS:
        out = (hi << np.uint64(32)) | lo
    elif gp.family == GEN_FINITE_BITS:
        # floor((hi * 2^32 + lo) * 2047 * 2^53 / 2^64) = hi * 2047 * 2^21 + floor(lo * 2047 / 2^11)
        v = hi * np.uint64(2047) * np.uint64(1 << 21) + ((lo * np.uint64(2047)) >> np.uint64(11))
        nmag = np.uint64(2047 << 52)
        sign = (v >= nmag).astype(np.uint64)
        out = (sign << np.uint64(63)) | (v - sign * nmag)
    elif gp.family == GEN_UNIFORM_EXP:
        nch = gp.exp_hi - gp.exp_lo + 1 + (1 if gp.exp_zero else 0)
        sign = hi >> np.uint64(31)
        idx = ((hi & np.uint64(0x7FFFFFFF)) * np.uint64(nch)) >> np.uint64(31)
        if gp.exp_zero:
            E = np.where(idx == 0, np.uint64(0), np.uint64(gp.exp_lo) + idx - np.uint64(1))
        else:
            E = np.uint64(gp.exp_lo) + idx
        out = (sign << np.uint64(63)) | (E << np.uint64(52)) | ((hi & np.uint64(0xFFFFF)) << np.uint64(32)) | lo
    elif gp.family == GEN_SIGNED_ZEROS:
        sign, kind = (hi >> np.uint64(29)) & np.uint64(1), hi >> np.uint64(30)
        mag = np.where(kind == 2, np.uint64(1023 << 52), np.where(kind == 3, np.uint64(1), np.uint64(0)))
        out = (sign << np.uint64(63)) | mag
    else:
        raise ValueError("family %d is not defined for binary64 output" % gp.family)
    return out.reshape(n_tiles, elems_per_tile)


def generate(gp, fmt_id, elems_per_tile, first_tile, n_tiles, threads=1):
    """Raw bit patterns (uint32 array, shape (n_tiles, elems_per_tile)) of one operand."""
    if fmt_id == E8M0:
        return _generate_scale_codes(gp, elems_per_tile, first_tile, n_tiles)
    if fmt_id == fm.FP64:
        return _generate_fp64(gp, elems_per_tile, first_tile, n_tiles, threads)
    f = fm.FORMATS[fmt_id]
    total = n_tiles * elems_per_tile
    if gp.family == GEN_ZERO:
        return np.zeros((n_tiles, elems_per_tile), dtype=np.uint32)
    g = np.arange(first_tile * elems_per_tile, first_tile * elems_per_tile + total, dtype=np.uint64)
    wpe = words_per_elem(gp, fmt_id)
    if gp.family in VALUE_FAMILIES:
        z = normal_values(gp, elems_per_tile, first_tile, n_tiles, threads)
        if gp.scale_scope == SCALE_TENSOR:
            z = z * (np.float64(gp.scale_target) / np.abs(z).max())
        elif gp.scale_scope == SCALE_TILE:
            z = z * (np.float64(gp.scale_target) / np.abs(z).max(axis=1, keepdims=True))
        elif gp.scale_scope == SCALE_FACTOR:
            z = z * np.float64(gp.scale_target)
        b32 = z.astype(np.float32).view(np.uint32).ravel()
        step = 1 << 18
        out = np.concatenate([cast_from_fp32(b32[i:i + step], fmt_id) for i in range(0, b32.size, step)])
        return out.reshape(n_tiles, elems_per_tile)
    r = _words(gp.seed, gp.operand, g * np.uint64(wpe)).astype(np.uint64)
    if gp.family == GEN_RANDOM_BITS:
        out = r & np.uint64((1 << f.width) - 1)
    elif gp.family == GEN_FINITE_BITS:
        nmag = _n_finite_magnitudes(f)
        v = (r * np.uint64(2 * nmag)) >> np.uint64(32)
        sign = (v >= nmag).astype(np.uint64)
        out = (sign << np.uint64(f.width - 1)) | (v - sign * np.uint64(nmag))
    elif gp.family in (GEN_UNIFORM_EXP, GEN_CANCELLING):
        if gp.family == GEN_CANCELLING:
            if fmt_id == fm.FP32:
                raise ValueError("CANCELLING is not defined for FP32")
            r_own = r
            r = _words(gp.seed, gp.operand, (g & ~np.uint64(1)) * np.uint64(wpe)).astype(np.uint64)   # the even partner's word
        nch = gp.exp_hi - gp.exp_lo + 1 + (1 if gp.exp_zero else 0)
        sign = r >> np.uint64(31)
        if fmt_id == fm.FP32:
            sel, nsel = r & np.uint64(0x7FFFFFFF), 31
            mant = _words(gp.seed, gp.operand, g * np.uint64(2) + np.uint64(1)).astype(np.uint64) & np.uint64(0x7FFFFF)
        else:
            nsel = 31 - f.mbits
            sel = (r >> np.uint64(f.mbits)) & np.uint64((1 << nsel) - 1)
            mant = r & np.uint64((1 << f.mbits) - 1)
        idx = (sel * np.uint64(nch)) >> np.uint64(nsel)
        if gp.exp_zero:
            E = np.where(idx == 0, np.uint64(0), np.uint64(gp.exp_lo) + idx - np.uint64(1))
        else:
            E = np.uint64(gp.exp_lo) + idx
        out = (sign << np.uint64(f.width - 1)) | (E << np.uint64(f.mbits)) | mant
        if gp.family == GEN_CANCELLING:
            odd = (g & np.uint64(1)) == 1
            if gp.operand == 0:
                out = np.where(odd, out ^ np.uint64(1 << (f.width - 1)), out)
            else:
                flip = odd & ((r_own & np.uint64(0xF)) == 0)
                out = np.where(flip, out ^ np.uint64(1), out)
    elif gp.family == GEN_SIGNED_ZEROS:
        sign, kind = (r >> np.uint64(29)) & np.uint64(1), r >> np.uint64(30)
        mag = np.where(kind == 2, np.uint64(f.bias << f.mbits), np.where(kind == 3, np.uint64(1), np.uint64(0)))
        out = (sign << np.uint64(f.width - 1)) | mag
    else:
        raise ValueError(gp.family)
    return out.astype(np.uint32).reshape(n_tiles, elems_per_tile)
