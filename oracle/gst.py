"""Group-scaled truncated FDPA.  Test infrastructure: see oracle/__init__.py.

Follows the paper's Sec. 4.1.3, paragraph "Group-Scaled Truncated FDPA (GST-FDPA)" and Algorithm "GST-FDPA", step
by step on exact rationals:

  Step 1  for every group g of G consecutive products: p_g = sum a_k b_k, exact; s_g = p_g * SignedSig(alpha) *
          SignedSig(beta) and e_g = Exp(alpha) + Exp(beta) with the scale factors of the group's block (one pair per
          K_block consecutive elements; the group lies inside one block)
  Step 2  the accumulator joins as term L/G: s = SignedSig(c), e = Exp(c); e_max over all L/G + 1 exponents; every
          term is aligned at e_max and truncated toward zero to F fractional bits; exact sum S
  Step 3  d = rho(S * 2^e_max)

Phi over a row: d <- c, then one such operation per L consecutive products (Algorithm "Phi_FDPA").
Scale factor types (Require line of the algorithm): E8M0 (SignedSig = 1, Exp = code - 127, code 255 = NaN) and UE4M3,
the unsigned E4M3 of NVFP4 (SignedSig and Exp of the E4M3 decoding with bias 7, exponent field 0: Exp = -6 and no
hidden bit; codes 0x7F and 0xFF are NaN; the top bit is otherwise ignored).
Table "GST-FDPA parameter selection": L = 64, G = 16, F = 35, RZ-FP32, K_block = 32 (MXFP4) or 16 (NVFP4).

Readings where the paper is silent: a NaN scale factor, a NaN accumulator or infinities follow Sec. 4.2 (the FP4
operands themselves are always finite); an exact-zero sum is +0.0; the NaN pattern is the model's nan_bits.
"""
from fractions import Fraction

from . import formats as fm
from .rounding import to_fp32

SCALE_E8M0, SCALE_UE4M3 = 0, 1


def decode_scale(code, scale_format):
    """(signed significand, exponent) of a scale factor, or None for a NaN code."""
    code = int(code) & 0xFF
    if scale_format == SCALE_E8M0:
        return None if code == 0xFF else (Fraction(1), code - 127)
    if scale_format == SCALE_UE4M3:
        d = fm.decode(code & 0x7F, fm.E4M3)
        return None if d.cls == fm.NAN else (Fraction(d.sig, 8), d.exp)
    raise ValueError(scale_format)


def _rz_frac(x, F):
    n = abs(x) * (1 << F)
    n = n.numerator // n.denominator
    r = Fraction(n, 1 << F)
    return -r if x < 0 else r


def gst_fdpa(a_bits, b_bits, c_bits, alpha, beta, G, k_block, F, out_round, scale_format, nan_bits=0x7FFFFFFF,
             ta=fm.E2M1, tb=fm.E2M1):
    """One GST-FDPA operation on L = len(a_bits) products.  alpha, beta: L / k_block scale codes each."""
    L = len(a_bits)
    if L % G or L % k_block or not (k_block % G == 0 or G % k_block == 0):
        raise ValueError("group and block sizes must divide the vector length and one another")
    if G > k_block:
        raise ValueError("a group lies inside one block of scale factors")
    dc = fm.decode(c_bits, fm.FP32)
    if dc.cls == fm.NAN:
        return nan_bits
    terms = []                                                     # (s_g, e_g)
    for g in range(L // G):
        sa, sb = decode_scale(alpha[g * G // k_block], scale_format), decode_scale(beta[g * G // k_block], scale_format)
        if sa is None or sb is None:
            return nan_bits
        p = sum((fm.decode(a_bits[k], ta).value * fm.decode(b_bits[k], tb).value for k in range(g * G, (g + 1) * G)), Fraction(0))
        terms.append((p * sa[0] * sb[0], sa[1] + sb[1]))
    if dc.cls == fm.INF:
        return 0xFF800000 if dc.sign else 0x7F800000
    terms.append((dc.signed_sig, dc.exp))
    e_max = max(e for _, e in terms)
    S = sum((_rz_frac(s * Fraction(2) ** (e - e_max), F) for s, e in terms), Fraction(0))
    return to_fp32(S * Fraction(2) ** e_max, out_round)


def emulate_element(a_bits, b_bits, c_bits, alpha, beta, L, G, k_block, F, out_round, scale_format, nan_bits=0x7FFFFFFF,
                    ta=fm.E2M1, tb=fm.E2M1):
    """Chain over K / L operations for one output element; alpha, beta: K / k_block scale codes of the row / column."""
    K = len(a_bits)
    L = K if L == 0 else min(L, K)
    if K % L or L % k_block:
        raise ValueError("K must be a multiple of L and L of the block size")
    d = int(c_bits)
    for k0 in range(0, K, L):
        q0, q1 = k0 // k_block, (k0 + L) // k_block
        d = gst_fdpa([int(x) for x in a_bits[k0:k0 + L]], [int(x) for x in b_bits[k0:k0 + L]], d, alpha[q0:q1], beta[q0:q1],
                     G, k_block, F, out_round, scale_format, nan_bits, ta, tb)
    return d
