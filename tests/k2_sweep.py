"""Shared pieces of the exhaustive k = 2 FP8 sweeps (CPU pin and GPU parity).

A fused dot-product-add of two FP8 products depends on the four operand codes only through the two products'
classes: NaN, an infinity with its sign, or (sign, e_k, s_k) -- the sign, the unnormalised exponent sum and the integer
significand product that Algorithm "T-FDPA" forms in its first step.  So the outputs of all 2^32 code tuples follow
from the outputs of all PAIRS OF CLASSES (a few thousand classes per type pairing), looked up through the class of
each (a, b) code pair.  Nothing here evaluates the model: classes come from the decoders, values from torch's float8
types, and the closed forms are plain binary64 arithmetic.
"""
import numpy as np

from oracle import formats as fm

PAIRINGS = [(fm.E4M3, fm.E4M3), (fm.E4M3, fm.E5M2), (fm.E5M2, fm.E4M3), (fm.E5M2, fm.E5M2)]
NAN_BITS = 0x7FC00000


def product_classes(ta, tb):
    """cls[a | b << 8] = class id of the product of codes a (type ta) and b (type tb); reps[c] = one (a, b) of class c;
    info[c] = ("nan",) | ("inf", sign) | ("fin", sign, e, s)."""
    da = [fm.decode(x, ta) for x in range(256)]
    db = [fm.decode(x, tb) for x in range(256)]
    ids, reps, info = {}, [], []
    cls = np.zeros(65536, dtype=np.int32)
    for b in range(256):
        for a in range(256):
            x, y = da[a], db[b]
            if x.cls == fm.NAN or y.cls == fm.NAN:
                k = ("nan",)
            elif x.cls == fm.INF or y.cls == fm.INF:
                k = ("nan",) if (x.cls == fm.ZERO or y.cls == fm.ZERO) else ("inf", x.sign ^ y.sign)
            else:
                k = ("fin", x.sign ^ y.sign, x.exp + y.exp, x.sig * y.sig)
            if k not in ids:
                ids[k] = len(reps)
                reps.append((a, b))
                info.append(k)
            cls[a | (b << 8)] = ids[k]
    return cls, np.array(reps, dtype=np.uint8), info


def class_pair_operands(reps):
    """A[n*n][1][2], B[n*n][1][2] (codes) for every ordered pair of classes (c0, c1), index c0 * n + c1."""
    n = len(reps)
    i0, i1 = np.divmod(np.arange(n * n, dtype=np.int64), n)
    A = np.stack([reps[i0, 0], reps[i1, 0]], axis=1).reshape(n * n, 1, 2)
    B = np.stack([reps[i0, 1], reps[i1, 1]], axis=1).reshape(n * n, 1, 2)
    return A, B


def _values(t):
    """Exact values of all 256 codes as binary64, through torch's float8 types (NaN / inf as such)."""
    import torch
    dt = torch.float8_e4m3fn if t == fm.E4M3 else torch.float8_e5m2
    return torch.arange(256, dtype=torch.uint8).view(dt).to(torch.float64).numpy()


def _exponents(t):
    """Unnormalised exponent of every code: max(exponent field, 1) - bias."""
    f = fm.FORMATS[t]
    E = (np.arange(256) >> f.mbits) & f.emax_field
    return np.maximum(E, 1) - f.bias


def closed_form_table(ta, tb, reps, info, F):
    """D for every ordered pair of classes, c = +0, no flush, RNE-FP32, evaluated in binary64 from the definition:
    e_max = max(e_0, e_1, Exp(c)); every product cut toward zero to a multiple of 2^(e_max - F); exact sum; one rounding.
    F = None: nothing is cut (the exact sum of the two products, rounded once).  Special values by the rules of Sec. 4.2."""
    n = len(reps)
    va, vb = _values(ta), _values(tb)
    ea, eb = _exponents(ta), _exponents(tb)
    a, b = reps[:, 0].astype(np.int64), reps[:, 1].astype(np.int64)
    kind = np.array([{"nan": 2, "inf": 1, "fin": 0}[k[0]] for k in info])
    sign = np.array([k[1] if len(k) > 1 else 0 for k in info])
    with np.errstate(invalid="ignore", over="ignore"):
        p = np.where(kind == 0, va[a] * vb[b], 0.0)               # exact: at most 8 significant bits
    e = (ea[a] + eb[b]).astype(np.int64)
    P0, P1 = p[:, None], p[None, :]
    E0, E1 = e[:, None], e[None, :]
    if F is None:
        # exact two-term sum in binary64: s + err (error-free transformation), rounded to odd when inexact, so that the
        # conversion to binary32 rounds the exact sum once
        s = P0 + P1
        bb = s - P0
        err = (P0 - (s - bb)) + (P1 - bb)
        bits = s.view(np.int64).copy()
        inexact = err != 0.0
        toward_zero = inexact & ((err < 0.0) != (s < 0.0))
        bits = np.where(toward_zero, bits - 1, bits)
        bits = np.where(inexact, bits | 1, bits)
        v = bits.view(np.float64)
    else:
        emax = np.maximum(np.maximum(E0, E1), -126)                 # the accumulator +0 takes part with Exp = -126
        sc = np.ldexp(1.0, (F - emax).astype(np.int64))
        v = (np.trunc(P0 * sc) + np.trunc(P1 * sc)) / sc            # integers below 2^53, exact
    with np.errstate(over="ignore"):
        out = v.astype(np.float32).view(np.uint32).astype(np.uint32)
    out = np.where(v == 0.0, np.uint32(0), out)                     # an exact zero is +0.0
    # special values: NaN anywhere, or infinities of both signs: NaN; else an infinity keeps its sign
    K0, K1 = kind[:, None], kind[None, :]
    S0, S1 = sign[:, None], sign[None, :]
    any_nan = (K0 == 2) | (K1 == 2) | ((K0 == 1) & (K1 == 1) & (S0 != S1))
    inf = ((K0 == 1) | (K1 == 1)) & ~any_nan
    inf_sign = np.where(K0 == 1, S0, S1)
    out = np.where(inf, np.where(inf_sign == 1, np.uint32(0xFF800000), np.uint32(0x7F800000)), out)
    out = np.where(any_nan, np.uint32(NAN_BITS), out)
    return out.reshape(n * n)
