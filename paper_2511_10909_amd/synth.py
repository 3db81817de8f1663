"""Seeded synthetic operand builders for tests: raw bit patterns only.

Nothing here performs any of the model's arithmetic; this module is imported by
tests to feed identical inputs to the CPU oracle and to the HIP library.
"""
import numpy as np

E4M3, E5M2, FP16, BF16, FP32 = 0, 1, 2, 3, 4
E2M3, E3M2, E2M1 = 6, 7, 8                      # FP6 and FP4: one code per byte, in its low bits
TF32 = 9                                        # whole binary32 words (the low 13 bits are drawn too: the models ignore them)
WIDTH = {E4M3: 8, E5M2: 8, FP16: 16, BF16: 16, FP32: 32, E2M3: 6, E3M2: 6, E2M1: 4, TF32: 32}     # bits of a code, sign on top
EBITS = {E4M3: 4, E5M2: 5, FP16: 5, BF16: 8, FP32: 8, E2M3: 2, E3M2: 3, E2M1: 2, TF32: 8}
MBITS = {E4M3: 3, E5M2: 2, FP16: 10, BF16: 7, FP32: 23, E2M3: 3, E3M2: 2, E2M1: 1, TF32: 23}
NP_DTYPE = {E4M3: np.uint8, E5M2: np.uint8, FP16: np.uint16, BF16: np.uint16, FP32: np.uint32, 5: np.uint8,   # 5: E8M0 scale codes
            E2M3: np.uint8, E3M2: np.uint8, E2M1: np.uint8, TF32: np.uint32}


def _is_special(bits, t):
    e = (bits >> MBITS[t]) & ((1 << EBITS[t]) - 1)
    man = bits & ((1 << MBITS[t]) - 1)
    if t == E4M3:
        return (e == 15) & (man == 7)
    if t in (E2M3, E3M2, E2M1):
        return np.zeros(np.shape(bits), dtype=bool)         # every code is a finite number
    return e == (1 << EBITS[t]) - 1


def random_bits(rng, shape, t, finite=True):
    """Uniform random bit patterns; with finite=True NaN/Inf codes are redrawn as zeros
    of the same sign."""
    b = rng.integers(0, 1 << WIDTH[t], size=shape, dtype=np.uint64)
    if finite:
        b = np.where(_is_special(b, t), b & (1 << (WIDTH[t] - 1)), b)
    return b.astype(NP_DTYPE[t])


def narrow_exponent_bits(rng, shape, t, e_lo, e_hi):
    """Random sign and mantissa, exponent field uniform in [e_lo, e_hi]."""
    s = rng.integers(0, 2, size=shape, dtype=np.uint64)
    e = rng.integers(e_lo, e_hi + 1, size=shape, dtype=np.uint64)
    man = rng.integers(0, 1 << MBITS[t], size=shape, dtype=np.uint64)
    return ((s << (WIDTH[t] - 1)) | (e << MBITS[t]) | man).astype(NP_DTYPE[t])


def sprinkle(rng, arr, codes, frac):
    """Overwrite a fraction of entries with the given special codes."""
    out = arr.copy()
    mask = rng.random(arr.shape) < frac
    pick = rng.integers(0, len(codes), size=arr.shape)
    out[mask] = np.asarray(codes, dtype=arr.dtype)[pick[mask]]
    return out


SPECIAL_CODES = {
    E4M3: [0x7F, 0xFF, 0x00, 0x80, 0x7E, 0x01],
    E5M2: [0x7C, 0xFC, 0x7D, 0x00, 0x80, 0x7B, 0x01],
    FP16: [0x7C00, 0xFC00, 0x7E00, 0x0000, 0x8000, 0x7BFF, 0x0001],
    BF16: [0x7F80, 0xFF80, 0x7FC0, 0x0000, 0x8000, 0x7F7F, 0x0001],
    FP32: [0x7F800000, 0xFF800000, 0x7FC00000, 0, 0x80000000, 0x7F7FFFFF, 1],
    TF32: [0x7F800000, 0xFF800000, 0x7FC00000, 0x7F802000, 0x7F801FFF, 0, 0x80000000, 0x7F7FFFFF, 0x00002000, 0x00001FFF],
    E2M3: [0x00, 0x20, 0x1F, 0x3F, 0x01], E3M2: [0x00, 0x20, 0x1F, 0x3F, 0x01], E2M1: [0x0, 0x8, 0x7, 0xF, 0x1],
}
