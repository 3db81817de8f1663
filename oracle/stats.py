"""Bitwise comparison statistics.  Test infrastructure: see oracle/__init__.py.

The paper's requirement is bit-for-bit equality of model and interface outputs
(Eq. 2, and Step 4 of Sec. 3.1).  The statistics kept per comparison are this
library's own definition:

  n_compared            number of element pairs
  n_mismatch_bits       pairs whose 32-bit patterns differ
  n_mismatch_nan_equiv  pairs where both are NaN but the patterns differ
  first_mismatch_index  smallest (index_base + i) with differing patterns, 2^64-1 if none
  max_ulp_dist          largest ordered-integer distance over pairs of non-NaN values
  ulp_hist[34]          bucket 0: distance 0 (equal, +0 vs -0, or both NaN);
                        bucket i in 1..32: distance in [2^(i-1), 2^i);
                        bucket 33: exactly one of the two is NaN

Ordered-integer distance: map FP32 bits b to key(b) = b if the sign bit is clear,
else -(b & 0x7FFFFFFF); the distance is |key(x) - key(y)| (so +0 and -0 coincide
and adjacent floats are at distance 1).  FP16 outputs: the same on 16-bit patterns.  FP64 outputs (width 64): the
same on 64-bit patterns, with bucket 32 also taking every distance of 2^32 and more.
"""
import numpy as np

NO_MISMATCH = (1 << 64) - 1
N_BUCKETS = 34


def ordered_key(bits, width=32):
    if width == 64:                      # (Python integers: the keys span 65 bits' worth of distance)
        sign = 1 << 63
        return np.array([-(int(b) & (sign - 1)) if int(b) & sign else int(b) for b in np.asarray(bits).ravel()], dtype=object)
    b = np.asarray(bits, dtype=np.uint32).astype(np.int64)
    sign = 1 << (width - 1)
    return np.where(b & sign, -(b & (sign - 1)), b)


def is_nan(bits, width=32):
    if width == 64:
        return (np.asarray(bits, dtype=np.uint64) & np.uint64(0x7FFFFFFFFFFFFFFF)) > np.uint64(0x7FF0000000000000)
    b = np.asarray(bits, dtype=np.uint32)
    return (b & ((1 << (width - 1)) - 1)) > (0x7F800000 if width == 32 else 0x7C00)


def empty_stats():
    return dict(n_compared=0, n_mismatch_bits=0, n_mismatch_nan_equiv=0,
                first_mismatch_index=NO_MISMATCH, max_ulp_dist=0, ulp_hist=[0] * N_BUCKETS)


def compare(d0, d1, stats=None, index_base=0, width=32):
    """Accumulate the comparison of two FP32 (width 32) or FP16 (width 16) bit arrays into `stats` (a dict)."""
    assert width in (64, 32, 16)
    st = empty_stats() if stats is None else stats
    x = np.asarray(d0, dtype=np.uint64 if width == 64 else np.uint32).ravel()
    y = np.asarray(d1, dtype=np.uint64 if width == 64 else np.uint32).ravel()
    assert x.shape == y.shape
    st["n_compared"] += int(x.size)
    diff = x != y
    st["n_mismatch_bits"] += int(diff.sum())
    nx, ny = is_nan(x, width), is_nan(y, width)
    st["n_mismatch_nan_equiv"] += int((diff & nx & ny).sum())
    if diff.any():
        st["first_mismatch_index"] = min(st["first_mismatch_index"], index_base + int(np.argmax(diff)))
    one_nan = nx ^ ny
    both_nan = nx & ny
    st["ulp_hist"][33] += int(one_nan.sum())
    st["ulp_hist"][0] += int(both_nan.sum())
    num = ~(nx | ny)
    dist = np.abs(ordered_key(x[num], width) - ordered_key(y[num], width))
    if dist.size:
        st["max_ulp_dist"] = max(st["max_ulp_dist"], int(dist.max()))
        # bucket = bit length of the distance (at most 32: only 64-bit patterns lie farther apart)
        bl = np.zeros(dist.shape, dtype=np.int64)
        for i in range(32):
            bl += (dist >= (1 << i)).astype(np.int64)
        for i, c in zip(*np.unique(bl, return_counts=True)):
            st["ulp_hist"][int(i)] += int(c)
    return st
