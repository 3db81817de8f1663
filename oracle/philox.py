"""Philox-4x32-10 (J. Salmon, M. Moraes, R. Dror, D. Shaw, "Parallel random numbers:
as easy as 1, 2, 3", SC'11), written from its published definition.
Test infrastructure: see oracle/__init__.py.

One call maps a 128-bit counter (c0..c3) and a 64-bit key (k0, k1) to four
32-bit words through ten rounds of
    (c0, c1, c2, c3) <- (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0))
with the key bumped by the Weyl constants (W0, W1) between rounds.
"""
import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised over numpy arrays (or scalars) of counters; returns four uint32 arrays."""
    c0 = np.asarray(c0, dtype=np.uint64) & MASK
    c1 = np.asarray(c1, dtype=np.uint64) & MASK
    c2 = np.asarray(c2, dtype=np.uint64) & MASK
    c3 = np.asarray(c3, dtype=np.uint64) & MASK
    k0 = int(k0) & MASK
    k1 = int(k1) & MASK
    for _ in range(10):
        p0 = np.uint64(M0) * c0          # < 2^64, exact in uint64
        p1 = np.uint64(M1) * c2
        n0 = (p1 >> np.uint64(32)) ^ c1 ^ np.uint64(k0)
        n1 = p1 & np.uint64(MASK)
        n2 = (p0 >> np.uint64(32)) ^ c3 ^ np.uint64(k1)
        n3 = p0 & np.uint64(MASK)
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return tuple(x.astype(np.uint32) for x in (c0, c1, c2, c3))
