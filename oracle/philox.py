"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11).

Test infrastructure only (see the package docstring).  The paper does not say
which generator its stochastic rounding used; Philox4x32-10 is this build's
reading, chosen because it is counter-based: the bits for coordinate g of
worker w are a pure function of (seed, w, g), so any chunk can be regenerated
anywhere.  Two independent implementations live here (Python big integers, one
block at a time; NumPy uint64 lanes) and the tests require them to agree with
each other and with the generator's published known-answer vectors.

Round function, as published: with counter words (c0, c1, c2, c3) and key
(k0, k1),
    (hi0, lo0) = M0 * c0   (32x32 -> 64 bit),  M0 = 0xD2511F53
    (hi1, lo1) = M1 * c2,                      M1 = 0xCD9E8D57
    (c0, c1, c2, c3) <- (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0)
ten rounds; before every round but the first the key is bumped by the Weyl
constants (0x9E3779B9, 0xBB67AE85).
"""

import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF


def philox4x32_10_scalar(counter, key):
    """One block with Python integers.  counter: 4 words, key: 2 words -> 4 words."""
    c0, c1, c2, c3 = (int(v) & MASK32 for v in counter)
    k0, k1 = (int(v) & MASK32 for v in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + W0) & MASK32
            k1 = (k1 + W1) & MASK32
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK32
        hi1, lo1 = p1 >> 32, p1 & MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return (c0, c1, c2, c3)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised blocks.  c0..c3 broadcastable integer arrays, k0/k1 scalars.

    Returns an array of shape (N, 4) of uint32, N = broadcast size.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(
        *(np.asarray(v, dtype=np.uint64) & np.uint64(MASK32) for v in (c0, c1, c2, c3))
    )
    c0, c1, c2, c3 = (v.reshape(-1).copy() for v in (c0, c1, c2, c3))
    k0 = int(k0) & MASK32
    k1 = int(k1) & MASK32
    m32 = np.uint64(MASK32)
    sh = np.uint64(32)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + W0) & MASK32
            k1 = (k1 + W1) & MASK32
        p0 = np.uint64(M0) * c0          # < 2^64, no wrap: both factors < 2^32
        p1 = np.uint64(M1) * c2
        hi0, lo0 = p0 >> sh, p0 & m32
        hi1, lo1 = p1 >> sh, p1 & m32
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
    return np.stack([c0, c1, c2, c3], axis=1).astype(np.uint32)
