"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11).

One round maps a 4x32-bit counter c and a 2x32-bit key k to
  (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0));
the key is advanced by the Weyl constants before every round but the first;
ten rounds are applied.
"""
import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """Scalar version on Python integers. ctr: 4 words, key: 2 words."""
    c0, c1, c2, c3 = (int(x) & MASK32 for x in ctr)
    k0, k1 = (int(x) & MASK32 for x in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + W0) & MASK32
            k1 = (k1 + W1) & MASK32
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0, p1 & MASK32,
                          (p0 >> 32) ^ c3 ^ k1, p0 & MASK32)
    return c0, c1, c2, c3


def philox4x32_10_array(c0, c1, c2, c3, k0, k1):
    """Vectorised version: uint64 arrays holding 32-bit values (broadcastable).
    Returns the four output words as uint64 arrays."""
    u = np.uint64
    c0, c1, c2, c3 = (np.asarray(x, dtype=u) for x in (c0, c1, c2, c3))
    k0, k1 = u(int(k0) & MASK32), u(int(k1) & MASK32)
    m32, sh = u(MASK32), u(32)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + u(W0)) & m32
            k1 = (k1 + u(W1)) & m32
        p0 = u(M0) * c0
        p1 = u(M1) * c2
        c0, c1, c2, c3 = ((p1 >> sh) ^ c1 ^ k0, p1 & m32,
                          (p0 >> sh) ^ c3 ^ k1, p0 & m32)
    return c0, c1, c2, c3
