"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11).

Test infrastructure: see the package docstring.

One call maps a 128-bit counter (four 32-bit words) and a 64-bit key (two
words) to four 32-bit outputs.  A round takes (c0, c1, c2, c3) to
(hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0));
after every round but the last the key words grow by the Weyl constants.
Pinned by the generator's published known-answer vectors (tests/golden).
"""
import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """counter: 4 python ints (32-bit), key: 2 python ints.  Returns 4 ints."""
    c0, c1, c2, c3 = (int(v) & MASK for v in counter)
    k0, k1 = (int(v) & MASK for v in key)
    for r in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = (((p1 >> 32) ^ c1 ^ k0) & MASK, p1 & MASK,
                          ((p0 >> 32) ^ c3 ^ k1) & MASK, p0 & MASK)
        if r != 9:
            k0 = (k0 + W0) & MASK
            k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def philox4x32_10_array(c0, c1, c2, c3, k0, k1):
    """Same function over NumPy arrays (broadcast), all values held in uint64."""
    c0, c1, c2, c3 = (np.asarray(v, dtype=np.uint64) & np.uint64(MASK) for v in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = np.uint64(int(k0) & MASK)
    k1 = np.uint64(int(k1) & MASK)
    m = np.uint64(MASK)
    s32 = np.uint64(32)
    for r in range(10):
        p0 = np.uint64(M0) * c0          # < 2^64, no wrap
        p1 = np.uint64(M1) * c2
        c0, c1, c2, c3 = ((p1 >> s32) ^ c1 ^ k0, p1 & m, (p0 >> s32) ^ c3 ^ k1, p0 & m)
        if r != 9:
            k0 = (k0 + np.uint64(W0)) & m
            k1 = (k1 + np.uint64(W1)) & m
    return c0, c1, c2, c3
