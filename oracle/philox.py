"""Philox4x32-10 counter-based generator (Salmon et al., SC'11), vectorised.

The paper only needs unbiased rounding (Corollary 2.1, item 1) and i.i.d.
sampling (Section 2, "Stochastic Optimization"); the generator is this build's
choice so that CPU and GPU draw identical streams.  Test infrastructure only.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(key, c0, c1, c2, c3):
    """Ten Philox rounds.  key = (k0, k1) python ints; c0..c3 broadcastable
    arrays / ints of 32-bit counter words.  Returns four uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(
        *(np.asarray(c, dtype=np.uint64) & _MASK for c in (c0, c1, c2, c3)))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0                      # 32x32 -> 64 bit product
        p1 = _M1 * c2
        n0 = (p1 >> _SH) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK
        n2 = (p0 >> _SH) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF       # key schedule (Weyl sequence)
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))
