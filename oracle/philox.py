"""Philox4x32-10 counter-based random numbers (oracle side; test infrastructure).

The paper is silent on the random number generator behind its "uniform sample
of nodes" (Sec. 2.1) and its degree-based fraction (Sec. 5.1, Table 1 caption).
The reading taken here is a stateless counter-based generator so that CPU and
GPU can draw identical ids: Philox4x32 with 10 rounds as published by Salmon,
Moraes, Dror and Shaw ("Parallel random numbers: as easy as 1, 2, 3", SC'11).

Two implementations live here on purpose: a scalar one on Python integers (the
definition, exact by construction) and a numpy one used for bulk draws.  Both
are pinned by the published known-answer vectors in tests/golden/.
"""
import numpy as np

# Round multipliers and Weyl key increments of the published algorithm.
_M0 = 0xD2511F53
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """One block: 4x32-bit counter, 2x32-bit key -> 4x32-bit output (Python ints)."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & _MASK32, p1 & _MASK32, \
                         ((p0 >> 32) ^ c3 ^ k1) & _MASK32, p0 & _MASK32
        k0 = (k0 + _W0) & _MASK32
        k1 = (k1 + _W1) & _MASK32
    return c0, c1, c2, c3


def philox4x32_10_np(c0, c1, c2, c3, k0, k1):
    """Vectorised blocks.  Counter words are uint64 arrays holding 32-bit values
    (broadcastable against each other); key words are Python ints.  Returns four
    uint64 arrays holding 32-bit values."""
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(x, dtype=np.uint64) for x in (c0, c1, c2, c3)))
    c0 = c0.copy(); c1 = c1.copy(); c2 = c2.copy(); c3 = c3.copy()
    m32 = np.uint64(_MASK32)
    sh = np.uint64(32)
    k0 = int(k0) & _MASK32
    k1 = int(k1) & _MASK32
    for _ in range(10):
        p0 = np.uint64(_M0) * c0          # 32x32 -> 64 bit, no overflow
        p1 = np.uint64(_M1) * c2
        n0 = (p1 >> sh) ^ c1 ^ np.uint64(k0)
        n2 = (p0 >> sh) ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, p1 & m32, n2, p0 & m32
        k0 = (k0 + _W0) & _MASK32
        k1 = (k1 + _W1) & _MASK32
    return c0, c1, c2, c3


def mulhi64(x, n):
    """High 64 bits of the 128-bit product x*n: maps a 64-bit word x onto [0, n).
    Scalar definition on Python integers."""
    return (int(x) * int(n)) >> 64


def mulhi64_np(x, n):
    """Vectorised mulhi64 for uint64 array x and Python int n < 2**63, by splitting
    x into 32-bit halves (schoolbook product)."""
    x = np.asarray(x, dtype=np.uint64)
    n = int(n)
    assert 0 <= n < (1 << 63)
    m32 = np.uint64(_MASK32)
    sh = np.uint64(32)
    xl = x & m32
    xh = x >> sh
    nl = np.uint64(n & _MASK32)
    nh = np.uint64(n >> 32)
    ll = xl * nl
    lh = xl * nh
    hl = xh * nl
    hh = xh * nh
    mid = (ll >> sh) + (lh & m32) + (hl & m32)       # < 3 * 2**32, fits
    return hh + (lh >> sh) + (hl >> sh) + (mid >> sh)
