"""Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC'11), the counter-based generator the layer's "PRNG state"
(Algorithm 1, Forward step 2 / Backward step 2) is realised with.

Test infrastructure: pure integer arithmetic in numpy uint64 so that every
32x32->64 product is exact.  Pinned by the authors' published known-answer
vectors (tests/golden/philox4x32_10_kat.txt).
"""
import numpy as np

# Round multipliers and key increments (Weyl constants) of Philox-4x32.
_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten-round Philox bijection of the 128-bit counter (c0..c3) under the
    64-bit key (k0, k1).  All arguments broadcast against each other; each is
    interpreted modulo 2**32.  Returns four uint32 arrays (r0, r1, r2, r3).
    """
    c0, c1, c2, c3, k0, k1 = (np.asarray(a, dtype=np.uint64) & _MASK
                              for a in (c0, c1, c2, c3, k0, k1))
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(c0, c1, c2, c3, k0, k1)
    for rnd in range(10):
        if rnd > 0:                       # key schedule: bump before rounds 2..10
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0                     # exact 64-bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(a.astype(np.uint32) for a in (c0, c1, c2, c3))


def philox4x32_10_scalar(counter, key):
    """Same bijection on Python ints (no numpy), used to cross-check the
    vectorised routine on random inputs.  counter: 4 ints, key: 2 ints."""
    c = [int(x) & 0xFFFFFFFF for x in counter]
    k = [int(x) & 0xFFFFFFFF for x in key]
    for rnd in range(10):
        if rnd:
            k[0] = (k[0] + 0x9E3779B9) & 0xFFFFFFFF
            k[1] = (k[1] + 0xBB67AE85) & 0xFFFFFFFF
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF,
             (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return tuple(c)
