"""Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11).

Test infrastructure only (see package docstring).  The RESCAL paper names no generator for its
resampling step (Alg. 4: "uniformRandom") or for the random initialisation (Alg. 3 step 1); this
build fixes a counter-based one so that a perturbed tensor is a pure function of
(seed, member, coordinates) and never has to be stored.

Two independent implementations live here on purpose: `philox4x32_10` (NumPy, vectorised over
counters) and `philox4x32_10_scalar` (plain Python integers, one block).  Tests require them to agree
word for word and to reproduce the known-answer vectors published with the generator.
"""
import numpy as np

# Multipliers and key increments (Weyl constants) of the 4x32 variant as published.
_M0 = 0xD2511F53
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10_scalar(counter, key):
    """One block.  counter: 4 ints < 2**32, key: 2 ints < 2**32 -> tuple of 4 ints."""
    c0, c1, c2, c3 = (int(c) & _MASK for c in counter)
    k0, k1 = (int(k) & _MASK for k in key)
    for _ in range(10):
        p0 = _M0 * c0            # 64-bit product of the first multiplier with word 0
        p1 = _M1 * c2            # 64-bit product of the second multiplier with word 2
        hi0, lo0 = p0 >> 32, p0 & _MASK
        hi1, lo1 = p1 >> 32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + _W0) & _MASK
        k1 = (k1 + _W1) & _MASK
    return c0, c1, c2, c3


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised blocks.  c0..c3 broadcastable integer arrays (values < 2**32), k0, k1 Python ints.

    Returns four uint32 arrays of the broadcast shape.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3)))
    c0, c1, c2, c3 = c0.copy(), c1.copy(), c2.copy(), c3.copy()
    m0, m1, mask = np.uint64(_M0), np.uint64(_M1), np.uint64(_MASK)
    s32 = np.uint64(32)
    k0 = int(k0) & _MASK
    k1 = int(k1) & _MASK
    for _ in range(10):
        p0 = m0 * c0             # < 2**64: both factors < 2**32
        p1 = m1 * c2
        n0 = (p1 >> s32) ^ c1 ^ np.uint64(k0)
        n1 = p1 & mask
        n2 = (p0 >> s32) ^ c3 ^ np.uint64(k1)
        n3 = p0 & mask
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & _MASK
        k1 = (k1 + _W1) & _MASK
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))
