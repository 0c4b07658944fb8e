"""Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC'11), vectorised over numpy arrays of counters.

Test infrastructure only (see the package docstring).  The paper asks only for a seeded
Gaussian P that can be re-generated instead of stored (Algorithm 1; Section 4.3 "eliminating
the need to store a projection matrix"); a counter-based generator is what makes that a pure
function of (seed, tensor, epoch, element).
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)   # multiplier applied to counter word 0
_M1 = np.uint64(0xCD9E8D57)   # multiplier applied to counter word 2
_W0 = 0x9E3779B9              # key word 0 increment per round (golden ratio)
_W1 = 0xBB67AE85              # key word 1 increment per round (sqrt(3) - 1)
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Return the four 32-bit output words for counter (c0,c1,c2,c3) and key (k0,k1).

    c0..c3 are array-likes of equal shape (values < 2**32); k0, k1 are Python ints.
    Output: four uint32 arrays of that shape.
    """
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0                      # 64-bit products of 32-bit values: no overflow
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        n0 = hi1 ^ c1 ^ np.uint64(k0)
        n2 = hi0 ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))
