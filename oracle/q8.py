"""Group-wise 8-bit weights (oracle side): the storage format and its re-quantisation.

Test infrastructure only (see the package docstring).  The paper combines APOLLO with "Int8 weight
quantization ... group size of 128" (Section 5.4, Table 6) and refers to Q-GaLore for the method;
it specifies nothing further.  Reading taken (the usual asymmetric min/max group quantiser, with
the stochastic rounding that keeps updates smaller than a code step from vanishing):

  * Format.  A weight matrix (row-major, row length a multiple of 128) is held as unsigned 8-bit
    codes q[e] and, per group of 128 consecutive elements, an fp32 pair (scale, zero):
        w[e] = zero + scale * q[e].
  * Step.  The codes are de-quantised, the update of Algorithm 1 (step 4) is applied to the real
    values, and every group is quantised again from its own new range:
        zero' = min w',  scale' = (max w' - min w') / 255,  x[e] = (w'[e] - zero') / scale'
    (x = 0 for a constant group, scale' = 0), and q'[e] = min(255, floor(x[e] + u[e])).
  * Rounding.  Nearest: u = 1/2.  Stochastic: u is uniform on {0, 1, ..., 65535} / 65536, drawn
    from Philox4x32-10 under the optimizer's seed with counter (o mod 2^32, step, 2^31 + tensor
    index, o div 2^32), o = e div 8: output word k (k = 0..3) gives element 8 o + 2 k its low and
    element 8 o + 2 k + 1 its high 16 bits.  (The projection's counters have a third word below
    2^31: the two streams cannot collide.)  E[q'] = x: the expected stored value is the real one.
"""
import numpy as np

from .philox import philox4x32_10

GROUP = 128
NEAREST, STOCHASTIC = "nearest", "stochastic"


class Q8Weights:
    """codes: uint8 (rows, cols); scale, zero: float64 arrays of fp32 values, (rows, cols / 128)."""

    def __init__(self, codes, scale, zero):
        self.codes = np.asarray(codes, dtype=np.uint8)
        self.scale = np.asarray(scale, dtype=np.float64)
        self.zero = np.asarray(zero, dtype=np.float64)
        rows, cols = self.codes.shape
        if cols % GROUP or self.scale.shape != (rows, cols // GROUP) or self.zero.shape != self.scale.shape:
            raise ValueError("row length must be a multiple of 128, one (scale, zero) per group")

    def dequantise(self):
        return dequantise_values(self.codes.astype(np.float64), self.scale, self.zero)


def dequantise_values(codes, scale, zero):
    """w = zero + scale * q for codes (rows, cols; as floating-point numbers) and per-group (rows,
    cols / 128) scale and zero.  Uses array methods common to numpy and torch only, so that a test
    can evaluate it on arrays that live on another device."""
    rows, cols = codes.shape
    q = codes.reshape(rows, cols // GROUP, GROUP)
    return (zero.reshape(rows, cols // GROUP, 1) + scale.reshape(rows, cols // GROUP, 1) * q).reshape(rows, cols)


def group_positions(w_exact, xp=np):
    """The range of every group of 128 consecutive elements of a row and the real-valued code positions
    in it: (lo, hi, x) with lo, hi of shape (rows, cols / 128) and x = 255 (w - lo) / (hi - lo) of shape
    (rows, cols), 0 for a constant group.  xp: the array namespace (numpy or torch)."""
    rows, cols = w_exact.shape
    g = w_exact.reshape(rows, cols // GROUP, GROUP)
    if xp is np:
        lo, hi = g.min(axis=2), g.max(axis=2)
    else:
        lo, hi = g.min(dim=2).values, g.max(dim=2).values
    rng = (hi - lo).reshape(rows, cols // GROUP, 1)
    safe = xp.where(rng > 0, rng, rng + 1.0)
    x = xp.where(rng > 0, (g - lo.reshape(rows, cols // GROUP, 1)) / (safe / 255.0), xp.zeros_like(g))
    return lo, hi, x.reshape(rows, cols)


def rounding_offsets(shape, mode, seed, tensor_id, step):
    """u[e] of the text above for every element of a (rows, cols) matrix."""
    rows, cols = shape
    if mode == NEAREST:
        return np.full(shape, 0.5)
    if mode != STOCHASTIC:
        raise ValueError("unknown rounding %r" % (mode,))
    e = np.arange(rows * cols, dtype=np.uint64)
    o = np.unique(e >> np.uint64(3))
    words = philox4x32_10(o & np.uint64(0xFFFFFFFF), np.uint64(step & 0xFFFFFFFF),
                          np.uint64(0x80000000 | tensor_id), o >> np.uint64(32),
                          seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = np.stack(words, axis=-1).astype(np.uint32)                    # (octets, 4)
    halves = np.stack([w & np.uint32(0xFFFF), w >> np.uint32(16)], axis=-1).reshape(-1)   # element order
    return (halves[: rows * cols].astype(np.float64) / 65536.0).reshape(shape)


def quantise(w_exact, u):
    """Group-wise quantisation of the real matrix w_exact with rounding offsets u.
    Returns (Q8Weights, x) with x the real-valued code positions before rounding."""
    w_exact = np.asarray(w_exact, dtype=np.float64)
    lo, hi, x = group_positions(w_exact)
    zero = lo.astype(np.float32).astype(np.float64)                   # stored in fp32
    scale = ((hi - lo) / 255.0).astype(np.float32).astype(np.float64)
    x = np.where(np.repeat(scale, GROUP, axis=1) > 0, x, 0.0)         # a range that vanishes in fp32 counts as constant
    codes = np.minimum(255.0, np.floor(x + u)).astype(np.uint8)
    return Q8Weights(codes, scale, zero), x
