"""Philox words -> N(0,1) variates -> the projection matrix P (oracle side).

Test infrastructure only (see the package docstring).

The paper draws P from a seeded Gaussian, variance 1/r, and re-generates it from the seed
instead of storing it (Algorithm 1; Section 4.1 "Generating random projection matrix";
Theorem A.1 states the variance 1/r).  For the GPU library and this oracle to agree on P to
the last bit, the map from random words to a Gaussian is fixed here as an explicit sequence
of IEEE-754 binary32 operations -- exact integer<->float conversions, round-to-nearest
multiply / add / subtract, fused multiply-add (one rounding), correctly rounded square root --
with frozen polynomial constants.  That sequence (a Box-Muller transform with its own log and
sin/cos range reductions) *is* the definition; its accuracy (a few 1e-7) is checked against
libm in the tests, but the bits are the contract.

Layout of the stream (for one tensor and one refresh epoch):
  key      = (seed & 0xffffffff, seed >> 32)
  counter  = (q_lo, epoch, tensor_id, q_hi) with q = kk * ceil(m/4) + floor(i/4) for the element
             P[kk, i]; the four output words x0..x3 give the elements i = 4*floor(i/4) + 0..3:
             (x0, x1) -> a Box-Muller pair (cos branch, sin branch), (x2, x3) -> the next pair.
  P[kk, i] = z, rounded to bfloat16 (nearest-even) when the gradient is bfloat16.
The 1/sqrt(r) of the variance is NOT folded into P: it multiplies the product P.G afterwards.
"""
import numpy as np

from .philox import philox4x32_10

f32 = np.float32
u32 = np.uint32

# ---- frozen constants of the recipe (binary32, written as exact hex floats) -------------
# -ln(u) = -(k*ln2 + log1p(t)),  log1p(t) ~ t + t^2 * q(t),  t in [sqrt(1/2)-1, sqrt(2)-1]
_LOGQ = [f32(float.fromhex(h)) for h in (
    "-0x1.fffff4p-2", "0x1.5556e6p-2", "-0x1.0006c4p-2", "0x1.98da68p-3",
    "-0x1.52fb66p-3", "0x1.30cecep-3", "-0x1.2773cap-3", "0x1.6fd5ap-4")]
_LN2_HI = f32(float.fromhex("0x1.62e4p-1"))      # 16 significant bits: k*LN2_HI is exact
_LN2_LO = f32(float.fromhex("0x1.7f7d1cp-20"))
_SQRT2_MANT = 0x3504F3                            # mantissa field of sqrt(2) in binary32
# sin(pi/4 x) ~ x * S(x^2),  cos(pi/4 x) ~ C(x^2),  x in [-1, 1)
_SIN = [f32(float.fromhex(h)) for h in (
    "0x1.921fb6p-1", "-0x1.4abbbap-4", "0x1.465ec6p-9", "-0x1.2d9bb8p-15")]
_COS = [f32(float.fromhex(h)) for h in (
    "0x1p+0", "-0x1.3bd392p-2", "0x1.03af5cp-6", "-0x1.4e5ed6p-12")]


def fma32(a, b, c):
    """IEEE-754 binary32 fused multiply-add round(a*b + c) with a single rounding.

    The product of two binary32 values is exact in binary64.  The sum p + c is formed in
    binary64 and, when inexact, replaced by its round-to-odd value (the neighbour with an odd
    significand); rounding that to binary32 then gives the correctly rounded result because
    binary64 carries more than 2*24+2 bits (Boldo & Melquiond, "Emulation of a FMA and
    correctly rounded sums", 2008).  Pinned against exact rational arithmetic in the tests.
    """
    a = np.asarray(a, dtype=f32).astype(np.float64)
    b = np.asarray(b, dtype=f32).astype(np.float64)
    c = np.asarray(c, dtype=f32).astype(np.float64)
    p = a * b                                   # exact
    s = p + c                                   # rounded to 53 bits
    # exact rounding error of s (Knuth two-sum): true value = s + e
    bb = s - p
    e = (p - (s - bb)) + (c - bb)
    s_bits = np.asarray(s).view(np.int64)
    even = (s_bits & 1) == 0
    toward = np.where(e > 0, np.inf, -np.inf)
    nxt = np.nextafter(s, toward)
    s_odd = np.where((e != 0) & even, nxt, s)
    return s_odd.astype(f32)


def _horner(coeffs, x):
    acc = np.full(x.shape, coeffs[-1], dtype=f32)
    for cf in coeffs[-2::-1]:
        acc = fma32(acc, x, cf)
    return acc


def radius_from_word(xa):
    """rho = sqrt(-2 ln u1) with u1 = ((xa >> 8) + 1) / 2^24 in (0, 1]  (binary32 recipe)."""
    xa = np.asarray(xa, dtype=u32)
    n1 = (xa >> u32(8)) + u32(1)                       # 1 .. 2^24, exact in binary32
    f = n1.astype(f32)
    bits = f.view(u32)
    e = (bits >> u32(23)).astype(np.int32) - np.int32(127)
    mbits = bits & u32(0x7FFFFF)
    big = mbits > u32(_SQRT2_MANT)                     # mantissa above sqrt(2): halve it
    mant = (mbits | np.where(big, u32(0x3F000000), u32(0x3F800000))).view(f32)
    k = e + big.astype(np.int32) - np.int32(24)        # u1 = mant * 2^k, mant in [sqrt(1/2), sqrt(2)]
    t = mant - f32(1.0)                                # exact (Sterbenz)
    q = _horner(_LOGQ, t)
    t2 = t * t
    lp = fma32(t2, q, t)                               # log(mant)
    kf = k.astype(f32)
    w = fma32(kf, _LN2_HI, fma32(kf, _LN2_LO, lp))     # ln(u1) <= 0
    return np.sqrt(f32(-2.0) * w)                      # *(-2) is exact; sqrt correctly rounded


def cos_sin_from_word(xb):
    """(cos, sin) of theta = 2 pi u2, u2 = (xb >> 8) / 2^24 in [0, 1)  (binary32 recipe).

    theta = kq*pi/2 + (pi/4) x with kq the nearest quarter turn and x in [-1, 1) exact.
    """
    xb = np.asarray(xb, dtype=u32)
    n2 = xb >> u32(8)
    kq = (n2 + u32(0x200000)) >> u32(22)               # 0 .. 4
    fi = n2.astype(np.int32) - (kq << u32(22)).astype(np.int32)   # -2^21 .. 2^21-1
    x = fi.astype(f32) * f32(2.0 ** -21)               # exact
    x2 = x * x
    sn = _horner(_SIN, x2) * x
    cs = _horner(_COS, x2)
    quad = kq & u32(3)
    c = np.select([quad == 0, quad == 1, quad == 2], [cs, -sn, -cs], default=sn)
    s = np.select([quad == 0, quad == 1, quad == 2], [sn, cs, -sn], default=-cs)
    return c.astype(f32), s.astype(f32)


def gaussian_pair(xa, xb):
    """Box-Muller: words (xa, xb) -> (rho*cos(theta), rho*sin(theta)), both binary32."""
    rho = radius_from_word(xa)
    c, s = cos_sin_from_word(xb)
    return rho * c, rho * s


def round_to_bf16(z):
    """Round binary32 to the nearest bfloat16 (ties to even); result kept as binary32."""
    bits = np.asarray(z, dtype=f32).view(u32).astype(np.uint64)
    bits = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return bits.astype(u32).view(f32)


def projection_words(seed, tensor_id, epoch, r, m):
    """The raw Philox words behind P: uint32 array of shape (r, ceil(m/4), 4)."""
    mq = (m + 3) // 4
    q = (np.arange(r, dtype=np.uint64)[:, None] * np.uint64(mq)
         + np.arange(mq, dtype=np.uint64)[None, :])
    x = philox4x32_10(q & np.uint64(0xFFFFFFFF), np.uint64(epoch), np.uint64(tensor_id),
                      q >> np.uint64(32), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(x, axis=-1)


def projection(seed, tensor_id, epoch, r, m, bf16):
    """Unit-variance projection matrix z of shape (r, m) as float64.

    Algorithm 1 draws P ~ N(0, 1/r); P = z / sqrt(r), and the division is applied by the
    caller to the product so that the bfloat16 rounding acts on z.
    """
    w = projection_words(seed, tensor_id, epoch, r, m)
    za, zb = gaussian_pair(w[..., 0], w[..., 1])
    zc, zd = gaussian_pair(w[..., 2], w[..., 3])
    z = np.stack([za, zb, zc, zd], axis=-1).reshape(r, -1)[:, :m]
    if bf16:
        z = round_to_bf16(z)
    return z.astype(np.float64)
