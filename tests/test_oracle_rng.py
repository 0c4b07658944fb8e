"""Pins for the oracle's random stream (no GPU).

What fixes it from outside: the published Philox known-answer vectors, exact rational
arithmetic (for the fused multiply-add emulation), libm (accuracy of the Box-Muller recipe),
torch's float32->bfloat16 conversion, and the laws a standard normal sample must obey.
"""
import hashlib
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats
import torch

from conftest import read_golden
from oracle import gauss
from oracle.philox import philox4x32_10


def test_philox_known_answers():
    kat = read_golden("philox_kat.txt")
    assert len(kat) == 3
    for name, line in kat.items():
        ins, outs = line.split("->")
        c0, c1, c2, c3, k0, k1 = (int(w, 16) for w in ins.split())
        want = [int(w, 16) for w in outs.split()]
        got = [int(v[0]) for v in philox4x32_10([c0], [c1], [c2], [c3], k0, k1)]
        assert got == want, name


def test_philox_is_a_bijection_on_a_small_slice():
    # distinct counters give distinct outputs (Philox is a permutation of the counter space)
    c0 = np.arange(20000)
    o = np.stack(philox4x32_10(c0, 0, 7, 0, 123, 456), axis=-1)
    assert len({tuple(row) for row in o.tolist()}) == len(c0)


def _round_fraction_to_f32(x):
    """Correctly round a Fraction to binary32 (ties to even) with integer arithmetic only."""
    if x == 0:
        return np.float32(0.0)
    sign = -1 if x < 0 else 1
    x = abs(x)
    # find e with 2^e <= x < 2^(e+1)
    e = x.numerator.bit_length() - x.denominator.bit_length()
    if Fraction(2) ** e > x:
        e -= 1
    if Fraction(2) ** (e + 1) <= x:
        e += 1
    assert -126 <= e <= 127
    scaled = x / Fraction(2) ** (e - 23)          # in [2^23, 2^24)
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return np.float32(sign * float(n) * 2.0 ** (e - 23))


def test_fma32_matches_exact_rational_arithmetic():
    rng = np.random.default_rng(5)
    a = rng.standard_normal(3000).astype(np.float32)
    b = rng.standard_normal(3000).astype(np.float32)
    c = (rng.standard_normal(3000) * 10.0 ** rng.integers(-8, 3, 3000)).astype(np.float32)
    # adversarial: a*b + c lands within a hair of a binary32 midpoint (double-rounding traps)
    one = np.float32(1.0)
    ulp = np.float32(2.0 ** -23)
    adv_a = np.array([1 + 2.0 ** -12, 1 + 2.0 ** -12, 3.0, 1 + 2.0 ** -23, 1 - 2.0 ** -24], np.float32)
    adv_b = np.array([2.0 ** -12, -(2.0 ** -12), 2.0 ** -25, 2.0 ** -24, 2.0 ** -24], np.float32)
    adv_c = np.array([one, one, one + ulp, one, one], np.float32)
    # a tiny product added to an exact midpoint candidate: c = 1, a*b = 2^-24 + 2^-60
    adv_a = np.append(adv_a, np.float32(2.0 ** -24 + 2.0 ** -47))
    adv_b = np.append(adv_b, np.float32(1 + 2.0 ** -13))
    adv_c = np.append(adv_c, one)
    a = np.concatenate([a, adv_a]); b = np.concatenate([b, adv_b]); c = np.concatenate([c, adv_c])
    got = gauss.fma32(a, b, c)
    for i in range(len(a)):
        exact = Fraction(float(a[i])) * Fraction(float(b[i])) + Fraction(float(c[i]))
        assert got[i] == _round_fraction_to_f32(exact), (i, a[i], b[i], c[i])


def test_fma32_differs_from_two_roundings_somewhere():
    # the emulation must not silently be round(round(a*b)+c): find a case that tells them apart
    a = np.float32(1 + 2.0 ** -12); b = np.float32(1 + 2.0 ** -12); c = np.float32(-1.0)
    fused = gauss.fma32(a, b, c)
    twice = np.float32(np.float32(a * b) + c)
    assert fused != twice
    assert float(fused) == 2.0 ** -11 + 2.0 ** -24


def _strided_words(stride):
    n = np.arange(0, 1 << 24, stride, dtype=np.uint32)
    edges = np.array([0, 1, 2, (1 << 24) - 2, (1 << 24) - 1, 1 << 23, (1 << 23) - 1,
                      0x200000, 0x1FFFFF, 0x5FFFFF, 0x600000, 0xA00000, 0xE00000, 0xDFFFFF],
                     dtype=np.uint32)
    n = np.unique(np.concatenate([n, edges]))
    return n, (n << np.uint32(8))


def test_radius_accuracy_against_libm():
    n, xa = _strided_words(61)
    rho = gauss.radius_from_word(xa).astype(np.float64)
    u1 = (n.astype(np.float64) + 1.0) / 2.0 ** 24
    ref = np.sqrt(-2.0 * np.log(u1))
    assert np.all(np.isfinite(rho)) and np.all(rho >= 0)
    assert np.max(np.abs(rho - ref)) < 6e-7
    pos = ref > 0
    assert np.max(np.abs(rho[pos] - ref[pos]) / ref[pos]) < 2.5e-7
    assert rho[n == (1 << 24) - 1][0] == 0.0            # u1 = 1 -> rho = 0
    assert rho.max() <= 5.7682                          # sqrt(2 * 24 * ln 2)


def test_cos_sin_accuracy_against_libm():
    n, xb = _strided_words(53)
    c, s = gauss.cos_sin_from_word(xb)
    th = 2.0 * np.pi * n.astype(np.float64) / 2.0 ** 24
    assert np.max(np.abs(c - np.cos(th))) < 2e-7
    assert np.max(np.abs(s - np.sin(th))) < 2e-7


def test_pair_is_radius_times_cosine_then_radius_times_sine():
    """Box-Muller's two outputs in their order: (rho cos theta, rho sin theta), against libm.  The two
    orders have the same distribution, so only this pin tells them apart."""
    n1, xa = _strided_words(59)
    n2, xb = _strided_words(67)
    k = min(len(n1), len(n2))
    n1, xa, n2, xb = n1[:k], xa[:k], n2[::-1][:k].copy(), xb[::-1][:k].copy()
    za, zb = gauss.gaussian_pair(xa, xb)
    rho = np.sqrt(-2.0 * np.log((n1.astype(np.float64) + 1.0) / 2.0 ** 24))
    th = 2.0 * np.pi * n2.astype(np.float64) / 2.0 ** 24
    assert np.max(np.abs(za - rho * np.cos(th))) < 3e-6
    assert np.max(np.abs(zb - rho * np.sin(th))) < 3e-6
    assert np.max(np.abs(za - rho * np.sin(th))) > 1.0            # and not the other way round


def test_low_byte_of_each_word_is_unused():
    xa = np.array([0x12345600, 0x123456FF], dtype=np.uint32)
    za, zb = gauss.gaussian_pair(xa, xa[::-1].copy())
    assert za[0] == za[1] and zb[0] == zb[1]


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    z = np.concatenate([rng.standard_normal(100000).astype(np.float32),
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 5.768], np.float32)])
    want = torch.from_numpy(z).to(torch.bfloat16).to(torch.float32).numpy()
    got = gauss.round_to_bf16(z)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_stream_layout_rows_quads_and_truncation():
    seed, tid, epoch = 0x1234567890ABCDEF, 5, 3
    r, m = 3, 10                                         # ceil(m/4) = 3 quads per row
    z = gauss.projection(seed, tid, epoch, r, m, bf16=False)
    assert z.shape == (r, m)
    # element P[1, 6] comes from counter q = 1*3 + 1, output words 2 (radius) and 3 (angle): cos branch
    x = philox4x32_10([4], [epoch], [tid], [0], seed & 0xFFFFFFFF, seed >> 32)
    zc, zd = gauss.gaussian_pair(x[2], x[3])
    za, zb = gauss.gaussian_pair(x[0], x[1])
    assert z[1, 4] == za[0] and z[1, 5] == zb[0] and z[1, 6] == zc[0] and z[1, 7] == zd[0]
    # a wider matrix with the same number of quads per row shares its leading columns
    z12 = gauss.projection(seed, tid, epoch, r, 12, bf16=False)
    assert np.array_equal(z12[:, :m], z)
    # other tensors / epochs / seeds give other streams
    for other in (gauss.projection(seed, tid + 1, epoch, r, m, False),
                  gauss.projection(seed, tid, epoch + 1, r, m, False),
                  gauss.projection(seed + 1, tid, epoch, r, m, False),
                  gauss.projection(seed + (1 << 32), tid, epoch, r, m, False)):
        assert not np.any(other == z)


def test_gaussian_moments_and_ks():
    z = gauss.projection(2024, 1, 0, 64, 32768, bf16=False).ravel()      # 2.1e6 samples
    N = z.size
    assert abs(z.mean()) < 5.0 / np.sqrt(N)
    assert abs(z.var() - 1.0) < 5.0 * np.sqrt(2.0 / N)
    assert abs(np.mean(z ** 3)) < 5.0 * np.sqrt(15.0 / N)
    assert abs(np.mean(z ** 4) - 3.0) < 5.0 * np.sqrt(96.0 / N)
    assert np.abs(z).max() <= 5.7682
    ks = scipy.stats.kstest(z[:400000], "norm")
    assert ks.pvalue > 1e-3
    # the two Box-Muller branches and neighbouring elements are uncorrelated
    zz = z.reshape(-1, 4)
    for i in range(4):
        for j in range(i + 1, 4):
            assert abs(np.mean(zz[:, i] * zz[:, j])) < 5.0 / np.sqrt(zz.shape[0])


def test_streams_of_different_tensors_and_epochs_are_uncorrelated():
    a = gauss.projection(9, 0, 0, 16, 8192, False).ravel()
    for tid, ep in ((1, 0), (0, 1)):
        b = gauss.projection(9, tid, ep, 16, 8192, False).ravel()
        assert abs(np.mean(a * b)) < 5.0 / np.sqrt(a.size)


def _digest(arr):
    return hashlib.sha256(np.ascontiguousarray(arr).view(np.uint32).tobytes()).hexdigest()


def test_recipe_digest_subset_matches_golden():
    """The stored digests (written by tests/golden/make_gauss_digests.py from the oracle alone)
    still describe the oracle: recompute the strided subset."""
    g = read_golden("gauss_recipe_digests.txt")
    stride = int(g["subset_stride"])
    n = np.arange(0, 1 << 24, stride, dtype=np.uint32) << np.uint32(8)
    assert _digest(gauss.radius_from_word(n)) == g["subset_radius_sha256"]
    c, s = gauss.cos_sin_from_word(n)
    assert _digest(c) == g["subset_cos_sha256"]
    assert _digest(s) == g["subset_sin_sha256"]
