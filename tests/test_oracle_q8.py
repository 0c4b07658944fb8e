"""Pins for the oracle's group-wise 8-bit weight format (no GPU): error bounds of both rounding
modes, exactness at the ends of a group's range, degenerate groups, the layout of the rounding
offsets over the Philox words, unbiasedness of stochastic rounding, and the step on such weights."""
import numpy as np
import pytest

from oracle import apollo, q8
from oracle.philox import philox4x32_10


def _rand_w(rng, rows=3, cols=256, scale=0.02):
    return rng.normal(size=(rows, cols)) * scale


@pytest.mark.parametrize("mode", [q8.NEAREST, q8.STOCHASTIC])
def test_quantisation_error_is_bounded_by_the_code_step(mode):
    rng = np.random.default_rng(1)
    w = _rand_w(rng)
    u = q8.rounding_offsets(w.shape, mode, seed=5, tensor_id=2, step=7)
    qw, x = q8.quantise(w, u)
    assert qw.codes.dtype == np.uint8 and qw.codes.shape == w.shape and qw.scale.shape == (3, 2)
    err = np.abs(qw.dequantise() - w) / np.repeat(qw.scale, 128, axis=1)
    assert err.max() <= (0.5 if mode == q8.NEAREST else 1.0) + 1e-4
    assert x.min() == 0.0 and abs(x.max() - 255.0) < 1e-9
    # the ends of every group's range are hit exactly: code 0 at the minimum, 255 at the maximum
    g = w.reshape(3, 2, 128)
    c = qw.codes.reshape(3, 2, 128)
    assert np.all(np.take_along_axis(c, g.argmin(axis=2)[..., None], 2) == 0)
    assert np.all(np.take_along_axis(c, g.argmax(axis=2)[..., None], 2) == 255)
    assert np.array_equal(qw.zero, g.min(axis=2).astype(np.float32).astype(np.float64))
    assert np.allclose(qw.scale, (g.max(axis=2) - g.min(axis=2)) / 255.0, rtol=1e-6)


def test_constant_group_and_row_length_check():
    w = np.full((1, 128), 0.375)
    qw, x = q8.quantise(w, q8.rounding_offsets(w.shape, q8.NEAREST, 0, 0, 1))
    assert not qw.codes.any() and qw.scale[0, 0] == 0.0 and qw.zero[0, 0] == 0.375 and not x.any()
    assert np.array_equal(qw.dequantise(), w)
    with pytest.raises(ValueError):
        q8.Q8Weights(np.zeros((2, 100), np.uint8), np.zeros((2, 1)), np.zeros((2, 1)))


def test_nearest_requantisation_of_stored_weights_is_the_identity_when_the_range_is_full():
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 256, size=(2, 256)).astype(np.uint8)
    codes[:, 0] = 0
    codes[:, 1] = 255
    codes[:, 128] = 0
    codes[:, 129] = 255
    qw = q8.Q8Weights(codes, np.full((2, 2), 2.0 ** -10), np.array([[-0.1, 0.2], [0.0, -3.0]], dtype=np.float32))
    again, _ = q8.quantise(qw.dequantise(), np.full(codes.shape, 0.5))
    assert np.array_equal(again.codes, codes)
    assert np.allclose(again.scale, qw.scale, rtol=1e-6) and np.allclose(again.zero, qw.zero, rtol=1e-7, atol=1e-9)


def test_rounding_offsets_layout_over_the_philox_words():
    seed, tid, step = 0x1234567890ABCDEF, 9, 41
    u = q8.rounding_offsets((2, 128), q8.STOCHASTIC, seed, tid, step)
    assert np.all(u >= 0) and np.all(u < 1) and np.array_equal(u * 65536, np.round(u * 65536))
    for e in (0, 1, 6, 7, 8, 133, 255):
        o, k, hi = e // 8, (e % 8) // 2, e % 2
        words = philox4x32_10(o, step, 0x80000000 | tid, 0, seed & 0xFFFFFFFF, seed >> 32)
        half = (int(words[k]) >> 16) if hi else (int(words[k]) & 0xFFFF)
        assert u.reshape(-1)[e] == half / 65536.0
    # every argument matters
    for other in (q8.rounding_offsets((2, 128), q8.STOCHASTIC, seed + 1, tid, step),
                  q8.rounding_offsets((2, 128), q8.STOCHASTIC, seed, tid + 1, step),
                  q8.rounding_offsets((2, 128), q8.STOCHASTIC, seed, tid, step + 1)):
        assert np.mean(other == u) < 0.01
    assert np.all(q8.rounding_offsets((1, 128), q8.NEAREST, seed, tid, step) == 0.5)
    with pytest.raises(ValueError):
        q8.rounding_offsets((1, 128), "up", seed, tid, step)


def test_stochastic_rounding_is_unbiased_and_rounds_up_with_probability_frac_x():
    # a group whose range is pinned by 0 and 255 and whose other elements all sit at code 100.25
    w = np.full((64, 128), 100.25)
    w[:, 0], w[:, 1] = 0.0, 255.0
    ups = []
    for step in range(1, 21):
        qw, x = q8.quantise(w, q8.rounding_offsets(w.shape, q8.STOCHASTIC, 77, 3, step))
        assert np.allclose(x[:, 2:], 100.25)
        ups.append(np.mean(qw.codes[:, 2:] == 101))
        assert np.all((qw.codes[:, 2:] == 100) | (qw.codes[:, 2:] == 101))
    n = 20 * 64 * 126
    assert abs(np.mean(ups) - 0.25) < 4 * np.sqrt(0.25 * 0.75 / n)
    # general weights: mean signed error of the stored value, in code steps, is zero within 4 sigma
    rng = np.random.default_rng(3)
    w = _rand_w(rng, rows=64, cols=512)
    qw, _ = q8.quantise(w, q8.rounding_offsets(w.shape, q8.STOCHASTIC, 78, 0, 1))
    e = (qw.dequantise() - w) / np.repeat(qw.scale, 128, axis=1)
    assert abs(e.mean()) < 4 * np.sqrt(1.0 / 6.0 / e.size) + 1e-6      # var of the SR error <= 1/4, ~1/6 for uniform frac


def test_step_on_q8_weights_by_hand_and_why_stochastic_rounding_is_there():
    rng = np.random.default_rng(4)
    w0 = _rand_w(rng, rows=1, cols=128)
    qw0, _ = q8.quantise(w0, np.full(w0.shape, 0.5))
    G = np.ones((1, 128))
    P = np.array([[1.0]])
    # beta = 0, eps = 0: R~ = sign(R), s = 1 / |R| * 1 ... with R = G (rank 1, one row): s_j = 1 / |G_j| = 1
    for mode in (q8.NEAREST, q8.STOCHASTIC):
        cfg = apollo.Config(rank=1, beta1=0.0, beta2=0.0, eps=0.0, nl_gamma=0.0, weight_dtype="q8",
                            weight_rounding=mode, seed=11)
        W = q8.Q8Weights(qw0.codes.copy(), qw0.scale.copy(), qw0.zero.copy())
        st = apollo.init_state(cfg, 1, 128)
        step_size = 0.2 * float(qw0.scale[0, 0])          # a fifth of a code step per optimizer step
        info = apollo.step(cfg, st, W, G, 1, step_size, P=P)
        assert np.allclose(info["W_exact"], qw0.dequantise() - step_size, rtol=0, atol=1e-15)
        assert np.array_equal(W.codes, np.minimum(255, np.floor(info["q8_x"] + info["q8_u"])).astype(np.uint8))
        if mode == q8.NEAREST:
            # every element moves by the same amount: the range, and so every code, stays as it was,
            # and only the group's zero point carries the update
            assert np.array_equal(W.codes, qw0.codes)
            assert W.zero[0, 0] == pytest.approx(qw0.zero[0, 0] - step_size, rel=1e-6)
    # a gradient on ONE element, smaller than half a code step: nearest rounding never moves it,
    # stochastic rounding moves it by the right amount on average
    j = int(np.argsort(w0[0])[64])         # an element in the middle of the group's range
    assert 0 < qw0.codes[0, j] < 255
    G1 = np.full((1, 128), 1e-30)          # (not exactly zero elsewhere: eps = 0 would give 0 / 0)
    G1[0, j] = 1.0
    # (tensor-wise factor: s = ||sign(R)|| / ||R|| = sqrt(128), the same for every element, so only
    # element j, whose gradient is not negligible, moves: by lr * sqrt(128))
    moved = {}
    for mode in (q8.NEAREST, q8.STOCHASTIC):
        cfg = apollo.Config(rank=1, mode=apollo.TENSOR, beta1=0.0, beta2=0.0, eps=0.0, nl_gamma=0.0,
                            weight_dtype="q8", weight_rounding=mode, seed=12)
        total = 0.0
        for trial in range(200):
            W = q8.Q8Weights(qw0.codes.copy(), qw0.scale.copy(), qw0.zero.copy())
            st = apollo.init_state(cfg, 1, 128)
            before = W.dequantise()[0, j]
            apollo.step(cfg, st, W, G1, 1 + trial, 0.3 * float(qw0.scale[0, 0]) / np.sqrt(128.0), P=P)
            total += before - W.dequantise()[0, j]
        moved[mode] = total / 200 / float(qw0.scale[0, 0])
    assert moved[q8.NEAREST] == pytest.approx(0.0, abs=1e-6)
    assert moved[q8.STOCHASTIC] == pytest.approx(0.3, abs=4 * np.sqrt(0.3 * 0.7 / 200))


def test_step_draws_its_rounding_offsets_for_its_own_tensor_and_step():
    """The offsets a step uses are the stream's values for (seed, tensor index, step number): the
    Philox words are computed here directly, for two tensors and two steps, and must differ between
    them (a step that passed another tensor's index or a shifted step number would reuse offsets)."""
    rng = np.random.default_rng(6)
    w0 = _rand_w(rng, rows=2, cols=128)
    qw0, _ = q8.quantise(w0, np.full(w0.shape, 0.5))
    G = rng.normal(size=(2, 128))
    seen = []
    for tensor_id, t in ((3, 5), (3, 4), (0, 5)):
        cfg = apollo.Config(rank=1, nl_gamma=0.0, weight_dtype="q8", weight_rounding=q8.STOCHASTIC, seed=77)
        W = q8.Q8Weights(qw0.codes.copy(), qw0.scale.copy(), qw0.zero.copy())
        info = apollo.step(cfg, apollo.init_state(cfg, 2, 128), W, G, t, 1e-3, tensor_id=tensor_id)
        o = np.arange(2 * 128 // 8, dtype=np.uint64)
        words = np.stack(philox4x32_10(o, np.uint64(t), np.uint64(0x80000000 + tensor_id), np.uint64(0) * o, 77, 0), axis=-1)
        u = np.stack([words & 0xFFFF, words >> 16], axis=-1).reshape(2, 128) / 65536.0
        assert np.array_equal(info["q8_u"], u)
        seen.append(u)
    assert not np.array_equal(seen[0], seen[1]) and not np.array_equal(seen[0], seen[2])
