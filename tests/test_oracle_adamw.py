"""Pins for the oracle's element-wise AdamW (no GPU): an independent library implementation,
closed forms for special gradients, the decoupled decay, and the literal Eq. 1 of Section 3.1."""
import math

import numpy as np
import pytest
import torch

from oracle import adamw


def _run(cfg, W0, grads, lr):
    W = np.array(W0, dtype=np.float64)
    st = adamw.init_state(W.size)
    for t, g in enumerate(grads, start=1):
        adamw.step(cfg, st, W, g, t, lr)
    return W, st


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_matches_torch_adamw_in_float64(wd):
    """torch.optim.AdamW (decoupled decay, bias correction, eps outside the square root) is an
    independent implementation of the same textbook rule."""
    rng = np.random.default_rng(5)
    W0 = rng.normal(size=257)
    grads = [rng.normal(size=257) * 10.0 ** rng.integers(-4, 1) for _ in range(12)]
    cfg = adamw.Config(beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=wd)
    W, st = _run(cfg, W0, grads, 3e-3)
    p = torch.nn.Parameter(torch.tensor(W0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(st.M, opt.state[p]["exp_avg"].numpy(), rtol=1e-12, atol=0)
    np.testing.assert_allclose(st.V, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-12, atol=0)


def test_constant_gradient_moves_by_lr_sign_each_step():
    """With a constant gradient the bias-corrected moments are exactly g and g^2 at every step,
    so (eps = 0) each step moves every element by lr in the direction of -sign(g)."""
    g = np.array([3.0, -0.25, 1e-6, -7e3])
    cfg = adamw.Config(beta1=0.9, beta2=0.999, eps=0.0)
    W, st = _run(cfg, np.zeros(4), [g] * 9, 0.01)
    np.testing.assert_allclose(W, -9 * 0.01 * np.sign(g), rtol=1e-12)
    t = 9
    np.testing.assert_allclose(st.M, (1 - 0.9 ** t) * g, rtol=1e-12)
    np.testing.assert_allclose(st.V, (1 - 0.999 ** t) * g * g, rtol=1e-12)


def test_zero_gradient_leaves_only_the_decoupled_decay():
    """G = 0: moments stay 0, 0 / (0 + eps) = 0, and W shrinks by (1 - lr lambda) per step,
    untouched by the adaptive scaling (that is what "decoupled" means)."""
    W0 = np.array([1.0, -2.0, 0.5])
    cfg = adamw.Config(weight_decay=0.2, eps=1e-8)
    W, st = _run(cfg, W0, [np.zeros(3)] * 5, 0.1)
    np.testing.assert_allclose(W, W0 * (1 - 0.1 * 0.2) ** 5, rtol=1e-13)
    assert not st.M.any() and not st.V.any()


def test_decay_uses_the_old_weight_and_adds_to_the_adam_term():
    g = np.array([2.0])
    cfg = adamw.Config(beta1=0.9, beta2=0.999, eps=0.0, weight_decay=0.5)
    W, _ = _run(cfg, np.array([4.0]), [g], 0.1)
    assert W[0] == pytest.approx(4.0 - 0.1 * 1.0 - 0.1 * 0.5 * 4.0, rel=1e-14)


def test_without_bias_correction_is_equation_one_literally():
    g = np.array([0.3, -1.5])
    b1, b2, eps, lr = 0.8, 0.99, 1e-3, 0.05
    cfg = adamw.Config(beta1=b1, beta2=b2, eps=eps, bias_correction=False)
    W, st = _run(cfg, np.zeros(2), [g], lr)
    expect = -lr * ((1 - b1) * g) / (np.sqrt((1 - b2) * g * g) + eps)
    np.testing.assert_allclose(W, expect, rtol=1e-14)
    # second step by hand
    g2 = np.array([-0.1, 0.7])
    adamw.step(cfg, st, W, g2, 2, lr)
    M2 = b1 * (1 - b1) * g + (1 - b1) * g2
    V2 = b2 * (1 - b2) * g * g + (1 - b2) * g2 * g2
    np.testing.assert_allclose(W, expect - lr * M2 / (np.sqrt(V2) + eps), rtol=1e-14)


def test_eps_sits_outside_the_square_root_and_after_the_bias_correction():
    g = np.array([1e-4])
    cfg = adamw.Config(beta1=0.9, beta2=0.999, eps=1e-4)
    W, _ = _run(cfg, np.zeros(1), [g], 1.0)
    # m^ = g, v^ = g^2: update g / (|g| + eps) = 1/2; eps inside the root would give 1/sqrt(1 + 1e4)...
    assert W[0] == pytest.approx(-0.5, rel=1e-12)


def test_rejects_bad_arguments():
    st = adamw.init_state(3)
    with pytest.raises(ValueError):
        adamw.step(adamw.Config(), st, np.zeros(3), np.zeros(3), 0, 0.1)
    with pytest.raises(ValueError):
        adamw.step(adamw.Config(), st, np.zeros(4), np.zeros(4), 1, 0.1)
    with pytest.raises(ValueError):
        adamw.step(adamw.Config(), st, np.zeros(3, dtype=np.float32), np.zeros(3), 1, 0.1)


def test_bfloat16_storage_rounds_on_store_and_computes_from_what_is_stored():
    """store_dtype="bf16" by hand on one element with beta = 0 (so M = g, V = g^2 exactly before
    rounding): g = 1 + 2^-10 is not a bfloat16 number (spacing 2^-7 above 1), so M is stored as 1 and
    V = g^2 = 1 + 2^-9 + 2^-20 as 1; the update uses the STORED moments, 1 / (sqrt(1) + 0) = 1, not
    g / |g|; the new weight 1 - 2^-9 - 2^-10 is 3/4 of the way from 1 down to the next bfloat16
    below it (spacing 2^-8 there) and is stored as 1 - 2^-8."""
    cfg = adamw.Config(beta1=0.0, beta2=0.0, eps=0.0, bias_correction=False, store_dtype="bf16")
    st = adamw.init_state(1)
    W = np.array([1.0])
    g = np.array([1.0 + 2.0 ** -10])
    u = adamw.step(cfg, st, W, g, 1, 2.0 ** -9 + 2.0 ** -10)
    assert st.M_exact[0] == g[0] and st.M[0] == 1.0
    assert st.V_exact[0] == g[0] ** 2 and st.V[0] == 1.0
    assert u[0] == 1.0
    assert st.W_exact[0] == 1.0 - 2.0 ** -9 - 2.0 ** -10 and W[0] == 1.0 - 2.0 ** -8
    # the same step kept in fp32 (fp64 here) rounds nothing
    cfg32 = adamw.Config(beta1=0.0, beta2=0.0, eps=0.0, bias_correction=False)
    st, W = adamw.init_state(1), np.array([1.0])
    adamw.step(cfg32, st, W, g, 1, 2.0 ** -9 + 2.0 ** -10)
    assert st.M[0] == g[0] and W[0] == 1.0 - 2.0 ** -9 - 2.0 ** -10


def test_bfloat16_storage_stays_within_half_an_ulp_per_step_and_adopts_roundings():
    rng = np.random.default_rng(17)
    cfg = adamw.Config(weight_decay=0.1, store_dtype="bf16")
    ref = adamw.Config(weight_decay=0.1)
    W = rng.normal(size=300)
    W = np.asarray(torch.tensor(W).to(torch.bfloat16).double())       # starts as bfloat16 numbers
    st = adamw.init_state(300)
    for t in range(1, 6):
        g = rng.normal(size=300) * 1e-2
        Wr, sr = W.copy(), adamw.init_state(300)
        sr.M, sr.V = st.M.copy(), st.V.copy()
        adamw.step(ref, sr, Wr, g, t, 1e-2)                           # the same step without rounding
        adamw.step(cfg, st, W, g, t, 1e-2)
        for got, exact in ((st.M, sr.M), (st.V, sr.V)):
            assert np.all(np.abs(got - exact) <= np.abs(exact) * 2.0 ** -8)      # half a unit in the last of 8 bits
            assert np.array_equal(np.asarray(torch.tensor(got).to(torch.bfloat16).double()), got)
        assert np.array_equal(np.asarray(torch.tensor(W).to(torch.bfloat16).double()), W)
        assert np.all(np.abs(W - st.W_exact) <= np.abs(st.W_exact) * 2.0 ** -8)
    # adopt_moments: what the hook returns is what is stored and what the update is formed from
    st2, W2 = adamw.init_state(2), np.zeros(2)
    u = adamw.step(adamw.Config(beta1=0.0, beta2=0.0, eps=0.0, bias_correction=False), st2, W2, np.array([3.0, -4.0]), 1, 1.0,
                   adopt_moments=lambda M, V: (np.array([6.0, -4.0]), V))
    assert st2.M.tolist() == [6.0, -4.0] and u.tolist() == [2.0, -1.0]
