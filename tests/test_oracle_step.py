"""Pins for the oracle's optimizer step (no GPU): brute force on tiny tensors, closed forms,
special cases that reduce to textbook Adam, the identities used in the paper's appendix,
the Johnson-Lindenstrauss law of Theorem A.1, and the numbers the paper prints."""
import copy
import math

import numpy as np
import pytest

from conftest import read_golden
from oracle import apollo, gauss

F32 = lambda v: float(np.float32(v))


def _cfg(**kw):
    base = dict(rank=2, mode=apollo.CHANNEL, seed=77, beta1=0.9, beta2=0.999, eps=1e-8,
                scale=1.0, weight_decay=0.0, nl_gamma=1.01, refresh_interval=200)
    base.update(kw)
    return apollo.Config(**base)


# ----------------------------------------------------------------------------- brute force
def _brute_force_run(cfg, W, grads, lr, tensor_id, bf16):
    """Scalar triple loops, lists of Python floats; written from Algorithm 1 independently of
    the vectorised oracle (only the random matrix z comes from oracle.gauss, pinned elsewhere)."""
    rows, cols = len(W), len(W[0])
    left = rows <= cols if cfg.side == "auto" else cfg.side == "left"
    m, n = (rows, cols) if left else (cols, rows)
    r = cfg.rank
    M = [[0.0] * n for _ in range(r)]
    V = [[0.0] * n for _ in range(r)]
    prev = 0.0
    W = [row[:] for row in W]
    for t, G in enumerate(grads, start=1):
        g = (lambda i, j: G[i][j]) if left else (lambda i, j: G[j][i])
        z = gauss.projection(cfg.seed, tensor_id, (t - 1) // cfg.refresh_interval, r, m, bf16)
        s = [0.0] * n
        a_all = b_all = 0.0
        a_col = [0.0] * n
        b_col = [0.0] * n
        for j in range(n):
            for k in range(r):
                acc = 0.0
                for i in range(m):
                    acc += float(z[k, i]) * g(i, j)
                Rkj = acc / math.sqrt(r)
                M[k][j] = cfg.beta1 * M[k][j] + (1 - cfg.beta1) * Rkj
                V[k][j] = cfg.beta2 * V[k][j] + (1 - cfg.beta2) * Rkj * Rkj
                mh = M[k][j] / (1 - cfg.beta1 ** t)
                vh = V[k][j] / (1 - cfg.beta2 ** t)
                rt = mh / (math.sqrt(vh) + cfg.eps)
                a_col[j] += rt * rt
                b_col[j] += Rkj * Rkj
            a_all += a_col[j]
            b_all += b_col[j]
        for j in range(n):
            if cfg.mode == apollo.CHANNEL:
                s[j] = math.sqrt(a_col[j]) / math.sqrt(b_col[j]) if b_col[j] > 0 else 0.0
            else:
                s[j] = math.sqrt(a_all) / math.sqrt(b_all) if b_all > 0 else 0.0
        sq = 0.0
        for j in range(n):
            for i in range(m):
                sq += (cfg.scale * s[j] * g(i, j)) ** 2
        norm = math.sqrt(sq)
        c = 1.0
        if cfg.nl_gamma > 0 and prev > 0 and norm / prev > cfg.nl_gamma:
            c = cfg.nl_gamma * prev / norm
            norm = cfg.nl_gamma * prev
        prev = norm
        Wn = [row[:] for row in W]
        for j in range(n):
            for i in range(m):
                (ri, ci) = (i, j) if left else (j, i)
                Wn[ri][ci] = W[ri][ci] - lr * cfg.scale * c * s[j] * g(i, j) - lr * cfg.weight_decay * W[ri][ci]
        W = Wn
    return np.array(W), np.array(M), np.array(V), prev


@pytest.mark.parametrize("rows,cols,mode,rank,bf16", [
    (5, 8, apollo.CHANNEL, 3, False),
    (8, 5, apollo.CHANNEL, 4, True),      # more rows than columns: projected along columns
    (6, 6, apollo.TENSOR, 1, False),
    (7, 4, apollo.TENSOR, 2, True),
])
def test_step_matches_brute_force(rows, cols, mode, rank, bf16):
    rng = np.random.default_rng(rows * 100 + cols)
    cfg = _cfg(rank=rank, mode=mode, refresh_interval=3, weight_decay=0.05,
               scale=1.0 if mode == apollo.CHANNEL else math.sqrt(128.0))
    W0 = rng.standard_normal((rows, cols)) * 0.02
    grads = [rng.standard_normal((rows, cols)) * 1e-2 for _ in range(6)]
    grads[4] = grads[3] * 2.0                         # a repeated direction makes ||R~|| grow again:
    grads[5] = grads[3] * 4.0                         # the limiter is hit at step 5 or 6
    grads[1][:, 2] = 0.0
    grads[1][2, :] = 0.0                              # a zero channel whichever side is projected
    if bf16:
        grads = [gauss.round_to_bf16(g.astype(np.float32)).astype(np.float64) for g in grads]
    st = apollo.init_state(cfg, rows, cols)
    W = W0.copy()
    hit = False
    for t, G in enumerate(grads, start=1):
        info = apollo.step(cfg, st, W, G, t, lr=1e-2, tensor_id=4, grad_is_bf16=bf16)
        hit |= info["c"] < 1.0
    assert hit, "the limiter case was not exercised"
    Wb, Mb, Vb, prevb = _brute_force_run(cfg, W0.tolist(), [g.tolist() for g in grads], 1e-2, 4, bf16)
    np.testing.assert_allclose(W, Wb, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(st.M, Mb, rtol=1e-11, atol=1e-18)
    np.testing.assert_allclose(st.V, Vb, rtol=1e-11, atol=1e-24)
    assert st.prev_norm == pytest.approx(prevb, rel=1e-12)


# ----------------------------------------------------------------------------- closed forms
def test_rank1_mini_by_hand():
    # 2 x 3 gradient, hand-set p = (0.5, -1):  R = p G = (-3.5, -4, -4.5)
    G = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    W = np.zeros((2, 3))
    cfg = _cfg(rank=1, mode=apollo.TENSOR, eps=0.0, scale=math.sqrt(128.0))
    st = apollo.init_state(cfg, 2, 3)
    info = apollo.step(cfg, st, W, G, 1, lr=0.01, P=np.array([[0.5, -1.0]]))
    np.testing.assert_allclose(info["R"], [[-3.5, -4.0, -4.5]])
    # step 1 with bias correction: M^ = R, V^ = R^2, so R~ = sign(R): ||R~|| = sqrt(3), ||R|| = sqrt(48.5)
    s = math.sqrt(3.0 / 48.5)
    np.testing.assert_allclose(info["s"], [s, s, s], rtol=1e-14)
    np.testing.assert_allclose(W, -0.01 * math.sqrt(128.0) * s * G, rtol=1e-13)
    # the stored norm is || alpha s G ||_F
    assert st.prev_norm == pytest.approx(math.sqrt(128.0) * s * math.sqrt(91.0), rel=1e-13)
    # raw moments (not bias corrected) are what is stored
    np.testing.assert_allclose(st.M, 0.1 * info["R"], rtol=1e-13)
    np.testing.assert_allclose(st.V, 0.001 * info["R"] ** 2, rtol=1e-11)


@pytest.mark.parametrize("mode", [apollo.CHANNEL, apollo.TENSOR])
def test_constant_gradient_closed_form(mode):
    rng = np.random.default_rng(3)
    m, n, r = 24, 40, 6
    G = rng.standard_normal((m, n))
    cfg = _cfg(rank=r, mode=mode, eps=1e-30, refresh_interval=1000)
    st = apollo.init_state(cfg, m, n)
    W = np.zeros((m, n))
    for t in range(1, 8):
        info = apollo.step(cfg, st, W, G, t, lr=1e-3)
        R = info["R"]
        # bias-corrected M^ = R and V^ = R^2 at every step -> |R~| = 1
        np.testing.assert_allclose(np.abs(info["Rt"]), 1.0, rtol=1e-9)
        if mode == apollo.CHANNEL:
            np.testing.assert_allclose(info["s"], math.sqrt(r) / np.linalg.norm(R, axis=0), rtol=1e-9)
        else:
            np.testing.assert_allclose(info["s"], math.sqrt(r * n) / np.linalg.norm(R), rtol=1e-9)
        assert info["c"] == 1.0                         # the norm never grows
    # seven identical updates
    np.testing.assert_allclose(W, -7 * 1e-3 * G * info["s"][None, :], rtol=1e-9)


def test_without_bias_correction_constant_gradient():
    rng = np.random.default_rng(4)
    G = rng.standard_normal((8, 12))
    cfg = _cfg(rank=3, eps=0.0, bias_correction=False, refresh_interval=1000)
    st = apollo.init_state(cfg, 8, 12)
    W = np.zeros((8, 12))
    for t in range(1, 5):
        info = apollo.step(cfg, st, W, G, t, lr=1e-3)
        want = (1 - cfg.beta1 ** t) / math.sqrt(1 - cfg.beta2 ** t)
        np.testing.assert_allclose(np.abs(info["Rt"]), want, rtol=1e-10)


# ------------------------------------------------------------- reduces to textbook Adam
def test_identity_projection_is_channelwise_adam():
    """With P = I (r = m) the step is Section 3.2's structured Adam: ordinary Adam moments on
    G, s_j = ||G~[:, j]|| / ||G[:, j]||, W <- W - lr G diag(s)."""
    rng = np.random.default_rng(11)
    m, n = 6, 9
    cfg = _cfg(rank=m, nl_gamma=0.0)
    st = apollo.init_state(cfg, m, n)
    W = rng.standard_normal((m, n))
    W_ref = W.copy()
    M = np.zeros((m, n)); V = np.zeros((m, n))
    for t in range(1, 6):
        G = rng.standard_normal((m, n)) * (0.5 + t)
        apollo.step(cfg, st, W, G, t, lr=3e-3, P=np.eye(m))
        M = 0.9 * M + 0.1 * G
        V = 0.999 * V + 0.001 * G ** 2
        Gt = (M / (1 - 0.9 ** t)) / (np.sqrt(V / (1 - 0.999 ** t)) + 1e-8)
        s = np.linalg.norm(Gt, axis=0) / np.linalg.norm(G, axis=0)
        W_ref = W_ref - 3e-3 * G * s[None, :]
        np.testing.assert_allclose(W, W_ref, rtol=1e-12)
    np.testing.assert_allclose(st.M, M, rtol=1e-13)
    np.testing.assert_allclose(st.V, V, rtol=1e-13)


def test_tall_tensor_equals_transposed_wide_tensor():
    rng = np.random.default_rng(12)
    cfg = _cfg(rank=3, weight_decay=0.1, refresh_interval=2)
    W1 = rng.standard_normal((10, 4)); W2 = W1.T.copy()
    s1 = apollo.init_state(cfg, 10, 4); s2 = apollo.init_state(cfg, 4, 10)
    assert s1.M.shape == (3, 10) and s2.M.shape == (3, 10)
    for t in range(1, 6):
        G = rng.standard_normal((10, 4))
        i1 = apollo.step(cfg, s1, W1, G, t, lr=1e-2, tensor_id=3)
        i2 = apollo.step(cfg, s2, W2, G.T.copy(), t, lr=1e-2, tensor_id=3)
        assert not i1["left"] and i2["left"]
    np.testing.assert_allclose(W1, W2.T, rtol=1e-14)
    np.testing.assert_allclose(s1.M, s2.M, rtol=1e-14)
    assert s1.prev_norm == pytest.approx(s2.prev_norm, rel=1e-14)


def test_forced_side_overrides_the_shape_rule():
    rng = np.random.default_rng(13)
    G = rng.standard_normal((4, 10))
    cfg = _cfg(rank=2, side="right")
    st = apollo.init_state(cfg, 4, 10)
    assert st.M.shape == (2, 4)                         # channels are the 4 rows now
    info = apollo.step(cfg, st, np.zeros((4, 10)), G, 1, lr=1e-2)
    assert info["s"].shape == (4,) and not info["left"]
    cfg = _cfg(rank=2, side="left")                     # and the other way: a tall tensor projected along its rows
    st = apollo.init_state(cfg, 10, 4)
    assert st.M.shape == (2, 4)                         # channels are the 4 columns
    info = apollo.step(cfg, st, np.zeros((10, 4)), G.T.copy(), 1, lr=1e-2)
    assert info["s"].shape == (4,) and info["left"]
    assert apollo.is_left(10, 4) is False and apollo.is_left(10, 4, "left") is True


# ------------------------------------------------------- identities from the appendix
def test_first_moment_is_linear_in_a_fixed_projection():
    """Appendix A.2: with P fixed, M^R_t = P M_t where M_t is full-rank Adam's first moment."""
    rng = np.random.default_rng(21)
    m, n, r = 7, 12, 4
    cfg = _cfg(rank=r, refresh_interval=1000, seed=5)
    st = apollo.init_state(cfg, m, n)
    W = np.zeros((m, n))
    P = gauss.projection(5, 0, 0, r, m, False) / math.sqrt(r)
    M_full = np.zeros((m, n))
    for t in range(1, 9):
        G = rng.standard_normal((m, n))
        apollo.step(cfg, st, W, G, t, lr=1e-3)
        M_full = cfg.beta1 * M_full + (1 - cfg.beta1) * G
    np.testing.assert_allclose(st.M, P @ M_full, rtol=1e-11, atol=1e-14)


def test_second_moment_l1_norm_identity():
    """Appendix A.3: ||V^R_t[:, j]||_1 = (1 - beta2) sum_k beta2^k ||R_{t-k}[:, j]||^2."""
    rng = np.random.default_rng(22)
    cfg = _cfg(rank=5, refresh_interval=3)
    st = apollo.init_state(cfg, 16, 20)
    W = np.zeros((16, 20))
    hist = []
    for t in range(1, 8):
        info = apollo.step(cfg, st, W, rng.standard_normal((16, 20)), t, lr=1e-3)
        hist.append(np.sum(info["R"] ** 2, axis=0))
    T = len(hist)
    want = (1 - cfg.beta2) * sum(cfg.beta2 ** k * hist[T - 1 - k] for k in range(T))
    np.testing.assert_allclose(np.sum(np.abs(st.V), axis=0), want, rtol=1e-12)


def test_power_of_two_scale_invariance():
    rng = np.random.default_rng(23)
    cfg = _cfg(rank=3, eps=0.0, refresh_interval=2)
    grads = [rng.standard_normal((8, 12)) for _ in range(5)]
    outs = []
    for k in (0, 7):
        st = apollo.init_state(cfg, 8, 12)
        W = np.zeros((8, 12))
        for t, G in enumerate(grads, start=1):
            info = apollo.step(cfg, st, W, G * 2.0 ** k, t, lr=1e-2)
        outs.append((W.copy(), info["s"].copy(), st.M.copy(), st.V.copy()))
    assert np.array_equal(outs[0][0], outs[1][0])                  # same update, bit for bit
    assert np.array_equal(outs[0][1], outs[1][1] * 2.0 ** 7)
    assert np.array_equal(outs[0][2] * 2.0 ** 7, outs[1][2])
    assert np.array_equal(outs[0][3] * 2.0 ** 14, outs[1][3])


# --------------------------------------------------------------------------- JL (Theorem A.1)
def test_projection_preserves_squared_norm_in_expectation():
    rng = np.random.default_rng(31)
    m, n, r = 64, 6, 8
    G = rng.standard_normal((m, n))
    ratios = []
    for seed in range(400):
        cfg = _cfg(rank=r, seed=seed)
        st = apollo.init_state(cfg, m, n)
        info = apollo.step(cfg, st, np.zeros((m, n)), G, 1, lr=0.0)
        ratios.append(np.sum(info["R"] ** 2, axis=0) / info["colsq"])
    ratios = np.concatenate(ratios)                      # 2400 samples of chi2_r / r
    assert abs(ratios.mean() - 1.0) < 4.0 * math.sqrt(2.0 / (r * ratios.size))
    assert ratios.var() == pytest.approx(2.0 / r, rel=0.15)
    # Theorem A.1 tail bound: Pr[|ratio - 1| >= e] <= 2 exp(-r e^2 / 8)
    for e in (0.5, 1.0):
        assert np.mean(np.abs(ratios - 1.0) >= e) <= 2.0 * math.exp(-r * e * e / 8.0)


def test_scaling_factor_ratio_follows_sqrt_rank_ratio():
    """Section 4.1, bounded update ratio: s^R_j / s_j ~ sqrt(r / m) against the full-rank factor
    (P = I), so factors at ranks r1, r2 are in the ratio sqrt(r1 / r2)."""
    rng = np.random.default_rng(32)
    m, n = 96, 128
    grads = [rng.standard_normal((m, n)) for _ in range(6)]

    def final_s(rank, P=None):
        cfg = _cfg(rank=rank, seed=1, nl_gamma=0.0)
        st = apollo.init_state(cfg, m, n)
        W = np.zeros((m, n))
        for t, G in enumerate(grads, start=1):
            info = apollo.step(cfg, st, W, G, t, lr=1e-3, P=P)
        return info["s"]

    s_full = final_s(m, P=np.eye(m))
    s16, s32 = final_s(16), final_s(32)
    assert np.median(s32 / s16) == pytest.approx(math.sqrt(2.0), rel=0.10)
    assert np.median(s16 / s_full) == pytest.approx(math.sqrt(16.0 / m), rel=0.10)


# ------------------------------------------------------------------------------- limiter
def test_limiter_bounds_growth_and_stored_norm_is_the_applied_norm():
    rng = np.random.default_rng(41)
    golden = read_golden("paper_constants.txt")
    gamma = float(golden["nl_gamma"])
    cfg = _cfg(rank=4, nl_gamma=gamma, weight_decay=0.02, scale=1.7)
    st = apollo.init_state(cfg, 16, 24)
    W = rng.standard_normal((16, 24))
    prev = 0.0
    hits = 0
    for t in range(1, 12):
        G = rng.standard_normal((16, 24)) * (3.0 if t in (4, 9) else 1.0)
        W_old = W.copy()
        info = apollo.step(cfg, st, W, G, t, lr=1e-2)
        if prev > 0:
            assert st.prev_norm <= gamma * prev * (1 + 1e-12)
        hits += info["c"] < 1.0
        applied = np.linalg.norm((W_old - W) - 1e-2 * cfg.weight_decay * W_old) / 1e-2
        assert applied == pytest.approx(st.prev_norm, rel=1e-9)
        prev = st.prev_norm
    assert hits >= 2


def test_limiter_off_and_first_step_unlimited():
    rng = np.random.default_rng(42)
    G = rng.standard_normal((6, 6))
    for gamma in (0.0, 1.01):
        cfg = _cfg(rank=2, nl_gamma=gamma)
        st = apollo.init_state(cfg, 6, 6)
        W = np.zeros((6, 6))
        i1 = apollo.step(cfg, st, W, G, 1, lr=1e-2)
        assert i1["c"] == 1.0                                   # nothing to compare with yet
        i2 = apollo.step(cfg, st, W, -G, 2, lr=1e-2)            # the moment nearly cancels: small norm
        assert i2["c"] == 1.0 and i2["norm"] < 0.2 * i1["norm"]
        i3 = apollo.step(cfg, st, W, -G, 3, lr=1e-2)            # and builds up again: growth > gamma
        assert (i3["c"] == 1.0) == (gamma == 0.0)
        if gamma > 0:
            assert i3["norm"] == pytest.approx(gamma * i2["norm"], rel=1e-13)


def test_zero_gradient_gives_zero_update_and_no_nan():
    cfg = _cfg(rank=2)
    st = apollo.init_state(cfg, 4, 6)
    W = np.ones((4, 6))
    info = apollo.step(cfg, st, W, np.zeros((4, 6)), 1, lr=1e-2)
    assert np.all(info["s"] == 0.0) and np.all(W == 1.0) and st.prev_norm == 0.0
    info = apollo.step(cfg, st, W, np.ones((4, 6)), 2, lr=1e-2)      # stored norm 0 = unset
    assert info["c"] == 1.0 and np.all(np.isfinite(W))


# ---------------------------------------------------------------------- refresh and resume
def test_projection_is_resampled_exactly_every_T_steps():
    rng = np.random.default_rng(51)
    G = rng.standard_normal((8, 8))
    cfg = _cfg(rank=2, refresh_interval=3)
    Rs = []
    st = apollo.init_state(cfg, 8, 8)
    for t in range(1, 8):
        Rs.append(apollo.step(cfg, st, np.zeros((8, 8)), G, t, lr=0.0)["R"])
    same = [np.array_equal(Rs[i], Rs[i + 1]) for i in range(6)]
    assert same == [True, True, False, True, True, False]          # epochs {1,2,3} {4,5,6} {7}


def test_resume_from_saved_state_is_bit_identical():
    rng = np.random.default_rng(52)
    cfg = _cfg(rank=3, refresh_interval=4)
    grads = [rng.standard_normal((6, 10)) for _ in range(10)]
    W_a = np.zeros((6, 10)); st_a = apollo.init_state(cfg, 6, 10)
    for t, G in enumerate(grads, start=1):
        apollo.step(cfg, st_a, W_a, G, t, lr=1e-2)
    W_b = np.zeros((6, 10)); st_b = apollo.init_state(cfg, 6, 10)
    for t, G in enumerate(grads[:5], start=1):
        apollo.step(cfg, st_b, W_b, G, t, lr=1e-2)
    st_c = copy.deepcopy(st_b); W_c = W_b.copy()
    for t, G in enumerate(grads[5:], start=6):
        apollo.step(cfg, st_c, W_c, G, t, lr=1e-2)
    assert np.array_equal(W_a, W_c) and np.array_equal(st_a.M, st_c.M) and np.array_equal(st_a.V, st_c.V)


# ------------------------------------------------------------------ numbers the paper prints
def test_state_size_matches_table_1_and_the_7b_figure():
    g = read_golden("paper_constants.txt")
    h, f, L = int(g["llama7b_hidden"]), int(g["llama7b_intermediate"]), int(g["llama7b_layers"])
    shapes = ([(h, h)] * 4 + [(f, h)] * 2 + [(h, f)]) * L
    cfg = _cfg(rank=256)
    elems = apollo.state_elements(cfg, shapes)
    assert elems == 809_500_672 + 2 * len(shapes)
    # bf16 state: the paper's table prints 1.6G for APOLLO at r = 256
    assert round(2 * elems / 1e9, 1) == float(g["llama7b_r256_state_gb"])
    # sizing the state by the smaller dimension would give 0.94 GB: the "larger dimension" reading holds
    wrong = sum(2 * 256 * min(r_, c_) for r_, c_ in shapes)
    assert round(2 * wrong / 1e9, 1) != float(g["llama7b_r256_state_gb"])
    mini = apollo.state_elements(_cfg(rank=1, mode=apollo.TENSOR), shapes)
    assert mini == sum(2 * max(s) + 2 for s in shapes)
    assert float(g["mini_scale_squared"]) == 128 and int(g["refresh_interval"]) == apollo.Config(rank=1).refresh_interval
    assert apollo.Config(rank=1).nl_gamma == float(g["nl_gamma"])


# ----------------------------------------------------------------------------- bfloat16 storage
def _is_bf16(x):
    b = np.asarray(x, dtype=np.float32).view(np.uint32)
    return np.all(np.asarray(x, dtype=np.float32).astype(np.float64) == x) and not np.any(b & 0xFFFF)


def test_stored_rounds_to_nearest_even_bfloat16():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: ties go to the even mantissa (1); 1 + 3 * 2^-8
    # is halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -(1.0 + 2.0 ** -8),
                  3.140625, 1e-30, 0.0])
    got = apollo.stored(x, "bf16")
    assert list(got[:5]) == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0, 3.140625]
    assert got[6] == 0.0 and abs(got[5] - 1e-30) <= 1e-30 * 2.0 ** -8
    assert _is_bf16(got)
    assert apollo.stored(x, "f32") is x
    with pytest.raises(ValueError):
        apollo.stored(x, "fp8")


def test_bf16_storage_equals_f32_when_every_result_is_representable():
    """Powers of two everywhere: betas 0.5 / 0.75, P and G small integers, lr a power of two --
    every moment and every weight is a bfloat16 number, so the two storage types must agree bit
    for bit over several steps (the rounding is the only difference between them)."""
    P = np.array([[1.0, 0.0, 1.0]])
    G = np.array([[2.0, 4.0, 0.0, 1.0], [1.0, 1.0, 1.0, 1.0], [2.0, 0.0, 4.0, 1.0]])
    out = {}
    for dt in ("f32", "bf16"):
        cfg = _cfg(rank=1, beta1=0.5, beta2=0.75, eps=0.0, nl_gamma=0.0, weight_dtype=dt, state_dtype=dt)
        st = apollo.init_state(cfg, 3, 4)
        W = np.zeros((3, 4))
        # one step only for W: s is not a power of two in general, W after the step is rounded
        info = apollo.step(cfg, st, W, G, 1, 0.0, P=P)
        out[dt] = (st.M.copy(), st.V.copy(), info["s"].copy())
        info2 = apollo.step(cfg, st, W, 2 * G, 2, 0.0, P=P)
        out[dt] += (st.M.copy(), st.V.copy())
    for a, b in zip(out["f32"], out["bf16"]):
        assert np.array_equal(a, b)
    assert _is_bf16(out["bf16"][0]) and _is_bf16(out["bf16"][3])


def test_bf16_moments_are_rounded_when_stored_and_the_factor_uses_the_stored_values():
    P = np.array([[1.0]])
    # R = G; beta1 = 0.5: M = R / 2 = 1 + 2^-8 -> tie -> stored 1; V = R^2 / 4 (beta2 = 0.75)
    R = 2.0 + 2.0 ** -7
    G = np.array([[R, 3.0]])
    cfg = _cfg(rank=1, beta1=0.5, beta2=0.75, eps=0.0, nl_gamma=0.0, bias_correction=False,
               state_dtype="bf16")
    st = apollo.init_state(cfg, 1, 2)
    info = apollo.step(cfg, st, np.zeros((1, 2)), G, 1, 0.0, P=P)
    assert info["M_exact"][0, 0] == 1.0 + 2.0 ** -8 and st.M[0, 0] == 1.0
    v_exact = R * R / 4
    assert info["V_exact"][0, 0] == v_exact
    v_st = float(apollo.stored(np.array([v_exact]), "bf16")[0])
    assert st.V[0, 0] == v_st and v_st != v_exact
    # s_0 = |M / sqrt(V)| / |R| from the STORED moments
    assert info["s"][0] == pytest.approx((1.0 / math.sqrt(v_st)) / R, rel=1e-15)
    assert info["s"][0] != pytest.approx(((1.0 + 2.0 ** -8) / math.sqrt(v_exact)) / R, rel=1e-6)
    # f32 storage keeps the exact values
    cfg32 = _cfg(rank=1, beta1=0.5, beta2=0.75, eps=0.0, nl_gamma=0.0, bias_correction=False)
    st32 = apollo.init_state(cfg32, 1, 2)
    apollo.step(cfg32, st32, np.zeros((1, 2)), G, 1, 0.0, P=P)
    assert st32.M[0, 0] == 1.0 + 2.0 ** -8


def test_adopt_moments_replaces_the_stored_state_and_feeds_the_rest_of_the_step():
    P = np.array([[1.0]])
    G = np.array([[2.0, 1.0]])
    cfg = _cfg(rank=1, beta1=0.5, beta2=0.75, eps=0.0, nl_gamma=0.0, bias_correction=False)
    st = apollo.init_state(cfg, 1, 2)
    seen = {}

    def adopt(M_exact, V_exact):
        seen["M"], seen["V"] = M_exact.copy(), V_exact.copy()
        return 2.0 * M_exact, V_exact

    info = apollo.step(cfg, st, np.zeros((1, 2)), G, 1, 0.0, P=P, adopt_moments=adopt)
    assert np.array_equal(seen["M"], [[1.0, 0.5]]) and np.array_equal(seen["V"], [[1.0, 0.25]])
    assert np.array_equal(st.M, [[2.0, 1.0]])
    # R~ = M / sqrt(V) = 2 (both channels), s = 2 / |R|
    assert np.allclose(info["s"], [1.0, 2.0])


def test_bf16_weights_round_after_the_update_and_small_updates_vanish():
    P = np.array([[1.0]])
    G = np.array([[1.0, 1.0]])
    cfg = _cfg(rank=1, beta1=0.0, beta2=0.0, eps=0.0, nl_gamma=0.0, weight_dtype="bf16")
    # first step: R~ = sign(R) = 1, s = 1: update lr * G
    W = np.array([[1.0, 1.0]])
    st = apollo.init_state(cfg, 1, 2)
    info = apollo.step(cfg, st, W, G, 1, 2.0 ** -7, P=P)
    assert np.array_equal(info["W_exact"], [[1.0 - 2.0 ** -7] * 2]) and np.array_equal(W, info["W_exact"])
    # an update below half an ulp of the stored weight (2^-9 at 1.0, going down: ulp 2^-8) is lost
    W = np.array([[1.0, 1.0]])
    st = apollo.init_state(cfg, 1, 2)
    info = apollo.step(cfg, st, W, G, 1, 2.0 ** -11, P=P)
    assert info["W_exact"][0, 0] == 1.0 - 2.0 ** -11 and np.array_equal(W, [[1.0, 1.0]])
    # decay and update are rounded once, together
    cfg2 = _cfg(rank=1, beta1=0.0, beta2=0.0, eps=0.0, nl_gamma=0.0, weight_dtype="bf16", weight_decay=0.5)
    W = np.array([[1.0, 1.0]])
    st = apollo.init_state(cfg2, 1, 2)
    info = apollo.step(cfg2, st, W, G, 1, 2.0 ** -9, P=P)
    assert info["W_exact"][0, 0] == 1.0 - 2.0 ** -9 - 2.0 ** -10      # 1 - 3 * 2^-10
    assert W[0, 0] == 1.0 - 2.0 ** -8                                 # nearest bf16 below 1 (spacing 2^-8): 3/4 of the way


# ----------------------------------------------------------------------------- no projection (Section 3.2)
def test_identity_projection_is_the_structured_rule_of_section_3_2_by_brute_force():
    """Full-rank moments of G, G~ = M^ / (sqrt(V^) + eps), s_j = ||G~[:, j]|| / ||G[:, j]|| (Eq. 2),
    update G diag(s): scalar loops on a small tensor, both orientations and a square one (where a
    sum over the wrong axis would still have the right length)."""
    rng = np.random.default_rng(8)
    for rows, cols in ((3, 5), (5, 3), (4, 4)):
        cfg = _cfg(projection="identity", rank=99, nl_gamma=0.0, eps=1e-6)
        left = rows <= cols
        m, n = (rows, cols) if left else (cols, rows)
        st = apollo.init_state(cfg, rows, cols)
        assert st.M.shape == (m, n)
        W = rng.normal(size=(rows, cols))
        Wb = [list(r) for r in W]
        M = [[0.0] * cols for _ in range(rows)]
        V = [[0.0] * cols for _ in range(rows)]
        for t in (1, 2, 3):
            G = rng.normal(size=(rows, cols))
            apollo.step(cfg, st, W, G, t, 0.1)
            Gt = [[0.0] * cols for _ in range(rows)]
            for i in range(rows):
                for j in range(cols):
                    M[i][j] = 0.9 * M[i][j] + 0.1 * G[i, j]
                    V[i][j] = 0.999 * V[i][j] + 0.001 * G[i, j] ** 2
                    Gt[i][j] = (M[i][j] / (1 - 0.9 ** t)) / (math.sqrt(V[i][j] / (1 - 0.999 ** t)) + 1e-6)
            for ch in range(n):
                idx = [(i, ch) for i in range(rows)] if left else [(ch, i) for i in range(cols)]
                num = math.sqrt(sum(Gt[i][j] ** 2 for i, j in idx))
                den = math.sqrt(sum(G[i, j] ** 2 for i, j in idx))
                for i, j in idx:
                    Wb[i][j] -= 0.1 * (num / den) * G[i, j]
        np.testing.assert_allclose(W, np.array(Wb), rtol=1e-12)


def test_identity_projection_on_a_single_row_is_textbook_adam():
    """m = 1: every channel holds one element, s_j = |G~_j| / |G_j|, so G diag(s) = sign(G) |G~|:
    element-wise AdamW as long as each element's gradient keeps its sign (the first moment then has
    the sign of the gradient); checked against the separate AdamW oracle (pinned against torch)."""
    from oracle import adamw
    rng = np.random.default_rng(9)
    cfg = _cfg(projection="identity", nl_gamma=0.0, weight_decay=0.05)
    acfg = adamw.Config(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)
    W = rng.normal(size=(1, 17))
    Wa = W.copy().reshape(-1)
    st, sa = apollo.init_state(cfg, 1, 17), adamw.init_state(17)
    sign = np.sign(rng.normal(size=(1, 17)))
    for t in range(1, 6):
        G = sign * np.abs(rng.normal(size=(1, 17)))
        apollo.step(cfg, st, W, G, t, 0.01)
        adamw.step(acfg, sa, Wa, G.reshape(-1), t, 0.01)
    np.testing.assert_allclose(W.reshape(-1), Wa, rtol=1e-12)
    # with a sign flip the structured rule follows the gradient's sign, Adam the moment's
    G = -sign * 1e-3
    W2, Wa2 = W.copy(), Wa.copy()
    apollo.step(cfg, st, W2, G, 6, 0.01)
    adamw.step(acfg, sa, Wa2, G.reshape(-1), 6, 0.01)
    assert np.all(np.sign(W2 - W * (1 - 0.01 * 0.05)) == -np.sign(G))
    assert np.all(np.sign(Wa2 - Wa * (1 - 0.01 * 0.05)) == np.sign(G).reshape(-1))


def test_identity_projection_equals_a_hand_set_identity_matrix_and_counts_full_rank_state():
    rng = np.random.default_rng(10)
    G = rng.normal(size=(4, 6))
    a, b = _cfg(projection="identity"), _cfg(rank=4)
    Wa, Wb = np.ones((4, 6)), np.ones((4, 6))
    sa, sb = apollo.init_state(a, 4, 6), apollo.init_state(b, 4, 6)
    for t in (1, 2):
        ia = apollo.step(a, sa, Wa, G * t, t, 0.1)
        ib = apollo.step(b, sb, Wb, G * t, t, 0.1, P=np.eye(4))
    assert np.array_equal(Wa, Wb) and np.array_equal(ia["s"], ib["s"])
    assert apollo.state_elements(a, [(4, 6), (6, 4)]) == 2 * (2 * 4 * 6 + 2)
    with pytest.raises(ValueError):
        apollo.step(a, sa, Wa, G, 3, 0.1, P=np.eye(4))


def test_adopt_factors_scales_the_update_but_not_the_reported_factors():
    P = np.array([[1.0]])
    G = np.array([[2.0, 1.0]])
    cfg = _cfg(rank=1, beta1=0.0, beta2=0.0, eps=0.0, nl_gamma=0.0)
    st = apollo.init_state(cfg, 1, 2)
    W = np.zeros((1, 2))
    info = apollo.step(cfg, st, W, G, 1, 0.5, P=P, adopt_factors=lambda s, c: (3.0 * s, 0.5 * c))
    # own factors: s_j = 1 / |G_j|, c = 1; the update uses 3 s and c / 2: W = -lr * 1.5 * sign(G)
    assert np.allclose(info["s"], [0.5, 1.0]) and info["c"] == 1.0
    assert np.allclose(W, [[-0.75, -0.75]])


@pytest.mark.parametrize("rows,cols", [(6, 11), (11, 6), (7, 7)])
@pytest.mark.parametrize("mode,rank,projection", [(apollo.CHANNEL, 3, "random"), (apollo.TENSOR, 1, "random"),
                                                  (apollo.CHANNEL, 1, "identity"), (apollo.TENSOR, 1, "identity")])
@pytest.mark.parametrize("bias_correction,state_dtype", [(True, "f32"), (False, "f32"), (True, "bf16")])
def test_first_step_closed_form_equals_the_recurrence_at_t_1(rows, cols, mode, rank, projection, bias_correction,
                                                             state_dtype):
    """first_step_closed_form restates step() at t = 1; both namespaces (numpy and torch) must give
    what the recurrence gives from a zero state: R, colsq, M, V, s, the norm, c = 1 and the weight
    change (gradient part + decay)."""
    import torch
    rng = np.random.default_rng(rows * 31 + cols)
    G = gauss.round_to_bf16(rng.standard_normal((rows, cols)).astype(np.float32) * 1e-2).astype(np.float64)
    G[:, 2] = 0.0 if rows <= cols else G[:, 2]          # a zero channel (0/0 in s_j) when channels are columns
    if rows > cols:
        G[2, :] = 0.0
    W0 = rng.standard_normal((rows, cols)) * 0.02
    cfg = apollo.Config(rank=rank, mode=mode, seed=77, eps=1e-8, scale=1.7, weight_decay=0.03, bias_correction=bias_correction,
                   state_dtype=state_dtype, projection=projection, refresh_interval=4)
    lr = 1e-2
    st = apollo.init_state(cfg, rows, cols)
    W = W0.copy()
    info = apollo.step(cfg, st, W, G, 1, lr, tensor_id=5, grad_is_bf16=True)
    m = min(rows, cols)
    z = None if projection == "identity" else gauss.projection(77, 5, 0, rank, m, True)
    for xp, conv, back in ((np, lambda x: x, lambda x: np.asarray(x)),
                           (torch, lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x)), lambda x: x.numpy() if hasattr(x, "numpy") else np.asarray(x))):
        cf = apollo.first_step_closed_form(cfg, conv(G), lr, z=conv(z), xp=xp)
        assert cf["left"] == info["left"] and cf["c"] == 1.0 == info["c"]
        for key in ("R", "colsq", "s"):
            np.testing.assert_allclose(back(cf[key]), info[key], rtol=1e-12, atol=1e-300, err_msg=key)
        np.testing.assert_allclose(back(cf["M"]), st.M, rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(back(cf["V"]), st.V, rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(float(cf["norm"]), info["norm"], rtol=1e-12)
        np.testing.assert_allclose(back(cf["dW_grad"]) - lr * cfg.weight_decay * W0, W - W0, rtol=1e-9, atol=1e-18)
    assert np.any(info["s"] == 0.0) or mode == apollo.TENSOR


def test_a_non_finite_step_does_not_replace_the_stored_norm():
    """A gradient with an inf in it makes the step's norm non-finite; the stored norm must survive it
    (a NaN there would make every later limiter comparison false)."""
    cfg = _cfg(rank=2, refresh_interval=10)
    rng = np.random.default_rng(3)
    G = rng.standard_normal((6, 9)) * 1e-2
    st = apollo.init_state(cfg, 6, 9)
    W = np.zeros((6, 9))
    apollo.step(cfg, st, W, G, 1, 1e-3)
    kept = st.prev_norm
    assert kept > 0
    bad = G.copy()
    bad[1, 2] = np.inf
    with np.errstate(all="ignore"):
        apollo.step(cfg, st, W, bad, 2, 1e-3)
    assert st.prev_norm == kept
