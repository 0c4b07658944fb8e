"""The APOLLO / APOLLO-Mini step in fp64, one weight matrix at a time (oracle side).

Test infrastructure only (see the package docstring).  Follows Algorithm 1 of the paper step
by step, in its notation: G (gradient), P (random projection), R = P G (low-rank gradient),
M^R / V^R (low-rank Adam moments, Section 4.1), R~ = M^R / (sqrt(V^R) + eps), the channel-wise
factor s_j = ||R~[:, j]|| / ||R[:, j]|| (Eq. 4) or the tensor-wise factor s = ||R~|| / ||R||
(Section 4.2, APOLLO-Mini), the norm-growth limiter (Eq. 3, gamma = 1.01) and the update
W <- W - lr * alpha * G S - lr * lambda * W (Algorithm 1, step 4; the caller passes the
ordinary gradient, so the update subtracts).

Readings taken where the paper is silent or inconsistent:
  * Algorithm 1 assumes m <= n.  A stored tensor with more rows than columns is handled as its
    transpose: the smaller dimension is projected away, channels run along the larger one
    (Section 3.2 forms its channels along the larger dimension; the state size 2nr+2 of Table 1 with
    n the larger dimension agrees).
  * Adam's bias correction is applied (Algorithm 1 calls "AdamW(R_t, ...)"); eps is added after
    the bias-corrected square root.  bias_correction=False gives the literal Section 4.1 formula.
  * P ~ N(0, 1/r) (Algorithm 1, Theorem A.1): unit-variance z times 1/sqrt(r).
  * The limiter acts on the Frobenius norm of the whole scaled gradient alpha * G diag(s), one
    number per tensor (Table 1 counts one stored norm); nothing is limited while the stored norm
    is 0 (first step); the stored norm is the one after limiting; a step whose norm is not finite
    (a gradient with inf or NaN in it) does not replace it.
  * A channel whose projected gradient is exactly zero gets s_j = 0 (0/0 otherwise).
  * M^R, V^R are kept when P is re-sampled.
  * Steps are 1-based: P is re-sampled when (t-1) mod T == 0, epoch = (t-1) div T.
  * Storage types.  The paper trains in the bfloat16 format and sizes its state at 2 bytes per
    element (Table 3), but gives no rounding rule.  Taken here: arithmetic in (at least) binary32;
    a quantity kept in bfloat16 (W with weight_dtype="bf16"; M^R, V^R with state_dtype="bf16") is
    rounded to nearest, ties to even, when it is stored, and everything computed after that uses
    the stored value: R~ is formed from the rounded moments, so the state alone determines the
    rest of the step and a resumed run repeats it.
"""
from dataclasses import dataclass

import numpy as np

from . import gauss, q8

CHANNEL = "channel"   # APOLLO: one factor per channel
TENSOR = "tensor"     # APOLLO-Mini: one factor per tensor


@dataclass
class Config:
    rank: int
    mode: str = CHANNEL
    seed: int = 0
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    scale: float = 1.0             # alpha
    weight_decay: float = 0.0      # lambda
    nl_gamma: float = 1.01         # gamma; 0 switches the limiter off
    refresh_interval: int = 200    # T
    bias_correction: bool = True
    side: str = "auto"             # "auto" | "left" (project rows) | "right" (project columns)
    weight_dtype: str = "f32"      # "f32" | "bf16" | "q8" (group-wise 8-bit codes, oracle.q8): storage of W
    weight_rounding: str = "nearest"   # "nearest" | "stochastic": rounding of the 8-bit codes
    state_dtype: str = "f32"       # "f32" | "bf16": storage type of M^R, V^R
    projection: str = "random"     # "random" (Algorithm 1) | "identity": the structured channel-wise
                                   # rule of Section 3.2 itself, full-rank moments of G (P = I, rank
                                   # ignored: r = m), the reference the low-rank factors approximate


def stored(x, dtype):
    """x as it reads back after being stored in `dtype`: unchanged for "f32" (the oracle keeps
    fp64 there), the nearest bfloat16 (ties to even) of its binary32 value for "bf16"."""
    if dtype == "f32":
        return x
    if dtype != "bf16":
        raise ValueError("unknown storage type %r" % (dtype,))
    return gauss.round_to_bf16(np.asarray(x, dtype=np.float64).astype(np.float32)).astype(np.float64)


class TensorState:
    """Per-tensor optimizer state: M^R, V^R (r x n) and the previous scaled-gradient norm."""

    def __init__(self, r, n):
        self.M = np.zeros((r, n), dtype=np.float64)
        self.V = np.zeros((r, n), dtype=np.float64)
        self.prev_norm = 0.0
        # Algorithm 1 keeps P_t between re-samplings; so does the oracle (P is NOT optimizer
        # state to be saved: it is a function of the seed, and is re-derived when missing).
        self.z = None
        self.z_key = None


def is_left(rows, cols, side="auto"):
    if side == "left":
        return True
    if side == "right":
        return False
    return rows <= cols


def init_state(cfg, rows, cols):
    left = is_left(rows, cols, cfg.side)
    n, m = (cols, rows) if left else (rows, cols)
    return TensorState(m if cfg.projection == "identity" else cfg.rank, n)


def step(cfg, state, W, G, t, lr, tensor_id=0, grad_is_bf16=False, P=None, adopt_moments=None,
         adopt_factors=None):
    """One optimizer step on one tensor.  W, G: float64 arrays (rows x cols); W is updated in
    place and also returned (with weight_dtype="q8", W is a q8.Q8Weights whose codes, scales and
    zeros are replaced).  t is the 1-based step.  P, if given, replaces the generated
    r x m projection INCLUDING its 1/sqrt(r) (used by tests to inject a hand-set matrix).
    adopt_moments, if given, is a function (M_exact, V_exact) -> (M, V) called right after the
    moment update; what it returns becomes the stored state and feeds the rest of the step.
    Parity tests of the bfloat16 state use it to check the other side's rounding of each moment
    and then to continue from that side's decisions (a rounding taken one way on a value that
    sits near a tie is as correct as the other; everything downstream must follow one of them).
    adopt_factors, if given, is a function (s, c) -> (s, c) called after the limiter; what it
    returns scales the update.  Parity tests of the 8-bit weights use it the same way: the other
    side's factors are first compared with the oracle's, then adopted, so that the integer codes of
    the new weights are compared on identical real-valued inputs (up to binary32 rounding).
    Returns a dict with the intermediate quantities (R, R~, s, colsq, norm, c, and the values
    before storage rounding: M_exact, V_exact, W_exact).
    """
    rows, cols = G.shape
    Wq = None
    if cfg.weight_dtype == "q8":
        Wq, W = W, W.dequantise()
    left = is_left(rows, cols, cfg.side)
    Gm = G if left else G.T                       # m x n with the projected dimension first
    m, n = Gm.shape
    r = cfg.rank

    # Step 1: gradient into the low-rank space (or, Section 3.2, no projection at all).
    if cfg.projection == "identity":
        if P is not None:
            raise ValueError("a hand-set P and projection='identity' exclude each other")
        R = Gm.copy()
    elif cfg.projection != "random":
        raise ValueError("unknown projection %r" % (cfg.projection,))
    elif P is None:
        epoch = (t - 1) // cfg.refresh_interval
        key = (cfg.seed, tensor_id, epoch, r, m, bool(grad_is_bf16))
        if state.z_key != key:                    # "if t mod T = 0: P_t <- N_seed(0, 1/r)"
            state.z = gauss.projection(cfg.seed, tensor_id, epoch, r, m, grad_is_bf16)
            state.z_key = key
        R = (state.z @ Gm) / np.sqrt(np.float64(r))
    else:
        R = np.asarray(P, dtype=np.float64) @ Gm

    # Step 2: low-rank moments and the Adam-normalised low-rank gradient.
    M_exact = cfg.beta1 * state.M + (1.0 - cfg.beta1) * R
    V_exact = cfg.beta2 * state.V + (1.0 - cfg.beta2) * R * R
    if adopt_moments is None:
        state.M, state.V = stored(M_exact, cfg.state_dtype), stored(V_exact, cfg.state_dtype)
    else:
        state.M, state.V = adopt_moments(M_exact, V_exact)
    if cfg.bias_correction:
        bc1 = 1.0 - cfg.beta1 ** t
        bc2 = 1.0 - cfg.beta2 ** t
    else:
        bc1 = bc2 = 1.0
    Rt = (state.M / bc1) / (np.sqrt(state.V / bc2) + cfg.eps)

    # Step 3: the scaling factor.
    a = np.sum(Rt * Rt, axis=0)                   # ||R~[:, j]||^2
    b = np.sum(R * R, axis=0)                     # ||R[:, j]||^2
    if cfg.mode == CHANNEL:
        s = np.zeros(n)
        nz = b > 0
        s[nz] = np.sqrt(a[nz]) / np.sqrt(b[nz])
    else:
        bt = b.sum()
        s = np.full(n, np.sqrt(a.sum()) / np.sqrt(bt) if bt > 0 else 0.0)

    # Norm-growth limiter on || alpha * G diag(s) ||_F.
    colsq = np.sum(Gm * Gm, axis=0)
    norm = cfg.scale * np.sqrt(np.sum(s * s * colsq))
    c = 1.0
    if cfg.nl_gamma > 0 and state.prev_norm > 0 and norm > cfg.nl_gamma * state.prev_norm:
        c = cfg.nl_gamma * state.prev_norm / norm
        norm = cfg.nl_gamma * state.prev_norm
    if np.isfinite(norm):                         # (a non-finite step leaves the stored norm alone)
        state.prev_norm = norm
    s_own, c_own = s, c
    if adopt_factors is not None:
        s, c = adopt_factors(s, c)

    # Step 4: update in the original space.
    U = cfg.scale * c * (Gm * s[None, :])         # the scaled gradient, m x n
    if not left:
        U = U.T
    W_exact = W - (lr * U + lr * cfg.weight_decay * W)
    out = {"R": R, "Rt": Rt, "s": s_own, "colsq": colsq, "norm": norm, "c": c_own, "left": left,
           "M_exact": M_exact, "V_exact": V_exact, "W_exact": W_exact}
    if Wq is not None:
        u = q8.rounding_offsets(W_exact.shape, cfg.weight_rounding, cfg.seed, tensor_id, t)
        new, x = q8.quantise(W_exact, u)
        Wq.codes, Wq.scale, Wq.zero = new.codes, new.scale, new.zero
        out["q8_x"], out["q8_u"] = x, u
    else:
        W[...] = stored(W_exact, cfg.weight_dtype)
    return out


def first_step_closed_form(cfg, G, lr, z=None, xp=np):
    """What Algorithm 1 gives at t = 1, written as the closed form it has there instead of as the
    recurrence: with M^R_0 = V^R_0 = 0 the moments are M^R_1 = (1 - beta1) R and V^R_1 = (1 - beta2) R^2,
    Adam's bias corrections at t = 1 are exactly 1 - beta1 and 1 - beta2, so R~ = R / (|R| + eps)
    (without bias correction: R~ = (1 - beta1) R / (sqrt(1 - beta2) |R| + eps)); the limiter has no
    stored norm yet, so c = 1; the weights start from W_0 and only the scaled gradient and the decay
    move them.  Pinned against step() at t = 1 on small tensors; the GPU tests use it to cover every
    tensor of a full-size set, where the recurrence would need the whole state on the host.

    G: rows x cols, fp64.  z: the unit-variance projection, r x m (P = z / sqrt(r)); None with
    projection="identity".  xp: the array namespace of G and z (numpy, or torch for arrays that live
    on another device; only sqrt, abs, where, zeros_like and array methods common to both are used).
    Returns R, colsq, M, V (as stored: r x n), s (n values; all equal for the tensor-wise factor), norm,
    c and dW_grad = -lr * alpha * G diag(s) in the tensor's own orientation (the decay term
    -lr * lambda * W_0 is the caller's to add: it needs W_0)."""
    rows, cols = G.shape
    left = is_left(rows, cols, cfg.side)
    Gm = G if left else G.T
    if cfg.projection == "identity":
        R = Gm
    else:
        R = (z @ Gm) / float(np.sqrt(np.float64(cfg.rank)))
    M = (1.0 - cfg.beta1) * R
    V = (1.0 - cfg.beta2) * R * R
    M, V = _stored_xp(M, cfg.state_dtype, xp), _stored_xp(V, cfg.state_dtype, xp)
    bc1, bc2 = ((1.0 - cfg.beta1), (1.0 - cfg.beta2)) if cfg.bias_correction else (1.0, 1.0)
    Rt = (M / bc1) / (xp.sqrt(V / bc2) + cfg.eps)
    a = (Rt * Rt).sum(0)
    b = (R * R).sum(0)
    colsq = (Gm * Gm).sum(0)
    if cfg.mode == CHANNEL:
        safe = xp.where(b > 0, b, b + 1.0)
        s = xp.where(b > 0, xp.sqrt(a) / xp.sqrt(safe), xp.zeros_like(b))
    else:
        bt = b.sum()
        st = xp.sqrt(a.sum()) / xp.sqrt(bt) if float(bt) > 0 else 0.0 * bt
        s = xp.zeros_like(b) + st
    norm = cfg.scale * xp.sqrt((s * s * colsq).sum())
    U = cfg.scale * (Gm * s[None, :])
    if not left:
        U = U.T
    return {"R": R, "colsq": colsq, "M": M, "V": V, "s": s, "norm": norm, "c": 1.0, "dW_grad": -lr * U, "left": left}


def _stored_xp(x, dtype, xp):
    """stored() for either array namespace (bfloat16 rounding goes through the host for numpy's)."""
    if dtype == "f32":
        return x
    if xp is np:
        return stored(x, dtype)
    import torch
    return x.to(torch.float32).to(torch.bfloat16).to(x.dtype)


def state_elements(cfg, shapes):
    """Number of stored optimizer-state scalars (Table 1: 2nr + 2 per tensor for APOLLO,
    2n + 2 for Mini at r = 1, n the larger dimension; the "+2" are the seed and the norm)."""
    total = 0
    for rows, cols in shapes:
        left = is_left(rows, cols, cfg.side)
        n, m = (cols, rows) if left else (rows, cols)
        total += 2 * n * (m if cfg.projection == "identity" else cfg.rank) + 2
    return total
