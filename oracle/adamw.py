"""Element-wise AdamW in fp64 (oracle side) for the parameters APOLLO does not project.

Test infrastructure only (see the package docstring).  The paper applies APOLLO to the attention
and MLP weight matrices; everything else (embeddings, norm gains, the output head) keeps the
optimizer it starts from, AdamW, whose rule Section 3.1 restates (Eq. 1): exponentially weighted
first and second moments M, V of the gradient, update M / (sqrt(V) + eps).  Section 3.1 leaves
weight decay aside; it is the decoupled decay of AdamW (Loshchilov & Hutter, ICLR 2019),
W <- W - lr * lambda * W with the old W, the same term Algorithm 1 (step 4) carries.  Adam's bias
correction is applied as for the low-rank moments (the same reading as in oracle.apollo): the
stored moments are the raw averages; bias_correction=False gives Eq. 1 literally.  The caller
passes the ordinary gradient, so the update subtracts.

Storage in bfloat16 (store_dtype="bf16": W, M and V of the tensor are kept in bfloat16, the paper's
all-bfloat16 training setting carried over to these parameters) follows the rule of oracle.apollo:
arithmetic in fp64 here (fp32 in the library), a stored quantity is rounded to nearest even when
it is written, and whatever is computed after that uses the stored value -- the update is formed
from the rounded moments, the new weight is rounded last.
"""
from dataclasses import dataclass

import numpy as np

from .apollo import stored


@dataclass
class Config:
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0      # lambda
    bias_correction: bool = True
    store_dtype: str = "f32"       # "f32" | "bf16": how W, M and V are kept between steps


class TensorState:
    """M, V of one parameter tensor (any shape, handled flat)."""

    def __init__(self, numel):
        self.M = np.zeros(numel, dtype=np.float64)
        self.V = np.zeros(numel, dtype=np.float64)


def init_state(numel):
    return TensorState(int(numel))


def step(cfg, state, W, G, t, lr, adopt_moments=None):
    """One AdamW step in place on the flat fp64 array W with gradient G at 1-based step t.

    Section 3.1, Eq. 1: M_t = beta1 M_{t-1} + (1 - beta1) G_t, V_t = beta2 V_{t-1} + (1 - beta2) G_t^2,
    G~_t = M^_t / (sqrt(V^_t) + eps) with M^ = M / (1 - beta1^t), V^ = V / (1 - beta2^t),
    W_{t+1} = W_t - lr G~_t - lr lambda W_t.  Returns G~_t.  The values before storage rounding
    are left in state.M_exact, state.V_exact, state.W_exact.  adopt_moments, if given, is a function
    (M_exact, V_exact) -> (M, V) whose result becomes the stored state and feeds the update (parity
    tests of bfloat16 storage check the other side's roundings with it and then follow them).
    """
    if t < 1:
        raise ValueError("steps are 1-based")
    W = np.asarray(W)
    G = np.asarray(G, dtype=np.float64).reshape(-1)
    if W.dtype != np.float64 or W.size != G.size or G.size != state.M.size:
        raise ValueError("W must be fp64 and W, G, state must have the same number of elements")
    state.M_exact = cfg.beta1 * state.M + (1.0 - cfg.beta1) * G
    state.V_exact = cfg.beta2 * state.V + (1.0 - cfg.beta2) * G * G
    if adopt_moments is None:
        state.M, state.V = stored(state.M_exact, cfg.store_dtype), stored(state.V_exact, cfg.store_dtype)
    else:
        state.M, state.V = adopt_moments(state.M_exact, state.V_exact)
    bc1 = 1.0 - cfg.beta1 ** t if cfg.bias_correction else 1.0
    bc2 = 1.0 - cfg.beta2 ** t if cfg.bias_correction else 1.0
    Gt = (state.M / bc1) / (np.sqrt(state.V / bc2) + cfg.eps)
    flat = W.reshape(-1)
    state.W_exact = flat - (lr * Gt + lr * cfg.weight_decay * flat)
    flat[...] = stored(state.W_exact, cfg.store_dtype)
    return Gt
