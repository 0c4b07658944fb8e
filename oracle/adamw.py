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
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class Config:
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0      # lambda
    bias_correction: bool = True


class TensorState:
    """M, V of one parameter tensor (any shape, handled flat)."""

    def __init__(self, numel):
        self.M = np.zeros(numel, dtype=np.float64)
        self.V = np.zeros(numel, dtype=np.float64)


def init_state(numel):
    return TensorState(int(numel))


def step(cfg, state, W, G, t, lr):
    """One AdamW step in place on the flat fp64 array W with gradient G at 1-based step t.

    Section 3.1, Eq. 1: M_t = beta1 M_{t-1} + (1 - beta1) G_t, V_t = beta2 V_{t-1} + (1 - beta2) G_t^2,
    G~_t = M^_t / (sqrt(V^_t) + eps) with M^ = M / (1 - beta1^t), V^ = V / (1 - beta2^t),
    W_{t+1} = W_t - lr G~_t - lr lambda W_t.  Returns G~_t.
    """
    if t < 1:
        raise ValueError("steps are 1-based")
    W = np.asarray(W)
    G = np.asarray(G, dtype=np.float64).reshape(-1)
    if W.dtype != np.float64 or W.size != G.size or G.size != state.M.size:
        raise ValueError("W must be fp64 and W, G, state must have the same number of elements")
    state.M *= cfg.beta1
    state.M += (1.0 - cfg.beta1) * G
    state.V *= cfg.beta2
    state.V += (1.0 - cfg.beta2) * G * G
    bc1 = 1.0 - cfg.beta1 ** t if cfg.bias_correction else 1.0
    bc2 = 1.0 - cfg.beta2 ** t if cfg.bias_correction else 1.0
    Gt = (state.M / bc1) / (np.sqrt(state.V / bc2) + cfg.eps)
    flat = W.reshape(-1)
    flat -= lr * Gt + lr * cfg.weight_decay * flat
    return Gt
