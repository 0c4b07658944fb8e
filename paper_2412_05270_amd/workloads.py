"""Seeded synthetic workloads: shapes and input generators shared by the tests, the smoke check
and the benchmark.  Nothing of the optimizer's arithmetic lives here.

The parameter sets take the LLaMA shapes of the paper's pre-training table (hidden /
intermediate size, layer count; per layer four hidden x hidden attention matrices, two
intermediate x hidden and one hidden x intermediate MLP matrices) and stand in for the
C4-trained models the paper measures on; values are random with the stated distributions.
"""
import math
from dataclasses import dataclass, field
from typing import List, Tuple

import torch


def llama_shapes(hidden, intermediate, layers):
    per_layer = [(hidden, hidden)] * 4 + [(intermediate, hidden)] * 2 + [(hidden, intermediate)]
    return per_layer * layers


@dataclass
class Workload:
    name: str
    config_id: int                      # seeds derive from it
    shapes: List[Tuple[int, int]]
    grad_dtype: torch.dtype
    grad_kind: str                      # "normal" | "student_t" | "colscale"
    grad_scale: float
    w_std: float = 0.02
    rank: int = 1
    mode: str = "channel"               # "channel" (APOLLO) | "tensor" (APOLLO-Mini)
    scale: float = 1.0                  # alpha
    refresh_interval: int = 200
    steps: int = 10
    lr: float = 0.01
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    nl_gamma: float = 1.01
    weight_decay: float = 0.0
    weight_dtype: torch.dtype = torch.float32   # storage type of W (torch.uint8: group-wise 8-bit codes)
    weight_rounding: str = "nearest"            # "nearest" | "stochastic": rounding of 8-bit codes
    state_dtype: torch.dtype = torch.float32    # storage type of the low-rank moments
    projection: str = "random"                  # "random" | "identity" (no projection: full-rank moments)
    extra: dict = field(default_factory=dict)

    @property
    def n_params(self):
        return sum(r * c for r, c in self.shapes)


MINI_SCALE = math.sqrt(128.0)


def workload(name):
    """The five configurations of the benchmark definition (and their Mini / channel variants)."""
    if name == "single256":
        return Workload(name, 1, [(256, 256)], torch.float32, "normal", 1e-2, rank=16, refresh_interval=5,
                        steps=10, lr=1e-3)
    if name == "llama60m":
        return Workload(name, 2, llama_shapes(512, 1376, 8), torch.bfloat16, "normal", 1e-3, rank=128,
                        refresh_interval=200, steps=100)
    if name == "llama1b":
        return Workload(name, 3, llama_shapes(2048, 5461, 24), torch.bfloat16, "student_t", 1e-3, rank=512,
                        steps=20)
    if name == "llama1b_mini":           # APOLLO-Mini on the 1B shapes: rows of 5461 elements start on no 16-byte boundary
        return Workload(name, 3, llama_shapes(2048, 5461, 24), torch.bfloat16, "student_t", 1e-3, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=20)
    if name == "llama7b_mini":
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=20)
    if name == "llama7b_r256":
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=256,
                        steps=20)
    if name == "llama7b_mini_bf16":      # the paper's all-bfloat16 setting: W and the moments in bf16
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=20, weight_dtype=torch.bfloat16,
                        state_dtype=torch.bfloat16)
    if name == "llama7b_r256_bf16":
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=256,
                        steps=20, weight_dtype=torch.bfloat16, state_dtype=torch.bfloat16)
    if name == "llama7b_mini_q8":        # Q-APOLLO-Mini: group-wise 8-bit weights, stochastic rounding
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=20, weight_dtype=torch.uint8,
                        weight_rounding="stochastic")
    if name == "llama7b_mini_q8_nearest":
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=20, weight_dtype=torch.uint8,
                        weight_rounding="nearest")
    if name == "llama7b_identity":       # Section 3.2's channel-wise rule with full-rank moments (no projection)
        return Workload(name, 4, llama_shapes(4096, 11008, 32), torch.bfloat16, "normal", 1e-3, rank=1,
                        steps=10, projection="identity")
    if name == "llama13b_mini":
        return Workload(name, 5, llama_shapes(5120, 13824, 40), torch.bfloat16, "colscale", 1.0, rank=1,
                        mode="tensor", scale=MINI_SCALE, steps=5)
    if name == "llama13b_r256":
        return Workload(name, 5, llama_shapes(5120, 13824, 40), torch.bfloat16, "colscale", 1.0, rank=256,
                        steps=5)
    raise KeyError(name)


def _generator(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_weights(wl, device):
    """Weights ~ N(0, w_std^2) (drawn in fp32, stored in the workload's weight type), one tensor per
    shape, seeded by the configuration."""
    gen = _generator(device, 1000 * wl.config_id)
    return [(torch.randn(s, generator=gen, device=device, dtype=torch.float32) * wl.w_std).to(wl.weight_dtype)
            for s in wl.shapes]


def make_q8_weights(wl, device):
    """Synthetic group-wise 8-bit weights: uniform random codes and, per group of 128 elements, a
    (scale, zero) pair that spans about +-4 w_std -- the shape and value range of quantised N(0,
    w_std^2) weights, without running a quantiser.  Returns (codes, metas): uint8 rows x cols and
    fp32 (rows * cols / 128, 2) tensors."""
    gen = _generator(device, 1000 * wl.config_id + 500)
    codes, metas = [], []
    for rows, cols in wl.shapes:
        assert cols % 128 == 0
        codes.append(torch.randint(0, 256, (rows, cols), generator=gen, device=device, dtype=torch.uint8))
        groups = rows * cols // 128
        span = wl.w_std * (7.0 + 2.0 * torch.rand(groups, generator=gen, device=device, dtype=torch.float32))
        metas.append(torch.stack([span / 255.0, -0.5 * span], dim=1).contiguous())
    return codes, metas


def _one_grad(shape, wl, gen, device, structure_along_rows):
    rows, cols = shape
    if wl.grad_kind == "normal":
        g = torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * wl.grad_scale
    elif wl.grad_kind == "student_t":
        # Student-t with 3 degrees of freedom: heavy-tailed entries, scale parameter grad_scale
        z = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        chi = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(3):
            chi += torch.randn(shape, generator=gen, device=device, dtype=torch.float32) ** 2
        g = z / torch.sqrt(chi / 3.0) * wl.grad_scale
    elif wl.grad_kind == "colscale":
        # per-column (or per-row) scales log-uniform in [1e-6, 1], 1 % of them exactly zero
        k = rows if structure_along_rows else cols
        u = torch.rand(k, generator=gen, device=device, dtype=torch.float32)
        sc = torch.pow(torch.tensor(10.0, device=device), -6.0 * u)
        dead = torch.rand(k, generator=gen, device=device, dtype=torch.float32) < 0.01
        sc = torch.where(dead, torch.zeros_like(sc), sc)
        g = torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * wl.grad_scale
        g = g * (sc[:, None] if structure_along_rows else sc[None, :])
    else:
        raise KeyError(wl.grad_kind)
    return g.to(wl.grad_dtype)


def make_grads(wl, step, device, out=None, boost=1.0):
    """Fresh gradients for 1-based `step` (seed = 1000 * config + step, tensor order fixed).
    `out`, a list of preallocated tensors, is filled in place when given.  With kind
    "colscale" the structure runs along the stored columns unless wl.extra["along"] == "channel",
    which puts it along the channel dimension (rows when rows > cols)."""
    gen = _generator(device, 1000 * wl.config_id + step)
    res = []
    for i, shape in enumerate(wl.shapes):
        along_rows = wl.extra.get("along") == "channel" and shape[0] > shape[1]
        g = _one_grad(shape, wl, gen, device, along_rows)
        if boost != 1.0:
            g = (g.float() * boost).to(wl.grad_dtype)
        if out is not None:
            out[i].copy_(g)
            res.append(out[i])
        else:
            res.append(g)
    return res


def dyadic_values(shape, gen, device, exp_lo=-1, exp_hi=0, significand_bits=8, dtype=torch.bfloat16):
    """Random values +-(1 + k / 2^(b-1)) * 2^e with k uniform in [0, 2^(b-1)) and e uniform in
    [exp_lo, exp_hi]: numbers with a b-bit significand (b <= 8: exact in bfloat16) and a narrow
    exponent range, so that sums and products of a few of them are exact in binary32.  Inputs for
    the tests of the storage rounding, where both sides must agree to the last bit."""
    b = significand_bits
    k = torch.randint(0, 1 << (b - 1), shape, generator=gen, device=device).to(torch.float32)
    e = torch.randint(exp_lo, exp_hi + 1, shape, generator=gen, device=device).to(torch.float32)
    sign = torch.randint(0, 2, shape, generator=gen, device=device).to(torch.float32) * 2.0 - 1.0
    v = sign * (1.0 + k / float(1 << (b - 1))) * torch.pow(torch.tensor(2.0, device=device), e)
    return v.to(dtype)
