"""Seeded sweep over option combinations: random small tensor lists (ragged shapes, both orientations,
shapes the matrix-core kernel takes, several tensors of one shape, one- to nine-row tensors with long
rows), ranks 1 to 128, channel- and tensor-wise factors, bf16 and fp32 gradients, bf16 storage of
the weights and of the moments, no projection, forced sides, refresh intervals 1 to 200, weight decay,
with and without bias correction, a boosted step that triggers the limiter -- every case stepped on
the GPU and in the fp64 oracle through parity_util.run_parity.

The comparison of R, colsq, M, V is the plain tolerance everywhere.  The factors s (and what they
scale) are allowed parity_util's per-channel widening here without the limits the benchmark
configurations are held to: among random small shapes there are channels whose projected gradient
falls next to zero or next to eps, where s_j amplifies the admissible error of R by any factor (the
limits are asserted where they mean something: tests/test_gpu_step.py, tests/test_gpu_large.py)."""
import math
import random

import pytest
import torch

from paper_2412_05270_amd import workloads as WL
from parity_util import run_parity

pytestmark = pytest.mark.gpu
CASES_PER_TEST = 12


def _shape(rng, rank):
    kind = rng.random()
    if kind < 0.15:
        s = (rng.choice([64, 128, 192, 256, 320]), rng.choice([256, 257, 300, 511, 512, 520, 777, 1025]))
    elif kind < 0.3:
        s = (rng.randint(rank, max(rank, 40)), rng.randint(rank, max(rank, 40)))
    elif kind < 0.4:
        s = (rng.randint(rank, max(rank, 9)), rng.randint(1 if rank == 1 else rank, 1200))
    else:
        s = (rng.randint(rank, 400), rng.randint(rank, 700))
    if rng.random() < 0.5:
        s = (s[1], s[0])
    return (max(s[0], rank), max(s[1], rank)) if min(s) < rank else s


def _case(index):
    rng = random.Random(77000 + index)
    rank = rng.choice([1, 1, 1, 2, 3, 5, 8, 16, 32, 32, 64, 96, 128])
    shapes = [_shape(rng, rank) for _ in range(rng.randint(1, 5))]
    if rng.random() < 0.3:
        shapes = shapes + shapes[:1] * rng.randint(1, 9)
    side = rng.choice(["auto", "auto", "left", "right"])
    if side != "auto":
        shapes = [s for s in shapes if (s[0] if side == "left" else s[1]) >= rank] or [(max(rank, 8), max(rank, 8))]
    wl = WL.Workload("sweep%d" % index, 60 + index, shapes, rng.choice([torch.bfloat16, torch.bfloat16, torch.float32]),
                     "normal", rng.choice([1e-3, 1e-2]), rank=rank, mode=rng.choice(["channel", "tensor"]),
                     scale=rng.choice([1.0, 2.0, math.sqrt(128.0)]), refresh_interval=rng.choice([1, 2, 3, 200]),
                     steps=rng.randint(2, 5), lr=10 ** rng.uniform(-4, -2), weight_decay=rng.choice([0.0, 0.0, 0.05]),
                     weight_dtype=torch.bfloat16 if rng.random() < 0.2 else torch.float32,
                     state_dtype=torch.bfloat16 if rng.random() < 0.2 else torch.float32,
                     projection="identity" if rng.random() < 0.12 else "random")
    return wl, side, rng.random() < 0.8, {rng.randint(2, wl.steps): 3.0}


@pytest.mark.parametrize("chunk", range(4))
def test_seeded_option_sweep(chunk):
    for index in range(chunk * CASES_PER_TEST, (chunk + 1) * CASES_PER_TEST):
        wl, side, bias_correction, boost = _case(index)
        print("case %d: rank %d %s %s %s side %s T %d W %s state %s %s" % (
            index, wl.rank, wl.mode, wl.grad_dtype, wl.shapes, side, wl.refresh_interval, wl.weight_dtype, wl.state_dtype,
            wl.projection), flush=True)
        run_parity(wl, list(range(len(wl.shapes))), wl.steps, side=side, bias_correction=bias_correction, boost=boost,
                   widen=True, max_widened_share=1.0, max_k=float("inf"), max_median_k=float("inf"))
