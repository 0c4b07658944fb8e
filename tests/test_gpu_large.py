"""GPU parity at the benchmark's full sizes: every tensor of the LLaMA-shaped sets is stepped on
the GPU in the launch configuration bench.py times; the fp64 oracle follows one tensor of each
distinct shape from the first and the last layer (the full sets do not fit host memory in
fp64).  Collected last by name so a failure here does not hide the smaller cases."""
import pytest
import torch

from paper_2412_05270_amd import workloads as WL
from parity_util import run_parity
from test_gpu_step import _first_and_last_layer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,steps", [
    ("llama1b", 3),
    ("llama7b_mini", 3),
    ("llama7b_r256", 2),
    ("llama13b_mini", 2),
    ("llama13b_r256", 2),
    ("llama7b_mini_bf16", 2),       # bfloat16 W and moments (valid-rounding checks)
    ("llama7b_r256_bf16", 2),
])
def test_full_size_sets(name, steps):
    wl = WL.workload(name)
    ids = _first_and_last_layer(wl)
    run_parity(wl, ids, steps, progress=True)
    torch.cuda.empty_cache()


def test_llama13b_zero_channels_on_the_tall_tensors():
    wl = WL.workload("llama13b_r256")
    wl.extra["along"] = "channel"
    wl.name = "llama13b_r256_channel_structure"
    wl.shapes = wl.shapes[:7]                      # one layer is enough for the edge case
    run_parity(wl, list(range(7)), 2, progress=True)
    torch.cuda.empty_cache()


def test_full_size_q8_mini():
    """LLaMA-7B shapes with group-wise 8-bit weights and stochastic rounding, every tensor stepped
    on the GPU, three tensors of the first and of the last layer followed by the oracle."""
    from test_gpu_q8 import _run
    wl = WL.workload("llama7b_mini_q8")
    _run(wl, 2, 1e-5, check_ids=_first_and_last_layer(wl), progress=True)
    torch.cuda.empty_cache()
