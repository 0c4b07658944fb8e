"""GPU parity of the structured channel-wise rule without projection (Section 3.2, Eq. 2:
APOLLO_PROJ_IDENTITY, full-rank moments of G) against the oracle, through the C ABI."""
import math

import pytest
import torch

import paper_2412_05270_amd as A
from paper_2412_05270_amd import workloads as WL
from parity_util import run_parity

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32

# both orientations; channel counts / row lengths that are and are not multiples of 4; one square
SHAPES = [(64, 264), (264, 64), (96, 333), (333, 96), (50, 77), (77, 50), (128, 128), (1, 40), (40, 1)]


@pytest.mark.parametrize("gdt", [BF, F32])
def test_channel_wise_full_rank_moments(gdt):
    wl = WL.Workload("identity_ch", 41, SHAPES, gdt, "normal", 1e-2, rank=1, refresh_interval=3, steps=5, lr=1e-2,
                     weight_decay=0.05, projection="identity")
    run_parity(wl, list(range(len(SHAPES))), wl.steps)


def test_tensor_wise_full_rank_moments():
    # (the limiter in this mode is exercised by test_gpu_step.test_limiter_is_exercised_and_matches)
    wl = WL.Workload("identity_tensor", 42, SHAPES[:7], BF, "normal", 1e-2, rank=1, mode="tensor", refresh_interval=3,
                     steps=6, lr=1e-2, projection="identity")
    run_parity(wl, list(range(7)), wl.steps, boost={4: 4.0})


def test_bf16_storage_with_full_rank_moments():
    wl = WL.Workload("identity_bf16", 43, SHAPES[:7], BF, "normal", 1e-2, rank=1, refresh_interval=3, steps=4,
                     lr=1e-2, weight_dtype=BF, state_dtype=BF, projection="identity")
    run_parity(wl, list(range(7)), wl.steps)


def test_state_size_and_unavailable_views():
    cfg = A.ApolloConfig(rank=0, mode=A.APOLLO_CHANNEL, seed=1, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                         weight_decay=0.0, nl_gamma=1.01, refresh_interval=10, bias_correction=1, side=0,
                         projection=A.APOLLO_PROJ_IDENTITY)
    shapes = [(64, 256, A.APOLLO_BF16), (256, 64, A.APOLLO_BF16)]
    per = 2 * 64 * 256 * 4 + 256
    assert A.apollo_state_bytes(cfg, shapes) == 2 * per
    w = [torch.zeros(s[:2], device="cuda:0") for s in shapes]
    g = [torch.ones(s[:2], dtype=BF, device="cuda:0") for s in shapes]
    st = A.ApolloStepper(cfg, w, g)
    st.step(1, 1e-3)
    torch.cuda.synchronize()
    assert st.debug(1, A.APOLLO_DBG_M).shape == (256, 64)
    out = torch.empty(16, device="cuda:0")
    assert A.apollo_debug_get(st.handle, 0, A.APOLLO_DBG_R, out.data_ptr(), 64) == A.APOLLO_EINVAL
    assert A.apollo_debug_fill_projection(st.handle, 0, 1, out.data_ptr(), A.APOLLO_F32) == A.APOLLO_EINVAL
    # a constant gradient of ones: G~ = 1 / (1 + eps) at step 1, s_j = 1 / (1 + eps), update lr * s
    assert torch.allclose(w[0], torch.full_like(w[0], -1e-3), rtol=1e-5)
    st.close()


@pytest.mark.parametrize("rank", [16, 64, 256])
def test_low_rank_factors_track_the_full_rank_ones_by_sqrt_r_over_m(rank):
    """What this mode is for (Section 4.1, Theorem 4.1): the channel factors computed in the random
    rank-r space approximate the full-rank factors of Section 3.2 up to the constant sqrt(r / m).
    Both are taken from the library on the same gradients over several steps; the mean ratio over
    the channels must be sqrt(r / m) within a few per cent (the spread of a single channel is about
    1 / sqrt(2 r)), in both orientations."""
    dev = "cuda:0"
    for shape in ((1024, 2048), (2048, 1024)):
        m, n = min(shape), max(shape)
        gen = torch.Generator(device=dev)
        gen.manual_seed(4400 + rank)
        W = [torch.zeros(shape, device=dev), torch.zeros(shape, device=dev)]
        G = torch.empty(shape, device=dev, dtype=BF)
        common = dict(mode=A.APOLLO_CHANNEL, seed=7, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0, weight_decay=0.0,
                      nl_gamma=0.0, refresh_interval=200, bias_correction=1, side=A.APOLLO_SIDE_AUTO)
        low = A.ApolloStepper(A.ApolloConfig(rank=rank, **common), [W[0]], [G], device=dev)
        full = A.ApolloStepper(A.ApolloConfig(rank=1, projection=A.APOLLO_PROJ_IDENTITY, **common), [W[1]], [G], device=dev)
        for t in range(1, 6):
            G.copy_((torch.randn(shape, generator=gen, device=dev) * 1e-2).to(BF))
            low.step(t, 1e-3)
            full.step(t, 1e-3)
            ratio = low.debug(0, A.APOLLO_DBG_S).double() / full.debug(0, A.APOLLO_DBG_S).double()
            assert ratio.numel() == n
            mean = float(ratio.mean()) / math.sqrt(rank / m)
            spread = float(ratio.std()) / math.sqrt(rank / m)
            assert abs(mean - 1.0) < 0.05, (shape, rank, t, mean)
            assert spread < 2.5 / math.sqrt(2.0 * rank), (shape, rank, t, spread)
        low.close()
        full.close()
