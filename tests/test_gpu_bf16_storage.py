"""GPU parity with bfloat16 storage of W and of the low-rank moments (through the C ABI).

A stored bfloat16 value is checked as a valid rounding: it must be the rounding (nearest even) of
some value within the usual tolerance of the oracle's unrounded result; the oracle then continues
from the library's stored moments, so that the factor, the norm and the weights are compared on
the same rounding decisions (parity_util.assert_rounds_within, oracle.apollo.step(adopt_moments=))."""
import math

import pytest
import torch

import paper_2412_05270_amd as A
from paper_2412_05270_amd import workloads as WL
from parity_util import run_parity

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32

# both orientations, one-tile and ragged channel counts, a channel count that is not a multiple of
# 4 (scalar path of the moment kernel) and a row length that is not (unaligned path of the update)
SHAPES = [(64, 264), (264, 64), (128, 520), (520, 128), (96, 333), (333, 96), (64, 64)]


@pytest.mark.parametrize("wdt,sdt", [(BF, BF), (F32, BF), (BF, F32)])
def test_channel_wise_bf16_storage(wdt, sdt):
    wl = WL.Workload("bf16_store_r32", 31, SHAPES, BF, "normal", 1e-2, rank=32, refresh_interval=3, steps=5,
                     lr=1e-2, weight_decay=0.05, weight_dtype=wdt, state_dtype=sdt)
    run_parity(wl, list(range(len(SHAPES))), wl.steps)


def test_generic_rank_with_fp32_gradients_and_bf16_storage():
    wl = WL.Workload("bf16_store_r6", 32, [(48, 96), (96, 48), (50, 77)], F32, "normal", 1e-2, rank=6,
                     refresh_interval=2, steps=5, lr=1e-2, weight_dtype=BF, state_dtype=BF)
    run_parity(wl, [0, 1, 2], wl.steps)


def test_rank_one_channel_wise_bf16_state():
    """Rank 1 with one factor per channel: s_j = |R~_j| / |R_j| is a single quotient, so a factor formed
    from the unrounded instead of the stored moments would be off by up to a bfloat16 unit in the last
    place (4e-3), far outside the tolerance."""
    wl = WL.Workload("bf16_store_r1c", 34, [(64, 264), (264, 64), (96, 333)], BF, "normal", 1e-2, rank=1,
                     refresh_interval=3, steps=5, lr=1e-2, weight_dtype=F32, state_dtype=BF)
    run_parity(wl, [0, 1, 2], wl.steps)


def test_mini_bf16_storage_with_limiter_hits():
    wl = WL.Workload("bf16_store_mini", 33, SHAPES, BF, "normal", 1e-2, rank=1, mode="tensor",
                     scale=math.sqrt(128.0), refresh_interval=3, steps=6, lr=1e-2, weight_dtype=BF, state_dtype=BF)
    hits = run_parity(wl, list(range(len(SHAPES))), wl.steps, boost={4: 4.0})
    assert hits > 0


def test_llama60m_bf16_storage():
    wl = WL.workload("llama60m")
    wl = WL.Workload("llama60m_bf16", wl.config_id, wl.shapes, wl.grad_dtype, wl.grad_kind, wl.grad_scale, rank=wl.rank,
                     refresh_interval=wl.refresh_interval, steps=4, weight_dtype=BF, state_dtype=BF)
    run_parity(wl, [0, 4, 6, 55], wl.steps)


def test_state_is_half_the_size_and_debug_views_are_fp32():
    cfg32 = A.ApolloConfig(rank=8, mode=A.APOLLO_CHANNEL, seed=1, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                           weight_decay=0.0, nl_gamma=1.01, refresh_interval=10, bias_correction=1, side=0)
    cfg16 = A.ApolloConfig(rank=8, mode=A.APOLLO_CHANNEL, seed=1, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                           weight_decay=0.0, nl_gamma=1.01, refresh_interval=10, bias_correction=1, side=0,
                           state_dtype=A.APOLLO_BF16)
    shapes = [(64, 256, A.APOLLO_BF16)]
    assert A.apollo_state_bytes(cfg32, shapes) == 2 * 8 * 256 * 4 + 256
    assert A.apollo_state_bytes(cfg16, shapes) == 2 * 8 * 256 * 2 + 256
    w = [torch.zeros(64, 256, device="cuda:0")]
    g = [torch.ones(64, 256, dtype=BF, device="cuda:0")]
    st = A.ApolloStepper(cfg16, w, g)
    st.step(1, 1e-3)
    m = st.debug(0, A.APOLLO_DBG_M)
    torch.cuda.synchronize()
    assert m.dtype == torch.float32 and m.shape == (8, 256)
    assert torch.equal(m, m.to(BF).float()) and float(m.abs().max()) > 0
    st.close()
