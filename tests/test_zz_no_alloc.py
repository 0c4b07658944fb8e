"""apollo_step_noalloc (the step with its scratch in the library's static device array, for callers
that cannot allocate) against apollo_init + apollo_step on the same inputs, through the C ABI: the
two run the same kernels, so weights and the whole state buffer must agree bit for bit.  Two
sequences in a row on the one shared scratch, the second on a smaller tensor list, then the first
list again (whatever a call leaves in the scratch must not matter to the next)."""
import math

import pytest
import torch

import paper_2412_05270_amd as A
from paper_2412_05270_amd import workloads as WL
from parity_util import make_configs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF = torch.bfloat16

BIG = [(256, 512), (512, 256), (128, 520), (520, 128), (96, 333), (64, 2056), (300, 520)]
SMALL = [(64, 264), (264, 64), (33, 33)]


def _one_sequence(wl, steps, tag):
    cfg, _ = make_configs(wl)
    shapes = [(r, c, A.APOLLO_BF16 if wl.grad_dtype == BF else A.APOLLO_F32) for r, c in wl.shapes]
    # reference: a handle with a workspace of its own
    w_ref = WL.make_weights(wl, DEV)
    w_new = [w.clone() for w in w_ref]
    grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
    ref = A.ApolloStepper(cfg, w_ref, grads, device=DEV)
    sb = A.apollo_state_bytes(cfg, shapes)
    assert 0 < A.apollo_workspace_bytes(cfg, shapes) <= A.APOLLO_NOALLOC_SCRATCH_BYTES
    state = torch.full((sb,), 0xA5, dtype=torch.uint8, device=DEV)       # garbage: the call zero-fills it at step 1
    tensors = (A.ApolloTensor * len(shapes))()
    for i, (w, g) in enumerate(zip(w_new, grads)):
        tensors[i] = A.ApolloTensor(w.data_ptr(), g.data_ptr(), None)
    stream = torch.cuda.current_stream(DEV).cuda_stream
    for t in range(1, steps + 1):
        WL.make_grads(wl, t, DEV, out=grads, boost=3.0 if t == 3 else 1.0)
        ref.step(t, wl.lr)
        rc = A.apollo_step_noalloc(cfg, shapes, tensors, state.data_ptr(), sb, t == 1, t, wl.lr, stream)
        assert rc == A.APOLLO_OK, (tag, t, A.apollo_last_error())
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            assert torch.equal(w_new[i], w_ref[i]), (tag, "W", t, i)
        assert torch.equal(state, ref.state), (tag, "state", t)
    ref.close()


@pytest.mark.parametrize("mode,rank,scale", [("channel", 32, 1.0), ("tensor", 1, math.sqrt(128.0)), ("channel", 6, 1.0)])
def test_noalloc_step_equals_the_handle_step_bit_for_bit(mode, rank, scale):
    big = WL.Workload("noalloc_big", 71, BIG, BF, "normal", 1e-2, rank=rank, mode=mode, scale=scale,
                      refresh_interval=2, steps=4, lr=1e-2, weight_decay=0.01)
    small = WL.Workload("noalloc_small", 72, SMALL, BF, "normal", 1e-2, rank=rank, mode=mode, scale=scale,
                        refresh_interval=2, steps=3, lr=1e-2, weight_decay=0.01)
    _one_sequence(big, big.steps, "first call sequence")
    _one_sequence(small, small.steps, "second, smaller")
    _one_sequence(big, 2, "first list again")


def test_noalloc_step_with_bf16_storage_and_fp32_gradients():
    wl = WL.Workload("noalloc_store", 73, SMALL + [(48, 96)], torch.float32, "normal", 1e-2, rank=4, refresh_interval=2,
                     steps=3, lr=1e-2, weight_dtype=BF, state_dtype=BF)
    _one_sequence(wl, wl.steps, "bf16 storage")


def test_noalloc_step_rejects_what_does_not_fit():
    cfg, _ = make_configs(WL.Workload("noalloc_rej", 74, [(64, 64)], BF, "normal", 1e-2, rank=4))
    state = torch.zeros(1 << 20, dtype=torch.uint8, device=DEV)
    w = torch.zeros(64, 64, device=DEV)
    g = torch.zeros(64, 64, dtype=BF, device=DEV)
    many = [(64, 64, A.APOLLO_BF16)] * (A.APOLLO_NOALLOC_MAX_TENSORS + 1)
    rc = A.apollo_step_noalloc(cfg, many, [(w.data_ptr(), g.data_ptr())] * len(many), state.data_ptr(), state.numel(), 1, 1, 1e-3)
    assert rc == A.APOLLO_EUNSUPPORTED and "at most 64" in A.apollo_last_error()
    torch.cuda.synchronize()
    assert not bool(w.any())                       # nothing ran
