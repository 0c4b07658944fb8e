"""The step in two parts (apollo_step_prepare + apollo_step_launch) and its replay from a HIP graph.

apollo_step_launch is captured once; every iteration then writes the step's scalars with
apollo_step_prepare and replays the graph, with the program's own eager work (fresh gradients,
synchronisations, comparisons) between the replays.  Every replay is compared bit for bit with an
ordinary stepper that gets the same gradients through apollo_step: across re-samplings of P (the kernel
that writes P is in the graph and decides on the device), with the limiter hit, for every projection
path."""
import math

import pytest
import torch

import paper_2412_05270_amd as A
from paper_2412_05270_amd import workloads as WL
from parity_util import make_configs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF = torch.bfloat16


def _pair(wl):
    cfg, _ = make_configs(wl)
    w_ref = WL.make_weights(wl, DEV)
    w_new = [w.clone() for w in w_ref]
    grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
    return A.ApolloStepper(cfg, w_ref, grads, device=DEV), A.ApolloStepper(cfg, w_new, grads, device=DEV), w_ref, w_new, grads


def _same(ref, new, w_ref, w_new, tag):
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(zip(w_ref, w_new)):
        assert torch.equal(a, b), (tag, "W", i)
    # (the workspaces differ in what the device copy of the step scalars holds; the state must not)
    assert torch.equal(ref.state, new.state), (tag, "state")


@pytest.mark.parametrize("mode,rank,scale,wdt", [("channel", 32, 1.0, torch.float32), ("channel", 96, 1.0, torch.float32),
                                                 ("tensor", 1, math.sqrt(128.0), torch.float32), ("channel", 6, 1.0, BF)])
def test_prepare_and_launch_equal_the_ordinary_step(mode, rank, scale, wdt):
    shapes = [(128, 512), (512, 128), (96, 333), (256, 256)]
    wl = WL.Workload("two_part", 81, shapes, BF, "normal", 1e-2, rank=rank, mode=mode, scale=scale, refresh_interval=3,
                     steps=7, lr=1e-2, weight_decay=0.01, weight_dtype=wdt, state_dtype=wdt)
    ref, new, w_ref, w_new, grads = _pair(wl)
    for t in range(1, wl.steps + 1):
        WL.make_grads(wl, t, DEV, out=grads, boost=4.0 if t == 5 else 1.0)
        ref.step(t, wl.lr)
        if t == 4:                       # the two ways mixed: an ordinary step in between
            new.step(t, wl.lr)
        else:
            new.prepare(t, wl.lr)
            new.launch()
        _same(ref, new, w_ref, w_new, "step %d" % t)
    ref.close()
    new.close()


@pytest.mark.parametrize("mode,rank,scale", [("channel", 128, 1.0), ("tensor", 1, math.sqrt(128.0))])
def test_replay_from_a_graph_equals_the_ordinary_step_at_every_replay(mode, rank, scale):
    shapes = [(128, 512)] * 3 + [(512, 128)] * 2 + [(256, 256)] * 4 + [(128, 333)]
    wl = WL.Workload("graph", 82, shapes, BF, "normal", 1e-2, rank=rank, mode=mode, scale=scale, refresh_interval=3,
                     steps=9, lr=1e-2, weight_decay=0.01)
    ref, new, w_ref, w_new, grads = _pair(wl)
    # one ordinary step first: it puts the tensor pointers on the device (a copy, which stays out of the graph)
    WL.make_grads(wl, 1, DEV, out=grads)
    ref.step(1, wl.lr)
    new.step(1, wl.lr)
    _same(ref, new, w_ref, w_new, "step 1")
    graph = torch.cuda.CUDAGraph()
    # the capture itself runs nothing; the weights must not move while it is recorded
    before = [w.clone() for w in w_new]
    with torch.cuda.graph(graph):
        new.launch()
    torch.cuda.synchronize()
    for a, b in zip(before, w_new):
        assert torch.equal(a, b)
    for t in range(2, wl.steps + 1):
        WL.make_grads(wl, t, DEV, out=grads, boost=4.0 if t == 6 else 1.0)       # eager work between the replays
        ref.step(t, wl.lr)
        new.prepare(t, wl.lr)
        graph.replay()
        _same(ref, new, w_ref, w_new, "replay at step %d" % t)
    # back to ordinary steps after the replays (the host no longer knows which P the scratch holds)
    WL.make_grads(wl, wl.steps + 1, DEV, out=grads)
    ref.step(wl.steps + 1, wl.lr)
    new.step(wl.steps + 1, wl.lr)
    _same(ref, new, w_ref, w_new, "ordinary step after the replays")
    del graph
    ref.close()
    new.close()


def test_the_replayable_step_is_refused_with_the_chunked_schedule():
    """APOLLO_SCHEDULE_CHUNKED keeps no P between steps and decides nothing on the device: the two-part step
    is not offered with it, and says so instead of running."""
    wl = WL.Workload("chunked_launch", 83, [(128, 512), (256, 256)], BF, "normal", 1e-2, rank=32)
    cfg, _ = make_configs(wl)
    cfg.schedule = A.APOLLO_SCHEDULE_CHUNKED
    weights = WL.make_weights(wl, DEV)
    grads = WL.make_grads(wl, 1, DEV)
    st = A.ApolloStepper(cfg, weights, grads, device=DEV)
    st.step(1, wl.lr)
    st.prepare(2, wl.lr)
    with pytest.raises(A.ApolloError) as err:
        st.launch()
    assert err.value.status == A.APOLLO_EUNSUPPORTED and "CHUNKED" in str(err.value)
    st.close()
