"""GPU parity of the whole step against the fp64 oracle, through the C ABI, on the benchmark's
configurations (all tensors stepped on the GPU in the launch configuration the benchmark uses;
the oracle follows a subset where the full set does not fit the host) and on edge cases."""
import math

import numpy as np
import pytest
import torch

import paper_2412_05270_amd as A
from paper_2412_05270_amd import workloads as WL
from parity_util import assert_close, make_configs, run_parity, to_host_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _first_and_last_layer(wl):
    """One tensor of each distinct shape from the first and from the last layer."""
    ids, seen = [], set()
    for i, s in enumerate(wl.shapes[:7]):
        if s not in seen:
            seen.add(s)
            ids.append(i)
    n = len(wl.shapes)
    return ids + [n - 7 + (i % 7) for i in ids]


def test_single256_fp32_all_steps():
    wl = WL.workload("single256")
    run_parity(wl, [0], wl.steps)                      # T = 5: crosses two refreshes


def test_llama60m_bf16_rank128():
    wl = WL.workload("llama60m")
    ids = list(range(len(wl.shapes)))
    run_parity(wl, ids, 12, compare_steps={1, 2, 7, 12})


def test_llama60m_long_run_subset():
    wl = WL.workload("llama60m")
    run_parity(wl, _first_and_last_layer(wl), wl.steps, compare_steps={1, 50, 100})


RAGGED = [(100, 36), (36, 100), (77, 130), (130, 77), (8, 8), (64, 2056), (300, 520), (1100, 264),
          (1500, 2056), (33, 33)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("mode,rank,scale", [("channel", 1, 1.0), ("tensor", 1, math.sqrt(128.0)),
                                             ("channel", 7, 1.0), ("tensor", 8, 2.0)])
def test_ragged_shapes_both_sides_with_weight_decay_and_limiter(dtype, mode, rank, scale):
    wl = WL.Workload("ragged", 7, RAGGED, dtype, "normal", 1e-2, rank=rank, mode=mode, scale=scale,
                     refresh_interval=3, steps=7, lr=1e-2, weight_decay=0.05)
    run_parity(wl, list(range(len(RAGGED))), wl.steps, boost={4: 3.0})


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rank_one_takes_the_streaming_kernel_for_any_row_length(dtype):
    """Row lengths that are not a multiple of 8 (rows that start on no 16-byte boundary, a ragged last
    octet) are served by the rank-1 kernels too, not by the general projection; their results are what
    test_ragged_shapes_both_sides_with_weight_decay_and_limiter compares with the oracle."""
    wl = WL.Workload("ragged", 7, RAGGED, dtype, "normal", 1e-2, rank=1, mode="tensor", scale=2.0)
    cfg, _ = make_configs(wl)
    weights = [torch.zeros(s, dtype=torch.float32, device=DEV) for s in RAGGED]
    grads = [torch.zeros(s, dtype=dtype, device=DEV) for s in RAGGED]
    st = A.ApolloStepper(cfg, weights, grads, device=DEV)
    for i in range(len(RAGGED)):
        assert st.path(i) == (A.APOLLO_PATH_RANK1, 0), (RAGGED[i], st.path(i))
    st.close()


# shapes chosen so that the matrix-core projection runs with 1, 2, 3 and 5 pipeline stages (m = 64,
# 128, 192, 320), a ragged (shifted) last channel tile (n = 264, 520, 1376), exactly one tile
# (n = 256), and both orientations
MFMA_SHAPES = [(64, 264), (264, 64), (128, 520), (520, 128), (192, 256), (256, 192), (320, 1376), (1376, 320)]


@pytest.mark.parametrize("rank", [32, 64, 96, 128, 256])
def test_matrix_core_projection_tile_configurations(rank):
    shapes = [s for s in MFMA_SHAPES if min(s) >= rank]
    wl = WL.Workload("mfma_cfg_r%d" % rank, 12, shapes, torch.bfloat16, "normal", 1e-2, rank=rank,
                     refresh_interval=2, steps=3, lr=1e-2)
    run_parity(wl, list(range(len(shapes))), wl.steps)


@pytest.mark.parametrize("rank", [32, 128])
def test_matrix_core_projection_rows_not_multiple_of_eight(rank):
    """Rows projected and a row length that is odd / not a multiple of 8 (LLaMA-1B's 2048 x 5461
    has this): the projection reads a row-padded copy of the gradient, and the shifted last channel
    tile reaches past n into the padding (n = 333: 2 channels, n = 259: 5, n = 1001: 7)."""
    shapes = [(128, 333), (192, 259), (128, 1001), (256, 262)]
    # and, with columns projected, channel counts that are not multiples of 8 (5461 x 2048 has this):
    # no padding there, the last tile ends exactly at n
    shapes += [(333, 128), (259, 192)]
    wl = WL.Workload("mfma_pad_r%d" % rank, 13, shapes, torch.bfloat16, "normal", 1e-2, rank=rank,
                     refresh_interval=2, steps=3, lr=1e-2)
    run_parity(wl, list(range(len(shapes))), wl.steps)


@pytest.mark.parametrize("side", ["left", "right"])
def test_forced_side_and_no_bias_correction(side):
    shapes = [(48, 96), (96, 48), (64, 64)]
    wl = WL.Workload("forced", 8, shapes, torch.bfloat16, "normal", 1e-2, rank=6, refresh_interval=2,
                     steps=5, lr=1e-2)
    run_parity(wl, [0, 1, 2], wl.steps, side=side, bias_correction=False)


def test_limiter_is_exercised_and_matches():
    """A gradient, its negative, then its negative again: the moment nearly cancels and builds up
    again, so the scaled-gradient norm grows by far more than gamma at step 3."""
    shapes = [(64, 128), (128, 64)]
    for mode, rank, proj in (("channel", 8, "random"), ("tensor", 1, "random"), ("channel", 1, "identity")):
        wl = WL.Workload("limiter", 9, shapes, torch.bfloat16, "normal", 1e-2, rank=rank, mode=mode,
                         refresh_interval=100, steps=4, lr=1e-2, projection=proj)
        cfg, ocfg = make_configs(wl)
        from oracle import apollo as O
        weights = WL.make_weights(wl, DEV)
        g0 = WL.make_grads(wl, 1, DEV)
        grads = [g.clone() for g in g0]
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        ost = [O.init_state(ocfg, *s) for s in shapes]
        W = [to_host_f64(w) for w in weights]
        hits = 0
        for t, sign in enumerate((1.0, -1.0, -1.0, 1.0), start=1):
            for g, src in zip(grads, g0):
                g.copy_((src.float() * sign).to(torch.bfloat16))
            st.step(t, wl.lr)
            torch.cuda.synchronize()
            for i in range(len(shapes)):
                info = O.step(ocfg, ost[i], W[i], to_host_f64(grads[i]), t, float(np.float32(wl.lr)), tensor_id=i,
                              grad_is_bf16=True)
                hits += info["c"] < 1.0
                assert_close("c", to_host_f64(st.debug(i, A.APOLLO_DBG_C)), [info["c"]], 1e-3)
                assert_close("norm", to_host_f64(st.debug(i, A.APOLLO_DBG_NORM)), [info["norm"]], 1e-3)
                assert_close("W", to_host_f64(weights[i]), W[i], 1e-3)
        assert hits >= 2
        st.close()


def test_zero_gradient_and_zero_channels():
    shapes = [(64, 128), (128, 64)]
    wl = WL.Workload("zeros", 10, shapes, torch.bfloat16, "colscale", 1.0, rank=4, refresh_interval=100,
                     steps=3, lr=1e-2, extra={"along": "channel"})
    run_parity(wl, [0, 1], wl.steps)
    # an all-zero gradient: no NaN, W unchanged, stored norm 0
    cfg, _ = make_configs(wl)
    weights = WL.make_weights(wl, DEV)
    w0 = [w.clone() for w in weights]
    grads = [torch.zeros(s, dtype=torch.bfloat16, device=DEV) for s in shapes]
    st = A.ApolloStepper(cfg, weights, grads, device=DEV)
    st.step(1, 0.01)
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(weights[i], w0[i])
        assert float(st.debug(i, A.APOLLO_DBG_NORM)[0]) == 0.0
        assert torch.all(st.debug(i, A.APOLLO_DBG_S) == 0)
    st.close()


def test_run_to_run_determinism_and_resume():
    wl = WL.Workload("resume", 11, [(96, 200), (200, 96), (512, 512)], torch.bfloat16, "normal", 1e-2, rank=16,
                     refresh_interval=4, steps=10, lr=1e-2)
    cfg, _ = make_configs(wl)

    def run(split):
        weights = WL.make_weights(wl, DEV)
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        for t in range(1, wl.steps + 1):
            if t == split:                      # checkpoint: state buffer out, new handle, state back in
                saved = st.state.clone()
                st.close()
                st = A.ApolloStepper(cfg, weights, grads, device=DEV, zero_state=False)
                st.state.copy_(saved)
            WL.make_grads(wl, t, DEV, out=grads)
            st.step(t, wl.lr)
        torch.cuda.synchronize()
        out = [w.clone() for w in weights] + [st.state.clone()]
        st.close()
        return out

    a, b, c = run(None), run(None), run(6)
    for x, y, z in zip(a, b, c):
        assert torch.equal(x, y)                # same inputs twice: bit-identical (no atomics)
        assert torch.equal(x, z)                # 10 steps == 5 + save/restore + 5


def test_overlapped_and_serial_schedules_agree_bit_for_bit():
    """Three shape groups with matrix-core projections: the overlapped schedule runs them as chains on
    two streams; the groups touch disjoint data, so W and the whole state must equal the serial
    schedule's exactly, step after step, and the caller's stream must see the step as ordinary
    in-order work (the comparison below reads W right after a synchronise of that stream only)."""
    shapes = [(128, 512)] * 3 + [(512, 128)] * 2 + [(256, 256)] * 4
    wl = WL.Workload("schedules", 14, shapes, torch.bfloat16, "normal", 1e-2, rank=64, refresh_interval=2, steps=6,
                     lr=1e-2, weight_decay=0.01)
    runs = []
    for schedule in (A.APOLLO_SCHEDULE_OVERLAP, A.APOLLO_SCHEDULE_SERIAL):
        cfg, _ = make_configs(wl)
        cfg.schedule = schedule
        weights = WL.make_weights(wl, DEV)
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        snaps = []
        for t in range(1, wl.steps + 1):
            WL.make_grads(wl, t, DEV, out=grads)
            st.step(t, wl.lr)
            torch.cuda.current_stream(DEV).synchronize()
            snaps.append([w.clone() for w in weights] + [st.state.clone()])
        st.close()
        runs.append(snaps)
    for a, b in zip(*runs):
        for x, y in zip(a, b):
            assert torch.equal(x, y)


@pytest.mark.parametrize("dtype,rank,sdt", [(torch.bfloat16, 64, torch.float32), (torch.bfloat16, 96, torch.bfloat16),
                                            (torch.float32, 8, torch.float32), (torch.bfloat16, 1, torch.float32)])
def test_chunked_and_serial_schedules_agree_bit_for_bit(dtype, rank, sdt, monkeypatch):
    """APOLLO_SCHEDULE_CHUNKED keeps no P between steps: every step generates it chunk by chunk of a
    shape group's tensors over one scratch region and projects each chunk before the next overwrites it.
    The same P, the same kernels per tensor: W and the whole state must equal the serial schedule's
    exactly at every step, with a smaller workspace, across re-samplings, for the matrix-core and the
    general projection (R of a matrix-core tensor is recomputed for the debug view from a P that has to
    be generated again: compared too).  The chunk size is a compile-time 128 MiB: tensors of 8 MiB of P
    each (rank 64 x 65536 columns would be needed) do not belong into a test, so the tensors here form
    one chunk per group -- the case of several chunks per group runs at full size in
    tests/test_gpu_large.py."""
    shapes = [(128, 512)] * 3 + [(512, 128)] * 2 + [(256, 256)] * 4 + [(96, 333)]
    wl = WL.Workload("chunked", 15, shapes, dtype, "normal", 1e-2, rank=rank, refresh_interval=2, steps=5,
                     lr=1e-2, weight_decay=0.01, state_dtype=sdt)
    runs, ws_bytes = [], []
    for schedule in (A.APOLLO_SCHEDULE_CHUNKED, A.APOLLO_SCHEDULE_SERIAL):
        cfg, _ = make_configs(wl)
        cfg.schedule = schedule
        weights = WL.make_weights(wl, DEV)
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        ws_bytes.append(st.workspace.numel())
        snaps = []
        for t in range(1, wl.steps + 1):
            WL.make_grads(wl, t, DEV, out=grads)
            st.step(t, wl.lr)
            torch.cuda.synchronize()
            snaps.append([w.clone() for w in weights] + [st.state.clone(), st.debug(1, A.APOLLO_DBG_R), st.debug(4, A.APOLLO_DBG_R)])
        st.close()
        runs.append(snaps)
    assert ws_bytes[0] < ws_bytes[1] or rank == 1        # (rank 1 has no scratch copy of P under any schedule)
    for a, b in zip(*runs):
        for x, y in zip(a, b):
            assert torch.equal(x, y)


def test_projection_scratch_follows_jumps_of_the_step_number():
    """The generated P stays in the workspace within a refresh interval and is re-generated when
    the step's interval differs from the one held: a handle that is stepped 1, 2, 7, 3, 8 (T = 3:
    intervals 0, 0, 2, 0, 2) must produce, at every step, exactly the R of a fresh handle that is
    given only that step."""
    shapes = [(128, 512), (512, 128)]
    wl = WL.Workload("jumps", 15, shapes, torch.bfloat16, "normal", 1e-2, rank=32, refresh_interval=3, steps=1, lr=1e-3)
    cfg, _ = make_configs(wl)
    weights = WL.make_weights(wl, DEV)
    grads = WL.make_grads(wl, 1, DEV)
    jumpy = A.ApolloStepper(cfg, [w.clone() for w in weights], grads, device=DEV)
    for t in (1, 2, 7, 3, 8):
        jumpy.step(t, wl.lr)
        fresh = A.ApolloStepper(cfg, [w.clone() for w in weights], grads, device=DEV)
        fresh.step(t, wl.lr)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            assert torch.equal(jumpy.debug(i, A.APOLLO_DBG_R), fresh.debug(i, A.APOLLO_DBG_R)), (t, i)
        fresh.close()
    # a step on another stream re-generates too (the copy was written in the first stream's order)
    other = torch.cuda.Stream(device=DEV)
    other.wait_stream(torch.cuda.current_stream(DEV))
    rc = A.apollo_step(jumpy.handle, jumpy._tensors, 8, wl.lr, other.cuda_stream)
    assert rc == A.APOLLO_OK
    other.synchronize()
    fresh = A.ApolloStepper(cfg, [w.clone() for w in weights], grads, device=DEV)
    fresh.step(8, wl.lr)
    torch.cuda.synchronize()
    assert torch.equal(jumpy.debug(0, A.APOLLO_DBG_R), fresh.debug(0, A.APOLLO_DBG_R))
    jumpy.close()
    fresh.close()


@pytest.mark.parametrize("grad_scale", [1e-17, 1e-13, 1e-8, 1e4, 1e15])
@pytest.mark.parametrize("mode,rank,scale", [("channel", 32, 1.0), ("tensor", 1, math.sqrt(128.0))])
def test_gradient_scales_far_from_one(grad_scale, mode, rank, scale):
    """Adam's normalisation makes the update independent of the gradient's scale; the fp32
    arithmetic has to carry that over the range bf16 gradients can take (squares of 1e-17 gradients
    are 1e-34, those of 1e15 gradients 1e30: both still inside fp32's range; for small gradients
    eps = 1e-8 is no longer negligible against sqrt(V), which the oracle models as well)."""
    shapes = [(64, 264), (264, 64), (128, 520)]
    wl = WL.Workload("scale_%g_%s" % (grad_scale, mode), 14, shapes, torch.bfloat16, "normal", grad_scale, rank=rank,
                     mode=mode, scale=scale, refresh_interval=2, steps=4, lr=1e-2, weight_decay=0.01)
    run_parity(wl, list(range(len(shapes))), wl.steps)


def test_thousands_of_small_tensors():
    """A long tensor list (the descriptor table, the tensor index in the grid and in the random
    stream's counter): 6000 small tensors of three shapes, the oracle following a few from the
    beginning, the middle and the end."""
    shapes = [(8, 16), (40, 8), (64, 264)] * 2000
    wl = WL.Workload("many_small", 15, shapes, torch.bfloat16, "normal", 1e-2, rank=4, refresh_interval=2, steps=3,
                     lr=1e-2)
    ids = [0, 1, 2, 2999, 3000, 3001, 5997, 5998, 5999]
    run_parity(wl, ids, wl.steps)
    # and a count per shape that is not a multiple of the eight XCDs, through the matrix-core projection
    shapes = [(64, 264), (264, 64)] * 1501 + [(64, 264)]
    wl = WL.Workload("many_small_r32", 16, shapes, torch.bfloat16, "normal", 1e-2, rank=32, refresh_interval=2,
                     steps=2, lr=1e-2)
    run_parity(wl, [0, 1, 1500, 1501, 3000, 3001, 3002], wl.steps)


def test_matrix_core_projection_at_rank_1024():
    """Four row tiles of 256 per channel tile (they share a tile of G on one XCD), the rank equal to
    the projected dimension of the smaller tensors."""
    shapes = [(1024, 1280), (1280, 1024), (2048, 1032)]
    wl = WL.Workload("mfma_r1024", 17, shapes, torch.bfloat16, "normal", 1e-2, rank=1024, refresh_interval=2,
                     steps=3, lr=1e-2)
    run_parity(wl, list(range(len(shapes))), wl.steps)


@pytest.mark.parametrize("name,steps", [("single256", 10), ("llama60m", 12)])
def test_weights_follow_an_independent_oracle_trajectory(name, steps):
    """The other parity runs start every step from the library's weights; here the oracle carries its
    own W from step 0 through all steps, with weight decay on (the decay term reads W), and the final
    weights must agree within the accumulated per-step bounds: config 1 with all its 10 steps (fp32,
    two re-samplings of P) and 12 steps of the LLaMA-60M set."""
    wl = WL.workload(name)
    wl.weight_decay = 0.1
    wl.name = name + "_independent_w"
    ids = [0] if name == "single256" else _first_and_last_layer(wl)
    stats = {}
    run_parity(wl, ids, steps, independent_w=True, stats=stats)
    assert 0.0 < stats["used"]["W_final"] <= 1.0


def test_non_finite_gradient_keeps_the_stored_norm_and_nan_survives_bf16_storage():
    """A step whose gradient holds an inf: the stored norm stays what it was (the oracle's reading:
    a non-finite norm is not remembered), and with bfloat16 weights the poisoned weights read back as
    NaN -- the rounding to bfloat16 must not turn a NaN into a finite number or a zero."""
    shapes = [(64, 264), (264, 64)]
    for rank, mode in ((32, "channel"), (1, "tensor")):
        wl = WL.Workload("nonfinite", 18, shapes, torch.bfloat16, "normal", 1e-2, rank=rank, mode=mode, refresh_interval=10,
                         steps=2, lr=1e-2, weight_dtype=torch.bfloat16)
        cfg, _ = make_configs(wl)
        weights = WL.make_weights(wl, DEV)
        grads = WL.make_grads(wl, 1, DEV)
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        st.step(1, wl.lr)
        kept = [float(st.debug(i, A.APOLLO_DBG_NORM)[0]) for i in range(2)]
        assert all(k > 0 and math.isfinite(k) for k in kept)
        for g in grads:
            g[3, 5] = float("inf")
        st.step(2, wl.lr)
        torch.cuda.synchronize()
        for i in range(2):
            assert float(st.debug(i, A.APOLLO_DBG_NORM)[0]) == kept[i]
            w = weights[i].float()
            assert bool(torch.isnan(w).any()) and not bool(torch.isinf(w).any())
        st.close()


def test_the_stepper_follows_the_current_stream_at_every_call():
    """The binding looks torch's current stream up per call: a stepper created on the default stream
    and stepped inside `with torch.cuda.stream(other)` runs on `other`, ordered after the gradients
    written there, and gives bit for bit what the same steps give on the default stream."""
    wl = WL.Workload("streams", 19, [(128, 512), (512, 128), (96, 200)], torch.bfloat16, "normal", 1e-2, rank=32,
                     refresh_interval=2, steps=4, lr=1e-2)
    cfg, _ = make_configs(wl)
    outs = []
    for use_other in (False, True):
        weights = WL.make_weights(wl, DEV)
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=DEV)
        torch.cuda.synchronize()
        other = torch.cuda.Stream(device=DEV)
        for t in range(1, wl.steps + 1):
            if use_other and t % 2 == 0:
                other.wait_stream(torch.cuda.current_stream(DEV))
                with torch.cuda.stream(other):
                    WL.make_grads(wl, t, DEV, out=grads)
                    st.step(t, wl.lr)                # no synchronisation in between: stream order must do
                torch.cuda.current_stream(DEV).wait_stream(other)
            else:
                WL.make_grads(wl, t, DEV, out=grads)
                st.step(t, wl.lr)
        torch.cuda.synchronize()
        outs.append([w.clone() for w in weights] + [st.state.clone()])
        st.close()
    for x, y in zip(*outs):
        assert torch.equal(x, y)
