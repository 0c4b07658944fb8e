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
    ("llama1b_mini", 3),            # rank 1 on rows of 5461 elements (unaligned 16-byte accesses, ragged last octet)
    ("llama7b_mini", 3),
    ("llama7b_r256", 2),
    ("llama13b_mini", 2),
    ("llama13b_r256", 2),
    ("llama7b_mini_bf16", 2),       # bfloat16 W and moments (valid-rounding checks)
    ("llama7b_r256_bf16", 2),
    ("llama7b_identity", 2),        # the structured rule without projection: full-rank moments
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


@pytest.mark.parametrize("shape,rank", [((2048, 589824), 64), ((589824, 2048), 64), ((2048, 589824), 1),
                                        ((589824, 2048), 1)])
def test_one_tensor_beyond_four_gibibytes_on_sampled_channels(shape, rank):
    """A single tensor of 1.2 G elements (W 4.8 GB, G 2.4 GB: element and byte offsets beyond 2^31 and
    2^32, channel counts far above any LLaMA shape), both orientations, matrix-core and rank-1
    projection.  With channel-wise factors and the limiter off every channel is independent of the
    others, so the oracle steps a sub-tensor made of sampled channels (same seed, tensor index and
    projected dimension, hence the same P) and must agree with those channels of the big one."""
    import numpy as np
    import paper_2412_05270_amd as A
    from oracle import apollo as O
    from parity_util import E_IN_BF16, TOL_BF16, assert_close, condition_factors, f32, make_configs, to_host_f64
    dev = "cuda:0"
    rows, cols = shape
    left = rows <= cols
    n = cols if left else rows
    wl = WL.Workload("huge_%dx%d_r%d" % (rows, cols, rank), 61, [shape], torch.bfloat16, "normal", 1e-2, rank=rank,
                     refresh_interval=200, steps=2, lr=1e-2, weight_decay=0.01, nl_gamma=0.0)
    cfg, ocfg = make_configs(wl, side="left" if left else "right")
    gen = torch.Generator(device=dev)
    gen.manual_seed(6100 + rank + rows % 7)
    W = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
    W *= wl.w_std
    G = torch.empty(shape, device=dev, dtype=torch.bfloat16)
    rng = np.random.default_rng(5)
    J = np.unique(np.concatenate([[0, 1, 2, 3, 254, 255, 256, 257, n - 258, n - 257, n - 256, n - 255, n - 2, n - 1],
                                  rng.integers(0, n, size=114)]))
    Jd = torch.as_tensor(J, device=dev)
    take = (lambda x: x[:, Jd]) if left else (lambda x: x[Jd, :])
    st = A.ApolloStepper(cfg, [W], [G], device=dev)
    state = O.init_state(ocfg, *((rows, len(J)) if left else (len(J), cols)))
    tol = TOL_BF16
    cf_acc = {}
    for t in (1, 2):
        for r0 in range(0, rows, 65536):              # gradients in slabs: no second 4.8 GB temporary
            r1 = min(rows, r0 + 65536)
            G[r0:r1] = (torch.randn((r1 - r0, cols), generator=gen, device=dev, dtype=torch.float32) * wl.grad_scale).to(torch.bfloat16)
        before = to_host_f64(take(W))
        st.step(t, wl.lr)
        torch.cuda.synchronize()
        W_sub = before.copy()
        info = O.step(ocfg, state, W_sub, to_host_f64(take(G)), t, f32(wl.lr), tensor_id=0, grad_is_bf16=True)
        f_chan, _ = condition_factors(info, state, ocfg, t, tol, E_IN_BF16, cf_acc)
        if rank >= 32:
            f_chan = np.ones_like(f_chan)        # rank 64: the stated tolerance itself
        tag = "%s step %d " % (wl.name, t)
        assert_close(tag + "colsq", to_host_f64(st.debug(0, A.APOLLO_DBG_COLSQ)[Jd]), info["colsq"], tol)
        assert_close(tag + "R", to_host_f64(st.debug(0, A.APOLLO_DBG_R)[:, Jd]), info["R"], tol)
        assert_close(tag + "M", to_host_f64(st.debug(0, A.APOLLO_DBG_M)[:, Jd]), state.M, tol)
        assert_close(tag + "V", to_host_f64(st.debug(0, A.APOLLO_DBG_V)[:, Jd]), state.V, tol)
        assert_close(tag + "s", to_host_f64(st.debug(0, A.APOLLO_DBG_S)[Jd]), info["s"], 0.0,
                     extra_abs=tol * f_chan * np.abs(info["s"]))
        after = to_host_f64(take(W))
        dw_ref = W_sub - before
        f_dw = f_chan[None, :] if left else f_chan[:, None]
        rms_dw = float(np.sqrt(np.mean(dw_ref * dw_ref)))
        assert_close(tag + "dW", after - before, dw_ref, 0.0,
                     extra_abs=tol * f_dw * (np.abs(dw_ref) + rms_dw) + np.abs(after) * 2.0 ** -24)
        print("%s: step %d compared on %d channels" % (wl.name, t, len(J)), flush=True)
    st.close()
    del W, G, st
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["llama7b_mini", "llama7b_r256", "llama1b", "llama1b_mini", "llama7b_identity"])
def test_every_tensor_of_a_full_set_at_step_one(name):
    """The recurrence of the oracle follows a handful of tensors of a full-size set; this covers ALL of
    them, every element, for the first step, where Algorithm 1 has a short closed form
    (oracle.apollo.first_step_closed_form, pinned on the CPU against the recurrence).  The oracle's
    function is evaluated in fp64 on the device arrays (its torch namespace) and compared under the
    same tolerance.  P is the oracle's own (generated on the host) for every tensor at rank 1 and for
    every ninth tensor otherwise (all three shapes, layers from the first to the last); for the others
    it is the library's generator view, which is compared bit for bit with the oracle's elsewhere.  It
    catches what depends on a tensor's position in the list."""
    import numpy as np
    import paper_2412_05270_amd as A
    from oracle import apollo as O
    from oracle import gauss
    from parity_util import TOL_BF16, f32, make_configs
    dev = "cuda:0"
    wl = WL.workload(name)
    cfg, ocfg = make_configs(wl)
    tol = TOL_BF16
    weights = WL.make_weights(wl, dev)
    grads = WL.make_grads(wl, 1, dev)
    before = [w.clone() for w in weights]
    st = A.ApolloStepper(cfg, weights, grads, device=dev)
    st.step(1, wl.lr)
    torch.cuda.synchronize()
    identity = wl.projection == "identity"

    def check(tag, got, ref, extra=0.0):
        got, ref = got.double(), torch.as_tensor(ref, device=dev, dtype=torch.float64).reshape(got.shape)
        rms = float(ref.pow(2).mean().sqrt())
        bad = (got - ref).abs() > tol * (ref.abs() + rms) + extra
        assert not bool(bad.any()), "%s: %d of %d elements off" % (tag, int(bad.sum()), bad.numel())

    own_p = 0
    for i, (rows, cols) in enumerate(wl.shapes):
        left = rows <= cols
        z = None
        if not identity:
            if wl.rank == 1 or i % 9 == 0:
                z = torch.from_numpy(gauss.projection(ocfg.seed, i, 0, wl.rank, min(rows, cols), True)).to(dev)
                own_p += 1
            else:
                z = st.projection(i, 1, True).double()
        cf = O.first_step_closed_form(ocfg, grads[i].double(), f32(wl.lr), z=z, xp=torch)
        tag = "%s tensor %d " % (name, i)
        own = (lambda x: x) if (left or not identity) else (lambda x: x.t())   # full-rank moments: the tensor's layout
        if not identity:
            check(tag + "R", st.debug(i, A.APOLLO_DBG_R), cf["R"])
        check(tag + "colsq", st.debug(i, A.APOLLO_DBG_COLSQ), cf["colsq"])
        check(tag + "M", st.debug(i, A.APOLLO_DBG_M), own(cf["M"]))
        check(tag + "V", st.debug(i, A.APOLLO_DBG_V), own(cf["V"]))
        check(tag + "s", st.debug(i, A.APOLLO_DBG_S), cf["s"][:1] if wl.mode == "tensor" else cf["s"])
        check(tag + "norm", st.debug(i, A.APOLLO_DBG_NORM), cf["norm"].reshape(1))
        check(tag + "c", st.debug(i, A.APOLLO_DBG_C), [cf["c"]])
        check(tag + "dW", weights[i].double() - before[i].double(), cf["dW_grad"], extra=weights[i].double().abs() * 2.0 ** -24)
        del cf, z
        if i % 56 == 55:
            print("%s: %d tensors compared (%d with the oracle's own P)" % (name, i + 1, own_p), flush=True)
    assert identity or own_p >= len(wl.shapes) // 9
    st.close()
    del weights, grads, before, st
    torch.cuda.empty_cache()


def test_chunked_schedule_at_full_size_equals_the_serial_one():
    """APOLLO_SCHEDULE_CHUNKED on the LLaMA-7B matrices at rank 256: the groups of 128 and 64 tensors are
    worked through in chunks of 64 (128 MiB of P), every chunk's P generated over the same scratch.  Steps
    200 and 201 (a re-sampling between them): every weight tensor and the whole state must carry the same
    bits as after the serial schedule (compared through exact integer fingerprints), with a quarter of
    the workspace."""
    import paper_2412_05270_amd as A
    from parity_util import make_configs
    dev = "cuda:0"
    wl = WL.workload("llama7b_r256")

    def fingerprint(x):
        return int(x.contiguous().view(torch.int32).to(torch.int64).sum())
    prints, ws = [], []
    for schedule in (A.APOLLO_SCHEDULE_SERIAL, A.APOLLO_SCHEDULE_CHUNKED):
        cfg, _ = make_configs(wl)
        cfg.schedule = schedule
        weights = WL.make_weights(wl, dev)
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=dev) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=dev)
        ws.append(st.workspace.numel())
        got = []
        for t in (200, 201):
            WL.make_grads(wl, t, dev, out=grads)
            st.step(t, wl.lr)
            torch.cuda.synchronize()
            got.append([fingerprint(w) for w in weights] + [fingerprint(st.state)])
        prints.append(got)
        st.close()
        del weights, grads, st
        torch.cuda.empty_cache()
    assert prints[0] == prints[1]
    assert ws[1] * 3 < ws[0]


def test_full_size_sets_run_on_the_kernels_meant_for_them():
    """No silent fallback: every tensor of the benchmark's sets is served by the projection kernel
    written for it (the library reports its choice per tensor)."""
    import paper_2412_05270_amd as A
    from parity_util import make_configs
    dev = "cuda:0"
    expect = {"llama60m": A.APOLLO_PATH_MATRIX_CORE, "llama1b": A.APOLLO_PATH_MATRIX_CORE,
              "llama1b_mini": A.APOLLO_PATH_RANK1,
              "llama7b_mini": A.APOLLO_PATH_RANK1, "llama7b_r256": A.APOLLO_PATH_MATRIX_CORE,
              "llama13b_mini": A.APOLLO_PATH_RANK1, "llama13b_r256": A.APOLLO_PATH_MATRIX_CORE,
              "llama7b_mini_q8": A.APOLLO_PATH_RANK1, "llama7b_identity": A.APOLLO_PATH_NONE,
              "single256": A.APOLLO_PATH_GENERAL}
    for name, path in expect.items():
        wl = WL.workload(name)
        cfg, _ = make_configs(wl)
        weights = [torch.empty(s, dtype=wl.weight_dtype, device=dev) for s in wl.shapes]
        grads = [torch.empty(s, dtype=wl.grad_dtype, device=dev) for s in wl.shapes]
        metas = None
        if wl.weight_dtype == torch.uint8:
            metas = [torch.empty((s[0] * s[1] // 128, 2), dtype=torch.float32, device=dev) for s in wl.shapes]
        st = A.ApolloStepper(cfg, weights, grads, device=dev, metas=metas)
        for i, (rows, cols) in enumerate(wl.shapes):
            got, padded = st.path(i)
            assert got == path, (name, i, (rows, cols), got)
            # only the 1B set's 2048 x 5461 tensors (rows projected, odd row length) need the padded copy
            assert padded == int(name == "llama1b" and (rows, cols) == (2048, 5461)), (name, i, (rows, cols), padded)
        st.close()
        del weights, grads, metas, st
        torch.cuda.empty_cache()


def test_every_tensor_of_the_full_8bit_set_at_step_one():
    """All 224 tensors of the 8-bit set (nearest rounding, where the offsets are a constant), first
    step, every group and element, against the oracle's definitions evaluated in fp64 on the device
    arrays: the de-quantised weights (oracle.q8.dequantise_values), the first step's update in closed
    form with the oracle's own rank-1 projection (oracle.apollo.first_step_closed_form), and the range
    and code positions of every group (oracle.q8.group_positions).  The new (scale, zero) of a group
    must be its range / 255 and its minimum, every code floor(x + 1/2) of its position x; a code whose
    x + 1/2 lies within 1e-3 of an integer may go either way."""
    import paper_2412_05270_amd as A
    from oracle import apollo as O
    from oracle import gauss, q8
    from parity_util import f32, make_configs
    dev = "cuda:0"
    wl = WL.workload("llama7b_mini_q8_nearest")
    cfg, ocfg = make_configs(wl)
    codes, metas = WL.make_q8_weights(wl, dev)
    grads = WL.make_grads(wl, 1, dev)
    before = [(c.clone(), m.clone()) for c, m in zip(codes, metas)]
    st = A.ApolloStepper(cfg, codes, grads, device=dev, metas=metas)
    lr = 3e-3                      # moves a typical weight by about one code step
    st.step(1, lr)
    torch.cuda.synchronize()
    moved = 0
    for i, (rows, cols) in enumerate(wl.shapes):
        c0, m0 = before[i]
        groups = cols // 128
        w = q8.dequantise_values(c0.double(), m0[:, 0].double().reshape(rows, groups), m0[:, 1].double().reshape(rows, groups))
        z = torch.from_numpy(gauss.projection(ocfg.seed, i, 0, 1, min(rows, cols), True)).to(dev)
        cf = O.first_step_closed_form(ocfg, grads[i].double(), f32(lr), z=z, xp=torch)
        wn = w + cf["dW_grad"]                                   # no weight decay in this workload
        lo, hi, x = q8.group_positions(wn, xp=torch)
        rng = hi - lo
        tag = "tensor %d " % i
        slack = (wn.abs().reshape(rows, groups, 128).max(dim=2).values + w.abs().reshape(rows, groups, 128).max(dim=2).values) * 2.0 ** -21
        new_scale, new_zero = metas[i][:, 0].double().reshape(rows, groups), metas[i][:, 1].double().reshape(rows, groups)
        assert bool(((new_zero - lo).abs() <= slack).all()), tag + "zero"
        assert bool(((new_scale - rng / 255.0).abs() <= slack / 255.0 + rng * 1e-6).all()), tag + "scale"
        got = codes[i].double()
        lo_c = torch.clamp(torch.floor(x + 0.5 - 1e-3), 0, 255)
        hi_c = torch.clamp(torch.floor(x + 0.5 + 1e-3), 0, 255)
        bad = (got < lo_c) | (got > hi_c)
        assert not bool(bad.any()), tag + "%d codes outside their interval" % int(bad.sum())
        assert float((lo_c == hi_c).double().mean()) > 0.99, tag + "intervals too wide"
        moved += int((got != c0.double()).sum())
        del w, wn, x, got, lo_c, hi_c, cf
        if i % 56 == 55:
            print("llama7b_mini_q8_nearest: %d tensors compared" % (i + 1), flush=True)
    assert moved > wl.n_params // 4          # the step did change the codes
    st.close()
    del codes, metas, grads, before, st
    torch.cuda.empty_cache()
