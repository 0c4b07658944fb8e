"""GPU parity of the step on group-wise 8-bit weights (APOLLO_Q8) against the oracle, through the
C ABI, in two stages.  (1) The moments, the factors s, the limiter factor c and the norm are held to
the usual tolerances.  (2) The oracle then adopts the library's s and c (step(adopt_factors=)) and
the new codes, scales and zero points are compared on identical real-valued inputs: codes are
integers decided by floating-point arithmetic, so with x the oracle's real-valued code position, u
the (bit-identical) rounding offset and dx the binary32 rounding error of x, a stored code must lie
in [floor(x - dx + u), floor(x + dx + u)].  Every step starts both sides from the library's stored
codes."""
import math

import numpy as np
import pytest
import torch

import paper_2412_05270_amd as A
from oracle import apollo as O
from oracle import q8 as Q
from paper_2412_05270_amd import workloads as WL
from parity_util import (E_IN_BF16, E_IN_F32, TOL_BF16, TOL_F32, assert_close, assert_rounds_within, condition_factors, f32, make_configs,
                         to_host_f64)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(wl, steps, lr, check_ids=None, progress=False):
    bf16 = wl.grad_dtype == torch.bfloat16
    tol = TOL_BF16 if bf16 else TOL_F32
    cfg, ocfg = make_configs(wl)
    state_bf16 = wl.state_dtype == torch.bfloat16
    cf_acc = {}
    if check_ids is None:
        # initial weights: N(0, w_std^2) quantised on the host (nearest)
        check_ids = list(range(len(wl.shapes)))
        w0 = [to_host_f64(w) for w in WL.make_weights(WL.Workload(wl.name, wl.config_id, wl.shapes, wl.grad_dtype,
                                                                   wl.grad_kind, wl.grad_scale), DEV)]
        codes, metas = [], []
        for w in w0:
            q, _ = Q.quantise(w, np.full(w.shape, 0.5))
            codes.append(torch.from_numpy(q.codes).to(DEV))
            metas.append(torch.from_numpy(np.stack([q.scale, q.zero], axis=-1).reshape(-1, 2).astype(np.float32)).to(DEV))
    else:
        codes, metas = WL.make_q8_weights(wl, DEV)     # the benchmark's synthetic codes and ranges
    grads = [torch.empty(s, dtype=wl.grad_dtype, device=DEV) for s in wl.shapes]
    st = A.ApolloStepper(cfg, codes, grads, device=DEV, metas=metas)
    states = {i: O.init_state(ocfg, *wl.shapes[i]) for i in check_ids}
    moved = 0
    for t in range(1, steps + 1):
        WL.make_grads(wl, t, DEV, out=grads)
        before = {}
        for i in check_ids:
            rows, cols = wl.shapes[i]
            mt = metas[i].double().cpu().numpy().reshape(rows, cols // 128, 2)
            before[i] = Q.Q8Weights(codes[i].cpu().numpy().copy(), mt[:, :, 0].copy(), mt[:, :, 1].copy())
        st.step(t, lr)
        torch.cuda.synchronize()
        if progress:
            print("%s: step %d/%d done, comparing" % (wl.name, t, steps), flush=True)
        for i in check_ids:
            rows, cols = wl.shapes[i]
            tag = "%s tensor %d step %d " % (wl.name, i, t)
            Wq = before[i]
            w_before = Wq.dequantise()
            old_codes = Wq.codes.copy()
            s_gpu = to_host_f64(st.debug(i, A.APOLLO_DBG_S))
            c_gpu = float(to_host_f64(st.debug(i, A.APOLLO_DBG_C))[0])
            n_ch = max(rows, cols)
            adopt = lambda s, c, s_gpu=s_gpu, c_gpu=c_gpu, n_ch=n_ch: (
                s_gpu if wl.mode == "channel" else np.full(n_ch, s_gpu[0]), c_gpu)
            adopt_mv = None
            if state_bf16:
                # bfloat16 moments: the library's roundings are checked against the oracle's unrounded
                # values and then adopted (as in the bfloat16-storage tests)
                M_gpu, V_gpu = to_host_f64(st.debug(i, A.APOLLO_DBG_M)), to_host_f64(st.debug(i, A.APOLLO_DBG_V))

                def adopt_mv(M_exact, V_exact, M_gpu=M_gpu, V_gpu=V_gpu, tag=tag):
                    assert_rounds_within(tag + "M", M_gpu, M_exact, tol)
                    assert_rounds_within(tag + "V", V_gpu, V_exact, tol)
                    return M_gpu, V_gpu
            info = O.step(ocfg, states[i], Wq, to_host_f64(grads[i]), t, f32(lr), tensor_id=i, grad_is_bf16=bf16,
                          adopt_factors=adopt, adopt_moments=adopt_mv)
            f_chan, f_norm = condition_factors(info, states[i], ocfg, t, tol, E_IN_BF16 if bf16 else E_IN_F32,
                                               cf_acc.setdefault(i, {}), moments_adopted=state_bf16)
            if not state_bf16:
                assert_close(tag + "M", to_host_f64(st.debug(i, A.APOLLO_DBG_M)), states[i].M, tol)
                assert_close(tag + "V", to_host_f64(st.debug(i, A.APOLLO_DBG_V)), states[i].V, tol)
            s_ref = info["s"] if wl.mode == "channel" else info["s"][:1]
            f_s = f_chan if wl.mode == "channel" else f_chan[:1]
            assert_close(tag + "s", s_gpu, s_ref, 0.0, extra_abs=tol * f_s * np.abs(s_ref))
            assert_close(tag + "norm", to_host_f64(st.debug(i, A.APOLLO_DBG_NORM)), [info["norm"]], tol * f_norm)
            assert_close(tag + "c", [c_gpu], [info["c"]], tol * (f_norm + 1.0))
            # with the factors adopted, what is left is binary32 rounding: of the de-quantised weight,
            # of the update term and of their difference
            dw = info["W_exact"] - w_before
            d = (np.abs(info["W_exact"]) + np.abs(w_before) + np.abs(dw)) * 2.0 ** -22
            dg = d.reshape(rows, cols // 128, 128).max(axis=2)
            mt = metas[i].double().cpu().numpy().reshape(rows, cols // 128, 2)
            scale_gpu, zero_gpu = mt[:, :, 0], mt[:, :, 1]
            assert np.all(np.abs(zero_gpu - Wq.zero) <= dg + 1e-30), tag + "zero"
            assert np.all(np.abs(scale_gpu - Wq.scale) <= 2 * dg / 255 + 1e-6 * Wq.scale + 1e-30), tag + "scale"
            with np.errstate(divide="ignore", invalid="ignore"):
                dx = np.where(Wq.scale > 0, 4 * dg / Wq.scale, 0.0) + 1e-3
            dx = np.repeat(dx, 128, axis=1)
            lo = np.clip(np.floor(info["q8_x"] - dx + info["q8_u"]), 0, 255)
            hi = np.clip(np.floor(info["q8_x"] + dx + info["q8_u"]), 0, 255)
            got = codes[i].cpu().numpy().astype(np.float64)
            bad = (got < lo) | (got > hi)
            assert not bad.any(), "%scodes: %d of %d outside their admissible interval" % (tag, int(bad.sum()), bad.size)
            # the check has teeth: all but a few per mille of the codes are pinned to a single value
            assert np.mean(lo == hi) > 0.99, tag + "intervals too wide: %.4f" % float(np.mean(lo == hi))
            moved += int(np.sum(got != old_codes))
    st.close()
    return moved


SHAPES = [(64, 256), (256, 128), (128, 384), (384, 128), (256, 256)]


@pytest.mark.parametrize("rounding", ["nearest", "stochastic"])
def test_channel_wise_q8_weights(rounding):
    wl = WL.Workload("q8_r32_" + rounding, 51, SHAPES, torch.bfloat16, "normal", 1e-2, rank=32, refresh_interval=3,
                     steps=5, lr=5e-4, weight_decay=0.05, weight_dtype=torch.uint8, weight_rounding=rounding)
    assert _run(wl, wl.steps, wl.lr) > 0


@pytest.mark.parametrize("rounding", ["nearest", "stochastic"])
def test_mini_q8_weights_fp32_gradients(rounding):
    wl = WL.Workload("q8_mini_" + rounding, 52, SHAPES, torch.float32, "normal", 1e-2, rank=1, mode="tensor",
                     scale=math.sqrt(128.0), refresh_interval=3, steps=5, lr=5e-5, weight_dtype=torch.uint8,
                     weight_rounding=rounding)
    assert _run(wl, wl.steps, wl.lr) > 0


def test_q8_weights_with_bfloat16_moments():
    """The paper's low-memory setting: 8-bit weights together with optimizer states in bfloat16."""
    wl = WL.Workload("q8_bf16_state", 53, SHAPES, torch.bfloat16, "normal", 1e-2, rank=32, refresh_interval=3,
                     steps=4, lr=5e-4, weight_dtype=torch.uint8, weight_rounding="stochastic",
                     state_dtype=torch.bfloat16)
    assert _run(wl, wl.steps, wl.lr) > 0


def test_small_updates_survive_only_with_stochastic_rounding():
    """With a learning rate that moves a weight by ~5 % of a code step, nearest rounding changes
    hardly any code while stochastic rounding changes about that fraction of them, every step."""
    moved = {}
    for rounding in ("nearest", "stochastic"):
        wl = WL.Workload("q8_small_" + rounding, 53, [(256, 256)], torch.bfloat16, "normal", 1e-2, rank=1, mode="tensor",
                         scale=1.0, refresh_interval=100, steps=4, lr=3e-5, weight_dtype=torch.uint8,
                         weight_rounding=rounding)
        moved[rounding] = _run(wl, wl.steps, wl.lr)
    assert moved["stochastic"] > 20 * max(1, moved["nearest"])


def test_q8_argument_checks():
    cfg = A.ApolloConfig(rank=4, mode=A.APOLLO_CHANNEL, seed=1, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                         weight_decay=0.0, nl_gamma=1.01, refresh_interval=10, bias_correction=1, side=0,
                         weight_dtype=A.APOLLO_Q8)
    assert A.apollo_state_bytes(cfg, [(64, 100, A.APOLLO_BF16)]) == 0
    assert "128" in A.apollo_last_error()
    codes = [torch.zeros(64, 128, dtype=torch.uint8, device=DEV)]
    meta = [torch.zeros(64, 2, device=DEV)]
    g = [torch.zeros(64, 128, dtype=torch.bfloat16, device=DEV)]
    st = A.ApolloStepper(cfg, codes, g, device=DEV, metas=meta)
    assert A.apollo_step(st.handle, [(codes[0].data_ptr(), g[0].data_ptr(), None)], 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step(st.handle, [(codes[0].data_ptr(), g[0].data_ptr(), meta[0].data_ptr() + 4)], 1, 0.1) == A.APOLLO_EINVAL
    st.step(1, 0.1)      # all-zero gradient on an all-zero constant tensor: stays put
    torch.cuda.synchronize()
    assert not codes[0].any() and not meta[0].any()
    st.close()
