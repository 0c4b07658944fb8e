"""The comparison the GPU parity tests apply, checked on the CPU against planted errors: the oracle
steps one LLaMA-7B attention matrix at rank 256 (no GPU, no library call), a copy of its results
plays the part of the library, and an error of five times the tolerance on ONE channel's factor, on
one element of the moments or on one element of the weight change must fail the comparison -- while
the unperturbed copy passes with the bound on that configuration being the stated tolerance itself
(no per-channel widening)."""
import numpy as np
import pytest
import torch

from oracle import apollo as O
from paper_2412_05270_amd import workloads as WL
from parity_util import E_IN_BF16, TOL_BF16, assert_close, condition_factors, make_configs, plain_tolerance_applies


@pytest.fixture(scope="module")
def stepped():
    wl = WL.workload("llama7b_r256")
    _, ocfg = make_configs(wl)
    rows, cols = wl.shapes[0]
    rng = np.random.default_rng(4)
    G = torch.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32) * 1e-3).to(torch.bfloat16).float().double().numpy()
    W = rng.standard_normal((rows, cols)) * 0.02
    state = O.init_state(ocfg, rows, cols)
    W0 = W.copy()
    info = O.step(ocfg, state, W, G, 1, float(np.float32(wl.lr)), tensor_id=0, grad_is_bf16=True)
    return wl, ocfg, state, info, W - W0


def test_rank_256_is_held_to_the_plain_tolerance(stepped):
    wl, ocfg, state, info, dW = stepped
    assert plain_tolerance_applies(wl)
    assert plain_tolerance_applies(WL.workload("llama7b_mini")) and plain_tolerance_applies(WL.workload("llama1b"))
    assert not plain_tolerance_applies(WL.Workload("r1c", 1, [(8, 8)], torch.bfloat16, "normal", 1e-2, rank=1))
    # the propagated-error factors would have widened next to nothing here either
    f_chan, f_norm = condition_factors(info, state, ocfg, 1, TOL_BF16, E_IN_BF16, {})
    assert np.mean(f_chan > 1.0) < 0.02 and f_chan.max() < 20.0 and f_norm < 1.1


def test_an_error_of_five_tolerances_on_one_channel_fails(stepped):
    wl, ocfg, state, info, dW = stepped
    tol = TOL_BF16
    s = info["s"]
    assert assert_close("s", s.copy(), s, 0.0, extra_abs=tol * np.abs(s)) == 0.0
    bad = s.copy()
    bad[1234] *= 1.0 + 5.0 * tol
    with pytest.raises(AssertionError, match="1 of 4096 elements off"):
        assert_close("s", bad, s, 0.0, extra_abs=tol * np.abs(s))
    # the same mistake as it shows in the weights: every element of that channel's column moves by 5 tol
    rms = float(np.sqrt(np.mean(dW * dW)))
    bad_dw = dW.copy()
    bad_dw[:, 1234] *= 1.0 + 5.0 * tol
    with pytest.raises(AssertionError):
        assert_close("dW", bad_dw, dW, 0.0, extra_abs=tol * (np.abs(dW) + rms) * 0.0 + tol * np.abs(dW))
    # one element of a moment off by 5 tol of (|x| + rms)
    M = state.M
    rms_m = float(np.sqrt(np.mean(M * M)))
    bad_m = M.copy()
    bad_m[17, 99] += 5.0 * tol * (abs(M[17, 99]) + rms_m)
    with pytest.raises(AssertionError, match="1 of"):
        assert_close("M", bad_m, M, tol)
    assert assert_close("M", M.copy(), M, tol) == 0.0
