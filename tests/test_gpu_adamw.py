"""GPU parity of the element-wise AdamW entry points (through the C ABI) against the fp64 oracle:
W, M and V element by element on seeded inputs.  Tolerance as for the APOLLO step: |x - ref| <=
tol (|ref| + rms ref), tol = 1e-5 with fp32 gradients and 1e-3 with bf16 gradients; the weight
additionally gets half an ulp of its fp32 store."""
import numpy as np
import pytest
import torch

import paper_2412_05270_amd as A
from oracle import adamw as O
from parity_util import TOL_BF16, TOL_F32, assert_close, assert_rounds_within, f32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _configs(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, bias_correction=True):
    cfg = A.ApolloAdamwConfig(beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                              bias_correction=1 if bias_correction else 0, reserved=0)
    ocfg = O.Config(beta1=f32(beta1), beta2=f32(beta2), eps=f32(eps), weight_decay=f32(weight_decay),
                    bias_correction=bias_correction)
    return cfg, ocfg


def _make(sizes, dtypes, seed):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    weights = [torch.randn(n, generator=gen, device=DEV) * 0.02 for n in sizes]
    grads = [torch.empty(n, dtype=dt, device=DEV) for n, dt in zip(sizes, dtypes)]
    return gen, weights, grads


def _fill(gen, grads, scale):
    for g in grads:
        g.copy_((torch.randn(g.numel(), generator=gen, device=DEV) * scale).to(g.dtype))


def _run(sizes, dtypes, steps, lr, seed=3, grad_scale=1e-3, store_bf16=False, **kw):
    cfg, ocfg = _configs(**kw)
    gen, weights, grads = _make(sizes, dtypes, seed)
    if store_bf16:
        weights = [w.to(torch.bfloat16) for w in weights]
        ocfg.store_dtype = "bf16"
    st = A.AdamwStepper(cfg, weights, grads, device=DEV)
    W = [w.double().cpu().numpy() for w in weights]
    ost = [O.init_state(n) for n in sizes]
    for t in range(1, steps + 1):
        _fill(gen, grads, grad_scale * (10.0 if t == 3 else 1.0))
        before = [w.double().cpu().numpy() for w in weights]
        st.step(t, lr)
        torch.cuda.synchronize()
        for i in range(len(sizes)):
            tol = TOL_BF16 if dtypes[i] == torch.bfloat16 else TOL_F32
            W[i] = before[i].copy()      # each step starts from the library's stored weight
            m, v = st.moments(i)
            if store_bf16:
                # bfloat16 storage: the library's stored moments must be valid roundings of the oracle's
                # unrounded ones; the oracle then continues from them, and the stored weight must be a
                # valid rounding of its unrounded new weight
                m_gpu, v_gpu = m.double().cpu().numpy(), v.double().cpu().numpy()
                tag = "[%d] step %d" % (i, t)

                def adopt(M_exact, V_exact, m_gpu=m_gpu, v_gpu=v_gpu, tag=tag, tol=tol):
                    # (one fused multiply-add per moment: the unrounded values differ by binary32 rounding only)
                    assert_rounds_within("M" + tag, m_gpu, M_exact, 1e-6, min_pinned=0.9)
                    assert_rounds_within("V" + tag, v_gpu, V_exact, 1e-6, min_pinned=0.9)
                    return m_gpu, v_gpu
                O.step(ocfg, ost[i], W[i], grads[i].double().cpu().numpy(), t, f32(lr), adopt_moments=adopt)
                dw = ost[i].W_exact - before[i]
                rms = float(np.sqrt(np.mean(dw * dw)))
                assert_rounds_within("W" + tag, weights[i].double().cpu().numpy(), ost[i].W_exact, 0.0,
                                     extra_abs=tol * (np.abs(dw) + rms) + np.abs(before[i]) * 2.0 ** -24)
                continue
            O.step(ocfg, ost[i], W[i], grads[i].double().cpu().numpy(), t, f32(lr))
            assert_close("M[%d] step %d" % (i, t), m.double().cpu().numpy(), ost[i].M, tol)
            assert_close("V[%d] step %d" % (i, t), v.double().cpu().numpy(), ost[i].V, tol)
            got = weights[i].double().cpu().numpy()
            ulp = np.abs(before[i]) * 2.0 ** -24
            assert_close("dW[%d] step %d" % (i, t), got - before[i], W[i] - before[i], tol, extra_abs=ulp)
            assert_close("W[%d] step %d" % (i, t), got, W[i], tol)
    st.close()


# sizes around the block (1024 elements) and quad (4 elements) boundaries, one single element,
# a norm-gain sized vector, an embedding-sized slab
SIZES = [1, 3, 4, 5, 1023, 1024, 1025, 4096, 4097, 2051, 1000 * 512 + 3]


def test_fp32_gradients_all_size_classes():
    _run(SIZES, [torch.float32] * len(SIZES), steps=5, lr=1e-3)


def test_bf16_gradients_with_weight_decay():
    _run(SIZES, [torch.bfloat16] * len(SIZES), steps=5, lr=1e-2, weight_decay=0.1)


@pytest.mark.parametrize("gdt", [torch.bfloat16, torch.float32])
def test_bfloat16_storage_of_weights_and_moments(gdt):
    """W, M and V kept in bfloat16 (the paper's all-bfloat16 setting for the non-projected parameters
    too): stored values are checked as valid roundings of the oracle's unrounded ones."""
    _run(SIZES, [gdt] * len(SIZES), 5, 1e-2, seed=9, weight_decay=0.05, store_bf16=True)


def test_mixed_dtypes_without_bias_correction():
    dt = [torch.float32 if i % 2 else torch.bfloat16 for i in range(len(SIZES))]
    _run(SIZES, dt, steps=4, lr=3e-3, bias_correction=False, beta1=0.8, beta2=0.95, eps=1e-6)


def test_llama_7b_sized_embedding_sampled():
    """One 32000 x 4096 embedding (131 M elements, bf16 gradient) and the 65 norm gains of
    LLaMA-7B in one launch; the oracle checks a random sample of the big tensor's elements and
    all of the small ones."""
    cfg, ocfg = _configs(weight_decay=0.01)
    sizes = [32000 * 4096] + [4096] * 65
    gen, weights, grads = _make(sizes, [torch.bfloat16] * len(sizes), 11)
    st = A.AdamwStepper(cfg, weights, grads, device=DEV)
    idx = torch.randint(0, sizes[0], (200_000,), generator=gen, device=DEV)
    idx[:8] = torch.tensor([0, 1, 2, 3, sizes[0] - 4, sizes[0] - 3, sizes[0] - 2, sizes[0] - 1], device=DEV)
    sample = lambda x, i: (x[idx] if i == 0 else x).double().cpu().numpy()
    ost = [O.init_state(idx.numel() if i == 0 else n) for i, n in enumerate(sizes)]
    for t in range(1, 4):
        _fill(gen, grads, 1e-3)
        before = [sample(w, i) for i, w in enumerate(weights)]
        st.step(t, 1e-2)
        torch.cuda.synchronize()
        for i in (0, 1, 65):
            W = before[i].copy()
            O.step(ocfg, ost[i], W, sample(grads[i], i), t, f32(1e-2))
            m, v = st.moments(i)
            assert_close("M", sample(m, i), ost[i].M, TOL_BF16)
            assert_close("V", sample(v, i), ost[i].V, TOL_BF16)
            got = sample(weights[i], i)
            assert_close("dW", got - before[i], W - before[i], TOL_BF16, extra_abs=np.abs(before[i]) * 2.0 ** -24)
    st.close()


def test_resume_and_changed_pointers():
    """A second handle on a copy of the state (zero_state = 0) and on different weight/gradient
    buffers continues exactly like the first."""
    cfg, _ = _configs(weight_decay=0.05)
    sizes = [5000, 777]
    gen, w1, g1 = _make(sizes, [torch.bfloat16, torch.float32], 21)
    a = A.AdamwStepper(cfg, w1, g1, device=DEV)
    for t in (1, 2):
        _fill(gen, g1, 1e-3)
        a.step(t, 1e-2)
    torch.cuda.synchronize()
    w2 = [w.clone() for w in w1]
    g2 = [torch.empty_like(g) for g in g1]
    b = A.AdamwStepper(cfg, w2, g2, device=DEV, zero_state=False)
    b.state.copy_(a.state)
    for t in (3, 4):
        _fill(gen, g1, 1e-3)
        for x, y in zip(g2, g1):
            x.copy_(y)
        a.step(t, 1e-2)
        b.step(t, 1e-2)
    torch.cuda.synchronize()
    for x, y in zip(w1, w2):
        assert torch.equal(x, y)
    assert torch.equal(a.state, b.state)
    a.close()
    b.close()


def test_step_argument_errors_on_a_live_handle():
    cfg, _ = _configs()
    _, w, g = _make([64], [torch.float32], 1)
    st = A.AdamwStepper(cfg, w, g, device=DEV)
    assert A.apollo_adamw_step(st.handle, st._tensors, 0, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_adamw_step(st.handle, st._tensors, 1, float("nan")) == A.APOLLO_EINVAL
    assert A.apollo_adamw_step(st.handle, [(w[0].data_ptr() + 4, g[0].data_ptr())], 1, 0.1) == A.APOLLO_EINVAL
    assert "aligned" in A.apollo_adamw_last_error(st.handle)
    assert A.apollo_adamw_step(st.handle, [(1 << 20, 1 << 21)] * 2, 1, 0.1) == A.APOLLO_EINVAL
    st.close()
