"""The adaptation step of AlphaTuning on the GPU: scale gradient + AdamW update through the C ABI (Section 4.1,
Appendix A) and the torch.autograd wrapper, against the CPU oracle."""
import numpy as np
import pytest

from _util import make_case, nmax_err, packed_to_dev, to_dev, to_host, tol_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


HP = dict(beta1=0.9, beta2=0.98, eps=1e-7, weight_decay=0.05)


@pytest.mark.parametrize("T,N,K,g,q,q_train,dtype,workspace", [
    (256, 256, 1024, 1024, 3, 1, "bf16", True),    # matrix-core path: update inside the final reduction
    (300, 264, 1056, 96, 4, 2, "bf16", True),      # per-32-column partial sums
    (8, 128, 512, 512, 3, 1, "bf16", True),        # streaming kernel + separate update kernel
    (40, 96, 256, 64, 2, 2, "f32", False),         # vector-ALU kernel + separate update kernel
])
def test_bwd_alpha_adamw_steps(bcq, oracle, T, N, K, g, q, q_train, dtype, workspace):
    """Three optimizer steps with a decaying learning rate.  The gradient the call returns is checked against the
    oracle's Eq. 4; the update is checked against the oracle's AdamW applied to that returned gradient, so the
    optimizer arithmetic is compared on identical inputs (fp32 on the GPU, fp64 in the oracle)."""
    import torch
    W, alpha, planes, packed, x, dy = make_case(2, "out", T, N, K, q, dtype, oracle, g=g)
    G = K // g
    alpha = alpha.reshape(q, N, G)
    d_packed, d_x, d_dy = packed_to_dev(packed), to_dev(x, dtype), to_dev(dy, dtype)
    d_alpha = to_dev(alpha)
    d_m = torch.zeros((q_train, N, G), dtype=torch.float32, device="cuda")
    d_v = torch.zeros_like(d_m)
    code = 0 if dtype == "f32" else 1
    ws = None
    if workspace:
        ws = torch.empty((max(bcq.workspace_bytes_grouped(3, T, N, K, g, q, code), 16),), dtype=torch.uint8, device="cuda")
    ref_da = oracle.bwd_alpha(planes, x, dy, q_train=q_train, grad_scale=1.0 / g, g=g).reshape(q_train, N, G)
    a_ref = alpha.astype(np.float64).copy()
    m_ref = np.zeros((q_train, N, G))
    v_ref = np.zeros((q_train, N, G))
    for step in (1, 2, 3):
        lr = 1e-3 * (1.0 - (step - 1) / 3.0)
        da = bcq.bcq_linear_bwd_alpha_adamw(d_packed, d_x, d_dy, g, d_alpha, d_m, d_v, step, lr, q_train=q_train,
                                            grad_scale=1.0 / g, workspace=ws, **HP)
        torch.cuda.synchronize()
        da = to_host(da)
        assert nmax_err(da, ref_da) <= tol_for(dtype)
        a_ref[:q_train], m_ref, v_ref = oracle.adamw_step(a_ref[:q_train], da, m_ref, v_ref, step, lr, **HP)
        got = to_host(d_alpha).astype(np.float64)
        assert np.allclose(got[:q_train], a_ref[:q_train], rtol=2e-6, atol=1e-9)
        assert np.array_equal(got[q_train:], alpha[q_train:].astype(np.float64))   # frozen planes untouched
        assert np.allclose(to_host(d_m), m_ref, rtol=2e-6, atol=2e-7 * np.abs(da).max())
        assert np.allclose(to_host(d_v), v_ref, rtol=2e-6, atol=1e-20)
        # carry the fp32 state the GPU really holds, so that rounding does not accumulate into the comparison
        a_ref[:q_train] = got[:q_train]
        m_ref, v_ref = to_host(d_m).astype(np.float64), to_host(d_v).astype(np.float64)


def test_alpha_adamw_step_alone(bcq, oracle):
    import torch
    rng = np.random.default_rng(5)
    a = rng.uniform(0.001, 0.05, size=(3, 70, 4)).astype(np.float32)
    g = (rng.standard_normal((2, 70, 4)) * 3).astype(np.float32)
    m = (rng.standard_normal((2, 70, 4)) * 0.1).astype(np.float32)
    v = rng.uniform(0, 1, size=(2, 70, 4)).astype(np.float32)
    d_a, d_m, d_v = to_dev(a), to_dev(m), to_dev(v)
    bcq.bcq_alpha_adamw_step(d_a, to_dev(g), d_m, d_v, 7, 3e-4, **HP)
    torch.cuda.synchronize()
    a_ref, m_ref, v_ref = oracle.adamw_step(a[:2], g, m, v, 7, 3e-4, **HP)
    assert np.allclose(to_host(d_a)[:2], a_ref, rtol=2e-6, atol=1e-9)
    assert np.array_equal(to_host(d_a)[2], a[2])
    # m = beta1 m + (1 - beta1) g cancels when m and g have opposite signs: absolute slack of an fp32 ulp of the terms
    assert np.allclose(to_host(d_m), m_ref, rtol=2e-6, atol=2e-7 * np.abs(g).max())
    assert np.allclose(to_host(d_v), v_ref, rtol=2e-6)


@pytest.mark.parametrize("T,g,q_train,dtype", [(96, None, 1, "bf16"), (6, None, 2, "bf16"), (64, 64, 3, "bf16"),
                                               (20, 128, 1, "f32")])
def test_autograd_module_matches_oracle(bcq, oracle, T, g, q_train, dtype):
    """BCQLinear forward / backward = Eq. 2, Eq. 3 and Eq. 4 of the oracle; only alpha[:q_train] gets a gradient."""
    import torch
    from paper_2210_03858_amd.autograd import BCQLinear
    N, K, q = 160, 256, 3
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, dtype, oracle, g=g)
    gg = K if g is None else g
    layer = BCQLinear(packed_to_dev(packed), to_dev(alpha), g=g, q_train=q_train, grad_scale=1.0 / gg)
    d_x = to_dev(x, dtype).reshape(2, T // 2, K).requires_grad_(True)
    y = layer(d_x)
    assert tuple(y.shape) == (2, T // 2, N)
    y.backward(to_dev(dy, dtype).reshape(2, T // 2, N))
    torch.cuda.synchronize()
    tol = tol_for(dtype)
    assert nmax_err(to_host(y).reshape(T, N), oracle.fwd(alpha, planes, x)) <= tol
    assert nmax_err(to_host(d_x.grad).reshape(T, K), oracle.bwd_input(alpha, planes, dy)) <= tol
    ref_da = oracle.bwd_alpha(planes, x, dy, q_train=q_train, grad_scale=1.0 / gg, g=g)
    assert nmax_err(to_host(layer.alpha_train.grad).reshape(ref_da.shape), ref_da) <= tol
    assert [n for n, p in layer.named_parameters()] == ["alpha_train"]


def test_autograd_training_loop_reduces_quantization_loss(bcq, oracle):
    """A few AdamW steps on alpha_1 only (the paper's recipe) move the quantized layer's output towards the
    full-precision layer's output on fixed synthetic activations."""
    import torch
    from paper_2210_03858_amd import synth
    from paper_2210_03858_amd.autograd import BCQLinear
    N, K, T, q = 256, 512, 128, 3
    W = synth.weights(2, "out", N, K)
    x = to_dev(synth.activations(2, "out", T, K, 1, "bf16"), "bf16")
    target = (x.float() @ to_dev(W).t())
    layer = BCQLinear.from_weight(to_dev(W), q, q_train=1)
    opt = torch.optim.AdamW(layer.parameters(), lr=2e-4, weight_decay=0.0)
    losses = []
    for _ in range(12):
        opt.zero_grad()
        loss = ((layer(x).float() - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < losses[0]
