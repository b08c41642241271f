"""Batched small-token calls (one operation over many independent layers in two launches) against the CPU oracle,
layer by layer and element by element, through the C ABI."""
import numpy as np
import pytest

from _util import TOL_BF16, make_case, nmax_err, packed_to_dev, to_dev, to_host
from paper_2210_03858_amd import synth

pytestmark = pytest.mark.gpu

OP_FWD, OP_DX, OP_DALPHA = 1, 2, 3


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


def _make_batch(bcq, oracle, config, shapes, T, q, poison=True):
    """shapes: list of (kind, N, K, extra).  Returns per-layer host references and device tensors."""
    import torch
    layers = []
    for kind, N, K, extra in shapes:
        W, alpha, planes, packed, x, dy = make_case(config, kind, T, N, K, q, "bf16", oracle, extra=extra)
        d_packed = packed_to_dev(packed)
        L = dict(N=N, K=K, tiled=bcq.bcq_pack_decode(d_packed), alpha=to_dev(alpha), x=to_dev(x, "bf16"),
                 dy=to_dev(dy, "bf16"),
                 # decode layout of the transposed twin [q][K][N/32]
                 tiled_t=bcq.bcq_pack_decode(bcq.bcq_pack_transposed(d_packed)) if N % 32 == 0 else None,
                 # outputs start as NaN: every element must be written by the batch
                 y=torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda"),
                 dx=torch.full((T, K), float("nan"), dtype=torch.bfloat16, device="cuda"),
                 dalpha=torch.full((q, N), float("nan"), dtype=torch.float32, device="cuda"),
                 ref=(alpha, planes, x, dy))
        layers.append(L)
    return layers


def _check_batch(bcq, oracle, layers, T, q, ops=(OP_FWD, OP_DX, OP_DALPHA), q_train=None, grad_scale=1.0):
    import torch
    plans = [bcq.batch_plan(op, layers, T, q, q_train=q_train, grad_scale=grad_scale) for op in ops]
    for plan in plans:
        bcq.bcq_linear_batched(plan)
    torch.cuda.synchronize()
    qt = q if q_train is None else q_train
    for i, L in enumerate(layers):
        alpha, planes, x, dy = L["ref"]
        if OP_FWD in ops:
            e = nmax_err(to_host(L["y"]), oracle.fwd(alpha, planes, x))
            assert e <= TOL_BF16, ("fwd", i, L["N"], L["K"], e)
        if OP_DX in ops:
            e = nmax_err(to_host(L["dx"]), oracle.bwd_input(alpha, planes, dy))
            assert e <= TOL_BF16, ("bwd_input", i, L["N"], L["K"], e)
        if OP_DALPHA in ops:
            ref = oracle.bwd_alpha(planes, x, dy, q_train=qt, grad_scale=grad_scale)
            e = nmax_err(to_host(L["dalpha"])[:qt], ref)
            assert e <= TOL_BF16, ("bwd_alpha", i, L["N"], L["K"], e)


MIXED = [("out", 256, 128, 0), ("qkv", 1000, 1280, 1), ("mlp_up", 48, 2560, 2), ("mlp_down", 1040, 640, 3),
         ("out", 16, 4096 + 128, 4), ("qkv", 2056, 384, 5), ("out", 70, 32 * 37, 6)]  # K % 128 != 0


@pytest.mark.parametrize("T,q", [(1, 1), (3, 2), (8, 4), (9, 3), (16, 4)])
def test_batched_fwd_and_dalpha_mixed_ragged_shapes(bcq, oracle, T, q):
    """Layers of different shapes in one batch, ragged row counts (N % 16 != 0, N < 128), one to 33 segments, one or
    two operand halves (T <= 8 / T > 8)."""
    layers = _make_batch(bcq, oracle, 3, MIXED, T, q)
    _check_batch(bcq, oracle, layers, T, q, ops=(OP_FWD, OP_DALPHA))


MIXED_DX = [("out", 512, 256, 0), ("qkv", 1280, 992, 1),  # N = 2.5 segments; ragged K (rows of the twin)
            ("mlp_up", 1024, 2560, 2), ("mlp_down", 128, 640, 3), ("out", 3840, 64, 4), ("qkv", 1536, 4128, 5),
            ("out", 96, 32, 6)]           # N % 128 != 0, a single 32-column word of K


@pytest.mark.parametrize("T,q", [(1, 1), (5, 2), (8, 4), (12, 3), (16, 4)])
def test_batched_input_gradient_mixed_shapes(bcq, oracle, T, q):
    """Input gradient: one virtual plane over q x ceil(N / 512) virtual segments; one to 8 chunks, ragged rows."""
    layers = _make_batch(bcq, oracle, 3, MIXED_DX, T, q)
    _check_batch(bcq, oracle, layers, T, q, ops=(OP_DX,))


def test_batched_q_train_and_grad_scale(bcq, oracle):
    T, q = 7, 4
    layers = _make_batch(bcq, oracle, 3, MIXED[:3], T, q)
    _check_batch(bcq, oracle, layers, T, q, ops=(OP_DALPHA,), q_train=1, grad_scale=1.0 / 1280)
    import torch
    for L in layers:  # rows of the untrained planes are not touched
        assert torch.isnan(L["dalpha"][1:]).all()


@pytest.mark.parametrize("config,T", [(3, 1), (3, 4), (3, 8), (5, 1), (5, 8), (5, 16)])
def test_batched_block_of_the_workloads(bcq, oracle, config, T):
    """The four layers of one block of workload 3 (d = 1280, every q) and workload 5 (d = 2560, q = 4) on the
    workloads' own seeds, forward + input gradient + scale gradient, every output element against the oracle."""
    cfg = synth.CONFIGS[config]
    for q in cfg["q"]:
        shapes = [(kind,) + synth.layer_shape(cfg["h"], kind) + (0,) for kind in cfg["kinds"]]
        layers = _make_batch(bcq, oracle, config, shapes, T, q)
        _check_batch(bcq, oracle, layers, T, q)


def test_batched_single_layer_and_repeated_run(bcq, oracle):
    """A batch of one layer; running a plan twice gives the same bits (the plan and workspace are reusable)."""
    import torch
    T, q = 8, 3
    layers = _make_batch(bcq, oracle, 3, [("mlp_up", 5120, 1280, 0)], T, q)
    plan = bcq.batch_plan(OP_FWD, layers, T, q)
    bcq.bcq_linear_batched(plan)
    torch.cuda.synchronize()
    first = layers[0]["y"].clone()
    layers[0]["y"].fill_(float("nan"))
    bcq.bcq_linear_batched(plan)
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), layers[0]["y"].view(torch.int16))
    alpha, planes, x, dy = layers[0]["ref"]
    assert nmax_err(to_host(first), oracle.fwd(alpha, planes, x)) <= TOL_BF16


def test_batched_graph_replay(bcq, oracle):
    """A batched call only launches kernels: captured into a HIP graph, every replay equals the eager result."""
    import torch
    T, q = 4, 2
    layers = _make_batch(bcq, oracle, 3, MIXED[:4], T, q)
    plans = [bcq.batch_plan(op, layers, T, q) for op in (OP_FWD, OP_DALPHA)]
    for plan in plans:
        bcq.bcq_linear_batched(plan)
    torch.cuda.synchronize()
    eager = [(L["y"].clone(), L["dalpha"].clone()) for L in layers]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for plan in plans:
            bcq.bcq_linear_batched(plan)
    for _ in range(3):
        for L in layers:
            L["y"].fill_(0)
            L["dalpha"].fill_(0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for L, (y, da) in zip(layers, eager):
            assert torch.equal(L["y"].view(torch.int16), y.view(torch.int16))
            assert torch.equal(L["dalpha"], da)


def test_batched_errors(bcq):
    import torch
    T, q, N, K = 4, 2, 256, 256
    z = lambda *s, dt=torch.bfloat16: torch.zeros(s, dtype=dt, device="cuda")
    base = dict(N=N, K=K, tiled=z(q * N * K // 32, dt=torch.int32), tiled_t=z(q * N * K // 32, dt=torch.int32),
                alpha=z(q, N, dt=torch.float32), x=z(T, K), dy=z(T, N), y=z(T, N), dx=z(T, K),
                dalpha=z(q, N, dt=torch.float32))
    for op, bad, status in ((OP_FWD, dict(K=48), 2), (OP_FWD, dict(y=None), 1), (OP_DX, dict(N=48), 2)):
        with pytest.raises(bcq.BcqError) as e:
            bcq.batch_plan(op, [dict(base, **bad)], T, q)
        assert e.value.status == status
    with pytest.raises(bcq.BcqError) as e:
        bcq.batch_plan(OP_FWD, [base], 17, q)
    assert e.value.status == 2
    with pytest.raises(bcq.BcqError) as e:
        bcq.batch_plan(OP_FWD, [base], T, 5)
    assert e.value.status == 2
    plan = bcq.batch_plan(OP_FWD, [base], T, q)
    plan.workspace = plan.workspace[:16]
    with pytest.raises(bcq.BcqError) as e:
        bcq.bcq_linear_batched(plan)
    assert e.value.status == 5
