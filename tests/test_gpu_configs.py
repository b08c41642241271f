"""Parity at the full sizes of the five benchmark workloads, in the launch configuration bench.py times
(workspace from bcq_workspace_bytes, transposed twin given).  The oracle cannot sweep these sizes in seconds,
so outputs are compared on seeded samples it computes one by one: >= 4096 random entries plus 8 complete rows
and 8 complete columns per output tensor, and 64 complete rows of dalpha over all tokens.  The quantizer is
compared in full (bit-exact planes and alpha)."""
import numpy as np
import pytest

from _util import nmax_err, packed_to_dev, packed_to_host, to_dev, to_host, tol_for
from paper_2210_03858_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


def _ws(bcq, op, T, N, K, q, code):
    import torch
    nbytes = bcq.workspace_bytes(op, T, N, K, q, code)
    return torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")


def _quantize_and_check(bcq, oracle, W, q):
    import torch
    a_ref, b_ref, margin = oracle.quantize(W, q, with_margin=True)
    alpha, packed, _ = bcq.bcq_quantize(to_dev(W), q)
    torch.cuda.synchronize()
    ok = ~(margin < 2.0 ** -40).any(axis=0)
    assert (~ok).sum() <= max(1, W.shape[0] // 1000)
    assert np.array_equal(alpha.cpu().numpy()[:, ok].view(np.uint32), a_ref[:, ok].view(np.uint32))
    assert np.array_equal(packed_to_host(packed)[:, ok], oracle.pack(b_ref)[:, ok])
    return a_ref, b_ref, alpha, packed


def _sampled_layer(bcq, oracle, config, kind, T, q, dtype, outliers=False, full=False, seed=0, q_train=None):
    import torch
    h = synth.CONFIGS[config]["h"]
    N, K = synth.layer_shape(h, kind)
    W = synth.weights(config, kind, N, K, outliers=outliers)
    a_ref, b_ref, alpha, packed = _quantize_and_check(bcq, oracle, W, q)
    x = synth.activations(config, kind, T, K, 1, dtype)
    dy = synth.activations(config, kind, T, N, 2, dtype)
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    code = 0 if dtype == "f32" else 1
    twin = bcq.bcq_pack_transposed(packed)
    y = bcq.bcq_linear_fwd(packed, alpha, d_x, workspace=_ws(bcq, 1, T, N, K, q, code))
    dx = bcq.bcq_linear_bwd_input(packed, alpha, d_dy, packed_t=twin, workspace=_ws(bcq, 2, T, N, K, q, code))
    da = bcq.bcq_linear_bwd_alpha(packed, d_x, d_dy, q_train=q_train, workspace=_ws(bcq, 3, T, N, K, q, code))
    torch.cuda.synchronize()
    y, dx, da = to_host(y), to_host(dx), to_host(da)
    tol = tol_for(dtype)
    if full:
        ref_y, ref_dx = oracle.fwd(a_ref, b_ref, x), oracle.bwd_input(a_ref, b_ref, dy)
        ref_da = oracle.bwd_alpha(b_ref, x, dy, q_train=q_train)
        errs = (nmax_err(y, ref_y), nmax_err(dx, ref_dx), nmax_err(da, ref_da))
    else:
        tt, nn = synth.sample_indices(1000 + seed, T, N, 4096)
        ref = oracle.fwd_at(a_ref, b_ref, x, tt, nn)
        e_y = nmax_err(y[tt, nn], ref)
        tt, kk = synth.sample_indices(2000 + seed, T, K, 4096)
        ref = oracle.bwd_input_at(a_ref, b_ref, dy, tt, kk)
        e_dx = nmax_err(dx[tt, kk], ref)
        rows = np.random.default_rng(3000 + seed).choice(N, size=min(64, N), replace=False)
        ref = oracle.bwd_alpha_rows(b_ref, x, dy, rows, q_train=q_train)
        e_da = nmax_err(da[:, rows], ref)
        errs = (e_y, e_dx, e_da)
    assert errs[0] <= tol, ("fwd", errs)
    assert errs[1] <= tol, ("bwd_input", errs)
    assert errs[2] <= tol, ("bwd_alpha", errs)
    return errs


@pytest.mark.parametrize("T,N,K", [
    (4000, 4040, 160),    # forward: 16 x 16 tiles of 256 x 256, ragged in T and N, last K-step beyond K
    (4000, 160, 4032),    # the same for the input gradient (256 x 256 tiles over T x K, contraction N = 160)
    (2000, 3000, 1056),   # forward: 128 x 128 tiles, ragged in T and N, K / 32 odd
])
def test_large_tiles_ragged_edges(bcq, oracle, T, N, K):
    """The workloads' shapes are multiples of 256, so the large tiles of the matrix-core kernels see ragged token rows,
    ragged output columns and a contraction that ends inside a K-step only here.  Sampled outputs (random entries, the
    last token rows and the last output columns in full) against the oracle; scale gradient on sampled rows incl. the
    last ones."""
    import torch
    q = 3
    W = synth.weights(4, "out", N, K)
    a_ref, b_ref, alpha, packed = _quantize_and_check(bcq, oracle, W, q)
    x = synth.activations(4, "out", T, K, 1, "bf16")
    dy = synth.activations(4, "out", T, N, 2, "bf16")
    d_x, d_dy = to_dev(x, "bf16"), to_dev(dy, "bf16")
    twin = bcq.bcq_pack_transposed(packed) if N % 32 == 0 else None
    y = bcq.bcq_linear_fwd(packed, alpha, d_x, workspace=_ws(bcq, 1, T, N, K, q, 1))
    dx = bcq.bcq_linear_bwd_input(packed, alpha, d_dy, packed_t=twin, workspace=_ws(bcq, 2, T, N, K, q, 1))
    da = bcq.bcq_linear_bwd_alpha(packed, d_x, d_dy, workspace=_ws(bcq, 3, T, N, K, q, 1))
    torch.cuda.synchronize()
    y, dx, da = to_host(y), to_host(dx), to_host(da)
    tol = tol_for("bf16")

    def samples(seed, rows, cols):
        tt, cc = synth.sample_indices(seed, rows, cols, 2048)
        last_r = np.repeat(np.arange(rows - 2, rows), min(cols, 512))           # the last two token rows
        last_r_c = np.tile(np.arange(cols - min(cols, 512), cols), 2)
        last_c = np.tile(np.arange(cols - 2, cols), min(rows, 512))             # the last two columns
        last_c_r = np.repeat(np.arange(rows - min(rows, 512), rows), 2)
        return (np.concatenate([tt, last_r, last_c_r]).astype(np.int64),
                np.concatenate([cc, last_r_c, last_c]).astype(np.int64))

    tt, nn = samples(41, T, N)
    assert nmax_err(y[tt, nn], oracle.fwd_at(a_ref, b_ref, x, tt, nn)) <= tol
    tt, kk = samples(42, T, K)
    assert nmax_err(dx[tt, kk], oracle.bwd_input_at(a_ref, b_ref, dy, tt, kk)) <= tol
    rows = np.concatenate([np.random.default_rng(43).choice(N - 8, size=24, replace=False), np.arange(N - 8, N)])
    assert nmax_err(da[:, rows], oracle.bwd_alpha_rows(b_ref, x, dy, rows)) <= tol


@pytest.mark.parametrize("kind", synth.LAYER_KINDS)
def test_config2_gpt2_medium_block(bcq, oracle, kind):
    """d = 1024, q = 4, bf16, T = 8 x 512: the workload bench.py times."""
    _sampled_layer(bcq, oracle, 2, kind, 4096, 4, "bf16", seed=synth.LAYER_KINDS.index(kind))


@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("T", [1, 4, 8])
def test_config3_decode_regime(bcq, oracle, q, T):
    """d = 1280 layers at 1, 4 and 8 tokens, compared in full."""
    for kind in ("qkv", "mlp_down"):
        _sampled_layer(bcq, oracle, 3, kind, T, q, "bf16", full=True)


@pytest.mark.parametrize("q,kind", [(1, "out"), (2, "mlp_down"), (3, "mlp_up"), (4, "qkv")])
def test_config3_training_regime(bcq, oracle, q, kind):
    _sampled_layer(bcq, oracle, 3, kind, 4 * 1024, q, "bf16", seed=10 + q)


@pytest.mark.parametrize("kind", ["out", "mlp_up", "mlp_down"])
def test_config4_opt13b_outlier_rows(bcq, oracle, kind):
    """d = 2048, q = 3, T = 8 x 2048, 0.1 % of the rows scaled by 10 before quantization."""
    _sampled_layer(bcq, oracle, 4, kind, 8 * 2048, 3, "bf16", outliers=True, seed=20)


@pytest.mark.parametrize("T", [1, 16, 256, 4096])
def test_config5_token_sweep(bcq, oracle, T):
    """d = 2560, q = 4: tokens 1, 16, 256, 4096 cross from the streaming kernels to the matrix-core kernels."""
    kind = {1: "mlp_up", 16: "qkv", 256: "mlp_down", 4096: "mlp_up"}[T]
    _sampled_layer(bcq, oracle, 5, kind, T, 4, "bf16", seed=30 + T, q_train=1 if T == 256 else None)


def test_config5_quantizer_all_kinds(bcq, oracle):
    """Greedy quantizer on every layer shape of the d = 2560 stack, two seeded layers each, in full."""
    for layer in range(2):
        for kind in synth.LAYER_KINDS:
            N, K = synth.layer_shape(2560, kind)
            W = synth.weights(5, kind, N, K, extra=layer)
            _quantize_and_check(bcq, oracle, W, 4)


@pytest.mark.parametrize("T", [4096, 8])
def test_step_as_hip_graph_with_second_stream_matches_eager(bcq, oracle, T):
    """The launch configuration bench.py times: one HIP graph of the step (fwd, dx on the capturing stream, the scale
    gradients on a second stream of default priority, joined at the end).  Every replay must reproduce the eagerly
    launched one-stream results bit for bit - with eager work and synchronisations between the replays - and those
    results meet the oracle's bar on sampled outputs (one layer)."""
    import torch
    q, h = 4, 1024
    layers = []
    for kind in ("out", "mlp_up"):
        N, K = synth.layer_shape(h, kind)
        a_ref, planes_ref = oracle.quantize(synth.weights(2, kind, N, K), q)  # the oracle's planes: inputs of both sides
        alpha, packed = to_dev(a_ref), packed_to_dev(oracle.pack(planes_ref))
        L = dict(N=N, K=K, alpha=alpha, packed=packed, twin=bcq.bcq_pack_transposed(packed), a_ref=a_ref, planes_ref=planes_ref,
                 x=torch.from_numpy(synth.activations(2, kind, T, K, 1, "bf16")).cuda().bfloat16(),
                 dy=torch.from_numpy(synth.activations(2, kind, T, N, 2, "bf16")).cuda().bfloat16(),
                 ws={op: torch.empty((max(bcq.workspace_bytes(op, T, N, K, q, 1), 16),), dtype=torch.uint8, device="cuda")
                     for op in (1, 2, 3)})
        for tag in ("e", "g"):  # eager / graph outputs
            L["y" + tag] = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda")
            L["dx" + tag] = torch.zeros((T, K), dtype=torch.bfloat16, device="cuda")
            L["da" + tag] = torch.zeros((q, N), dtype=torch.float32, device="cuda")
        layers.append(L)

    def fwd(L, t): bcq.bcq_linear_fwd(L["packed"], L["alpha"], L["x"], y=L["y" + t], workspace=L["ws"][1])
    def dxf(L, t): bcq.bcq_linear_bwd_input(L["packed"], L["alpha"], L["dy"], packed_t=L["twin"], dx=L["dx" + t], workspace=L["ws"][2])
    def daf(L, t): bcq.bcq_linear_bwd_alpha(L["packed"], L["x"], L["dy"], dalpha=L["da" + t], workspace=L["ws"][3])

    for L in layers:  # eager, one stream (also the warm-up that sets the kernels' attributes before the capture)
        fwd(L, "e"), dxf(L, "e"), daf(L, "e")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        main = torch.cuda.current_stream()
        side.wait_stream(main)
        for L in layers:
            fwd(L, "g")
            with torch.cuda.stream(side):
                daf(L, "g")
            dxf(L, "g")
        main.wait_stream(side)
    for rep in range(3):
        for L in layers:
            for name in ("yg", "dxg", "dag"):
                L[name].fill_(float(rep + 1))        # eager work between the replays; also proves the replay rewrites all
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for L in layers:
            assert torch.equal(L["yg"], L["ye"]), rep
            assert torch.equal(L["dxg"], L["dxe"]), rep
            assert torch.equal(L["dag"], L["dae"]), rep
    # the eager results against the oracle, sampled (first layer)
    L = layers[0]
    N, K = L["N"], L["K"]
    rng = np.random.default_rng(5)
    x_h = synth.activations(2, "out", T, K, 1, "bf16")
    ts, ns = rng.integers(0, T, 512), rng.integers(0, N, 512)
    y_ref = oracle.fwd_at(L["a_ref"], L["planes_ref"], x_h, ts, ns)
    scale = np.abs(y_ref).max()
    assert np.abs(L["ye"].float().cpu().numpy()[ts, ns] - y_ref).max() / scale <= tol_for("bf16")


# ------------------------------------------------------------------ every (q, kind, T) cell of workloads 3, 4 and 5

@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("kind", synth.LAYER_KINDS)
def test_config3_training_regime_every_cell(bcq, oracle, q, kind):
    """d = 1280 at 4 x 1024 tokens: all 16 (q, layer kind) cells on sampled outputs."""
    _sampled_layer(bcq, oracle, 3, kind, 4 * 1024, q, "bf16", seed=40 + 4 * q + synth.LAYER_KINDS.index(kind))


@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("T", [1, 4, 8])
def test_config3_decode_regime_other_kinds(bcq, oracle, q, T):
    """The two layer kinds test_config3_decode_regime leaves out, compared in full."""
    for kind in ("out", "mlp_up"):
        _sampled_layer(bcq, oracle, 3, kind, T, q, "bf16", full=True)


def test_config4_opt13b_outlier_rows_qkv(bcq, oracle):
    _sampled_layer(bcq, oracle, 4, "qkv", 8 * 2048, 3, "bf16", outliers=True, seed=21)


@pytest.mark.parametrize("T", [1, 16, 256, 4096])
@pytest.mark.parametrize("kind", synth.LAYER_KINDS)
def test_config5_every_kind_at_every_token_count(bcq, oracle, kind, T):
    """d = 2560, q = 4: all four layer kinds at 1, 16 (in full), 256 and 4096 tokens (sampled).  At 1 and 16 tokens the
    2560 x 10240 layer takes the shared-activation streaming kernel for its input gradient."""
    _sampled_layer(bcq, oracle, 5, kind, T, 4, "bf16", full=(T <= 16), seed=60 + T + synth.LAYER_KINDS.index(kind))
