"""Parity of the group-wise entry points (scales alpha[q][N][K/g]; Appendix C group-wise paragraph, Table 1 rows
with g < h_in, Table 4 group sizes) with the CPU oracle, through the C ABI.

Bar as for the row-wise path: sign planes and packed words bit-exact, alpha bit-exact except vectors whose fp64
mean sits on an fp32 rounding boundary, floating-point outputs within the normalised max-abs tolerances of _util.
"""
import numpy as np
import pytest

from _util import decode_layout, make_case, nmax_err, packed_to_dev, packed_to_host, to_dev, to_host, tol_for
from paper_2210_03858_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


def _sync():
    import torch
    torch.cuda.synchronize()


def _ws(bcq, op, T, N, K, g, q, code):
    import torch
    nbytes = bcq.workspace_bytes_grouped(op, T, N, K, g, q, code)
    return torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")


def _check_quantize(bcq, oracle, W, q, g):
    """Group-wise quantizer: compare per length-g vector (N K / g of them)."""
    import torch
    N, K = W.shape
    G = K // g
    a_ref, b_ref, margin = oracle.quantize(W, q, with_margin=True, g=g)
    a_ref, margin = a_ref.reshape(q, N * G), margin.reshape(q, N * G)
    ws = torch.full((4,), 77, dtype=torch.int32, device="cuda")
    alpha, packed, planes = bcq.bcq_quantize_grouped(to_dev(W), q, g, want_planes=True, workspace=ws)
    _sync()
    assert int(ws[0].item()) == 0
    assert tuple(alpha.shape) == (q, N, G)
    packed = packed_to_host(packed)
    planes_gpu = oracle.unpack(packed, K)
    assert np.array_equal(planes.cpu().numpy(), planes_gpu)
    alpha_v = alpha.cpu().numpy().reshape(q, N * G)
    pv = planes_gpu.reshape(q, N * G, g)
    bv = b_ref.reshape(q, N * G, g)
    # A mean of few fp32 values has few significant bits and often sits EXACTLY on an fp32 rounding boundary;
    # such sums are exact in fp64 in any order, so most "fragile" vectors still agree.  Those that differ must be
    # fragile, rare, one ulp apart in the plane that differs first, and self-consistent (forced re-run below).
    fragile = (margin < 2.0 ** -40).any(axis=0)
    ok = ~fragile
    assert np.array_equal(alpha_v[:, ok].view(np.uint32), a_ref[:, ok].view(np.uint32))
    assert np.array_equal(pv[:, ok], bv[:, ok])
    differs = (alpha_v.view(np.uint32) != a_ref.view(np.uint32)).any(axis=0)
    assert differs.sum() <= max(1, N * G // 1000)
    for v in np.nonzero(fragile)[0]:
        _, b_forced = oracle.quantize_row_forced(W.reshape(N * G, g)[v], q, alpha_v[:, v], np.ones(q, np.uint8))
        assert np.array_equal(b_forced, pv[:, v])
    if not differs.any():
        assert np.array_equal(packed, oracle.pack(b_ref))
    return alpha, packed


@pytest.mark.parametrize("q,N,K,g", [(3, 64, 1024, 256), (4, 37, 1280, 64), (2, 16, 96, 32), (1, 8, 4096, 2048),
                                     (4, 50, 2560, 1280), (3, 5, 16384 * 2, 16384), (2, 200, 1056, 96)])
def test_quantize_grouped_bit_exact(bcq, oracle, q, N, K, g):
    W = synth.weights(1, "out", N, K, extra=K + g)
    _check_quantize(bcq, oracle, W, q, g)


def test_quantize_grouped_equals_rowwise_call_at_g_equal_k(bcq, oracle):
    import torch
    W = synth.weights(1, "out", 96, 512)
    a1, p1, _ = bcq.bcq_quantize(to_dev(W), 3)
    a2, p2, _ = bcq.bcq_quantize_grouped(to_dev(W), 3, 512)
    _sync()
    assert torch.equal(a1.view(torch.int32), a2.view(torch.int32).reshape(3, 96)) and torch.equal(p1, p2)


def _run_layer(bcq, oracle, config, kind, T, N, K, g, q, dtype, q_train=None, grad_scale=1.0, twin=True,
               workspace=True):
    W, alpha, planes, packed, x, dy = make_case(config, kind, T, N, K, q, dtype, oracle, g=g)
    if alpha.ndim == 2:  # g == K: the oracle returns the row-wise shape
        alpha = alpha[:, :, None]
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_twin = bcq.bcq_pack_transposed(d_packed) if (twin and N % 32 == 0) else None
    code = 0 if dtype == "f32" else 1
    ws = (lambda op: _ws(bcq, op, T, N, K, g, q, code)) if workspace else (lambda op: None)
    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, d_x, g, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, d_dy, g, packed_t=d_twin, workspace=ws(2))
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, q_train=q_train, grad_scale=grad_scale,
                                          workspace=ws(3))
    _sync()
    tol = tol_for(dtype)
    a_or = alpha if g != K else alpha[:, :, 0]
    ref_da = oracle.bwd_alpha(planes, x, dy, q_train=q_train, grad_scale=grad_scale, g=g)
    errs = (nmax_err(to_host(y), oracle.fwd(a_or, planes, x)),
            nmax_err(to_host(dx), oracle.bwd_input(a_or, planes, dy)),
            nmax_err(to_host(da).reshape(ref_da.shape), ref_da))
    assert errs[0] <= tol, ("fwd", errs)
    assert errs[1] <= tol, ("bwd_input", errs)
    assert errs[2] <= tol, ("bwd_alpha", errs)
    return errs


SHAPES = [
    # T, N, K, g, q
    (1, 64, 64, 32, 1),        # one token, two groups
    (4, 1280, 1280, 256, 2),   # few tokens, groups that are no whole 512-column segments: tiled kernels
    (8, 96, 160, 32, 3),
    (33, 304, 416, 32, 4),     # per-32-column partial sums, ragged tiles in every extent
    (300, 544, 1024, 512, 3),  # groups of two whole 256-column tiles
    (300, 544, 1056, 96, 3),   # group size that is no power of two
    (17, 35, 64, 32, 8),       # N % 8 != 0: vector-ALU kernels
    (260, 256, 1024, 256, 4),  # one group per 256-column tile
    (65, 128, 768, 768, 2),    # g = K through the group-wise entry points
    (70, 264, 2048, 1024, 4),  # g = K / 2, the setting of the OPT experiments (Table 7)
]


STREAM_SHAPES = [
    # few tokens with groups of whole 512-column segments: the streaming kernels (with workspace and twin); the
    # input gradient streams at every group size
    (1, 64, 1024, 512, 1),
    (4, 1056, 2048, 512, 4),     # one segment per group
    (8, 320, 3072, 1024, 3),     # three groups: waves own whole groups
    (9, 96, 4096, 2048, 8),      # two halves (T > 8), every plane
    (16, 512, 5120, 512, 2),     # ten groups over up to eight waves
    (31, 64, 1536, 512, 4),      # two token tiles (forward and input gradient only stream here)
    (5, 160, 1280, 64, 4),       # small groups: only the input gradient streams (20 sets per plane)
    (8, 2560, 1024, 512, 4),
]


@pytest.mark.parametrize("T,N,K,g,q", STREAM_SHAPES)
def test_grouped_small_token_streaming_parity(bcq, oracle, T, N, K, g, q):
    for workspace, twin in ((True, True), (True, False), (False, False)):
        _run_layer(bcq, oracle, 3, "out", T, N, K, g, q, "bf16", workspace=workspace, twin=twin)


MANY_ROWS = [
    # plane matrices with many rows: the workgroups share the re-coded activations through LDS
    # T, N, K, g, q
    (8, 14336, 4096, 4096, 4),    # two parts of the contraction axis, whole chunks: guard-free instantiation
    (5, 14352, 4608, 4608, 3),    # ragged rows, 9 segments over two parts (5 + 4): guarded instantiation
    (8, 14336, 4096, 1024, 4),    # group-wise scales, two segments per group
    (3, 14400, 6144, 1536, 2),    # three-segment groups: parts of 6 segments, chunks straddle groups
    (12, 28672, 4096, 4096, 4),   # two register halves per token tile (9 .. 16 tokens): one part, 8 row tiles
    (16, 28688, 4608, 512, 1),    # the same with group-wise scales and ragged rows
    (1, 14336, 4096 + 32, 4128, 4),  # K / 32 not a multiple of 4: falls back to the per-wave kernel
]


@pytest.mark.parametrize("T,N,K,g,q", MANY_ROWS)
def test_many_rows_streaming_parity(bcq, oracle, T, N, K, g, q):
    """Forward and scale gradient (the input gradient of these shapes streams a plane matrix with few rows)."""
    W, alpha, planes, packed, x, dy = make_case(3, "mlp_up", T, N, K, q, "bf16", oracle, g=g)
    if alpha.ndim == 2:
        alpha = alpha[:, :, None]
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_x, d_dy = to_dev(x, "bf16"), to_dev(dy, "bf16")
    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, d_x, g, workspace=_ws(bcq, 1, T, N, K, g, q, 1))
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=_ws(bcq, 3, T, N, K, g, q, 1))
    _sync()
    tol = tol_for("bf16")
    a_or = alpha if g != K else alpha[:, :, 0]
    ref_da = oracle.bwd_alpha(planes, x, dy, g=g)
    assert nmax_err(to_host(y), oracle.fwd(a_or, planes, x)) <= tol
    assert nmax_err(to_host(da).reshape(ref_da.shape), ref_da) <= tol


MANY_COLUMNS = [
    # input gradient of layers with many columns: the transposed twin is a plane matrix with many rows (K of them) and
    # the workgroups share the re-coded, per-plane scaled activations through LDS; virtual segments = q * N / 512
    # T, N, K, q
    (8, 2048, 14336, 4),    # two parts of 8 virtual segments (planes 0-1 / 2-3): guard-free instantiation
    (5, 3072, 14368, 3),    # ragged rows; 18 virtual segments in parts of 9 that straddle the planes: guarded
    (12, 2048, 28672, 4),   # two register halves per token tile: one part, 8 row tiles
    (40, 2048, 28672, 2),   # three token tiles (grid y), the last one ragged
    (8, 1024, 14336, 4),    # too few segments for the shared form: per-wave kernel
    (7, 2560, 10240, 4),    # 160 workgroups: the smallest twin that takes the shared form (20 virtual segments, guarded)
]


@pytest.mark.parametrize("T,N,K,q", MANY_COLUMNS)
def test_many_columns_input_gradient_streaming(bcq, oracle, T, N, K, q):
    W, alpha, planes, packed, x, dy = make_case(3, "mlp_down", T, N, K, q, "bf16", oracle)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha[:, :, None])
    d_twin = bcq.bcq_pack_transposed(d_packed)
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, to_dev(dy, "bf16"), K, packed_t=d_twin,
                                          workspace=_ws(bcq, 2, T, N, K, K, q, 1))
    _sync()
    assert nmax_err(to_host(dx), oracle.bwd_input(alpha, planes, dy)) <= tol_for("bf16")


@pytest.mark.parametrize("T,N,K,g,q", [(8, 2048, 14336, 1024, 4), (12, 2048, 28672, 512, 3),
                                       # groups of 160 columns: a shared-activation workgroup (64 or 128 rows of the twin)
                                       # would straddle two groups, so these must take the per-wave kernel
                                       (8, 2560, 10240, 160, 4), (8, 2560, 20480, 160, 2),
                                       (8, 2560, 10240, 128, 2)])  # 128-row workgroups inside 128-column groups
def test_many_columns_input_gradient_streaming_groupwise(bcq, oracle, T, N, K, g, q):
    """Group-wise scales: one set of scaled activations per plane and scale group; a workgroup's rows of the twin lie
    in one group."""
    W, alpha, planes, packed, x, dy = make_case(3, "mlp_down", T, N, K, q, "bf16", oracle, g=g)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_twin = bcq.bcq_pack_transposed(d_packed)
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, to_dev(dy, "bf16"), g, packed_t=d_twin,
                                          workspace=_ws(bcq, 2, T, N, K, g, q, 1))
    _sync()
    assert nmax_err(to_host(dx), oracle.bwd_input(alpha, planes, dy)) <= tol_for("bf16")  # alpha is [q][N][K / g]


def test_many_rows_two_token_tiles_and_partial_training(bcq, oracle):
    """17 .. 31 tokens are two token tiles of the forward (grid y); the scale gradient of the first planes only."""
    T, N, K, q = 20, 28672, 4096, 2
    W, alpha, planes, packed, x, dy = make_case(3, "mlp_up", T, N, K, q, "bf16", oracle)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha[:, :, None])
    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, to_dev(x, "bf16"), K, workspace=_ws(bcq, 1, T, N, K, K, q, 1))
    tiled = bcq.bcq_pack_decode(d_packed)
    y_dec = bcq.bcq_linear_fwd_decode(tiled, d_alpha, to_dev(x, "bf16"), workspace=_ws(bcq, 1, T, N, K, K, q, 1))
    T2 = 7
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, to_dev(x[:T2], "bf16"), to_dev(dy[:T2], "bf16"), K, q_train=1,
                                          grad_scale=0.5, workspace=_ws(bcq, 3, T2, N, K, K, q, 1))
    _sync()
    tol = tol_for("bf16")
    ref = oracle.fwd(alpha, planes, x)
    assert nmax_err(to_host(y), ref) <= tol
    assert nmax_err(to_host(y_dec), ref) <= tol
    ref_da = oracle.bwd_alpha(planes, x[:T2], dy[:T2], q_train=1, grad_scale=0.5)
    assert nmax_err(to_host(da).reshape(ref_da.shape), ref_da) <= tol


def test_grouped_streaming_equals_rowwise_streaming_when_scales_repeat(bcq, oracle):
    """Group-wise scales that repeat one value per row must give the row-wise result of the same kernels
    (forward and input gradient); the scale gradient summed over the groups must equal the row-wise one."""
    import torch
    T, N, K, g, q = 8, 256, 2048, 512, 3
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, "bf16", oracle)
    d_packed, d_x, d_dy = packed_to_dev(packed), to_dev(x, "bf16"), to_dev(dy, "bf16")
    d_twin = bcq.bcq_pack_transposed(d_packed)
    a_row = to_dev(alpha[:, :, None])
    a_grp = to_dev(np.repeat(alpha[:, :, None], K // g, axis=2))
    y_r = bcq.bcq_linear_fwd_grouped(d_packed, a_row, d_x, K, workspace=_ws(bcq, 1, T, N, K, K, q, 1))
    y_g = bcq.bcq_linear_fwd_grouped(d_packed, a_grp, d_x, g, workspace=_ws(bcq, 1, T, N, K, g, q, 1))
    dx_r = bcq.bcq_linear_bwd_input_grouped(d_packed, a_row, d_dy, K, packed_t=d_twin,
                                            workspace=_ws(bcq, 2, T, N, K, K, q, 1))
    dx_g = bcq.bcq_linear_bwd_input_grouped(d_packed, a_grp, d_dy, g, packed_t=d_twin,
                                            workspace=_ws(bcq, 2, T, N, K, g, q, 1))
    da_r = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, K, workspace=_ws(bcq, 3, T, N, K, K, q, 1))
    da_g = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=_ws(bcq, 3, T, N, K, g, q, 1))
    _sync()
    tol = tol_for("bf16")
    assert nmax_err(to_host(y_g), to_host(y_r)) <= tol
    assert torch.equal(dx_g, dx_r)  # same re-coded activations per plane, same order of sums
    assert nmax_err(to_host(da_g).sum(axis=2), to_host(da_r)[:, :, 0]) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,N,K,g,q", SHAPES)
def test_grouped_layer_parity(bcq, oracle, dtype, T, N, K, g, q):
    for workspace, twin in ((False, False), (True, True), (True, False)):
        _run_layer(bcq, oracle, 3, "out", T, N, K, g, q, dtype, workspace=workspace, twin=twin)


def test_grouped_q_train_and_grad_scale(bcq, oracle):
    """Training alpha_1 only with the paper's 1/g damping (Eq. 4), coarse and fine partial sums."""
    _run_layer(bcq, oracle, 2, "out", 128, 256, 1024, 256, 4, "bf16", q_train=1, grad_scale=1.0 / 256)
    _run_layer(bcq, oracle, 2, "out", 128, 256, 1024, 64, 4, "bf16", q_train=2, grad_scale=1.0 / 64)
    _run_layer(bcq, oracle, 2, "out", 64, 256, 512, 128, 3, "f32", q_train=2, grad_scale=0.5)


def test_grouped_fp32_integer_case_is_exact(bcq, oracle):
    """Small-integer activations and power-of-two scales that differ between groups: every partial sum is exact
    in fp32, so the fp32 path must reproduce the oracle exactly (catches any slip in the group index)."""
    rng = np.random.default_rng(8)
    T, N, K, g, q = 19, 160, 224, 32, 3
    planes = rng.choice(np.array([-1, 1], np.int8), size=(q, N, K))
    alpha = np.ldexp(1.0, rng.integers(-3, 3, size=(q, N, K // g))).astype(np.float32)
    x = rng.integers(-8, 9, size=(T, K)).astype(np.float32)
    dy = rng.integers(-4, 5, size=(T, N)).astype(np.float32)
    d_packed = packed_to_dev(oracle.pack(planes))
    y = bcq.bcq_linear_fwd_grouped(d_packed, to_dev(alpha), to_dev(x), g)
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, to_dev(alpha), to_dev(dy), g)
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, to_dev(x), to_dev(dy), g)
    _sync()
    assert np.array_equal(to_host(y).astype(np.float64), oracle.fwd(alpha, planes, x))
    assert np.array_equal(to_host(dx).astype(np.float64), oracle.bwd_input(alpha, planes, dy))
    assert np.array_equal(to_host(da).astype(np.float64), oracle.bwd_alpha(planes, x, dy, g=g))


def test_grouped_bwd_alpha_is_deterministic(bcq, oracle):
    import torch
    T, N, K, g, q = 512, 768, 1024, 64, 4
    W, alpha, planes, packed, x, dy = make_case(2, "qkv", T, N, K, q, "bf16", oracle, g=g)
    d_packed, d_x, d_dy = packed_to_dev(packed), to_dev(x, "bf16"), to_dev(dy, "bf16")
    ws = _ws(bcq, 3, T, N, K, g, q, 1)
    a = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=ws).clone()
    b = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=ws)
    _sync()
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("kind,g", [("qkv", 64), ("out", 256), ("mlp_up", 512), ("mlp_down", 1024), ("mlp_down", 64)])
def test_config2_block_grouped_sampled(bcq, oracle, kind, g):
    """GPT-2-medium layer shapes at T = 4096, q = 3 with the group sizes of Table 4, quantized on the GPU,
    in the launch configuration the benchmark uses; outputs compared on seeded samples."""
    import torch
    T, q, dtype = 4096, 3, "bf16"
    N, K = synth.layer_shape(1024, kind)
    W = synth.weights(2, kind, N, K, extra=g)
    alpha, packed = _check_quantize(bcq, oracle, W, q, g)
    a_ref, b_ref = oracle.quantize(W, q, g=g)
    d_packed = packed_to_dev(packed)
    x = synth.activations(2, kind, T, K, 1, dtype, g)
    dy = synth.activations(2, kind, T, N, 2, dtype, g)
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    twin = bcq.bcq_pack_transposed(d_packed)
    d_alpha = to_dev(a_ref)  # the oracle's scales: fragile vectors may differ by an ulp on the GPU
    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, d_x, g, workspace=_ws(bcq, 1, T, N, K, g, q, 1))
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, d_dy, g, packed_t=twin,
                                          workspace=_ws(bcq, 2, T, N, K, g, q, 1))
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=_ws(bcq, 3, T, N, K, g, q, 1))
    torch.cuda.synchronize()
    y, dx, da = to_host(y), to_host(dx), to_host(da)
    planes_gpu = oracle.unpack(packed, K)  # equal to b_ref except on fragile vectors
    tol = tol_for(dtype)
    tt, nn = synth.sample_indices(5000 + g, T, N, 4096)
    assert nmax_err(y[tt, nn], oracle.fwd_at(a_ref, planes_gpu, x, tt, nn)) <= tol
    tt, kk = synth.sample_indices(6000 + g, T, K, 4096)
    assert nmax_err(dx[tt, kk], oracle.bwd_input_at(a_ref, planes_gpu, dy, tt, kk)) <= tol
    rows = np.random.default_rng(7000 + g).choice(N, size=32, replace=False)
    assert nmax_err(da[:, rows], oracle.bwd_alpha_rows(planes_gpu, x, dy, rows, g=g)) <= tol


DECODE_SHAPES = [
    # T, N, K, g, q
    (1, 16, 512, 512, 1),          # one tile, one segment
    (8, 1000, 1056, 1056, 3),      # ragged rows (N % 16 != 0) and a last segment of 32 columns
    (4, 2560, 2560, 2560, 4),      # a layer of workload 5
    (16, 96, 4096, 4096, 8),       # two register halves, every plane
    (31, 64, 1536, 512, 2),        # two token tiles, group-wise scales
    (8, 14336, 4096, 4096, 4),     # many rows: activations shared through LDS, guard-free instantiation
    (5, 14352, 4608, 1536, 3),     # many rows, ragged, group-wise, guarded instantiation
    (12, 28672, 4096, 4096, 2),    # many rows, two register halves, one part
]


@pytest.mark.parametrize("T,N,K,g,q", DECODE_SHAPES)
def test_decode_layout_and_forward(bcq, oracle, T, N, K, g, q):
    """bcq_pack_decode is bit-exact against the layout definition; bcq_linear_fwd_decode meets the forward's bar."""
    import torch
    W, alpha, planes, packed, x, dy = make_case(3, "mlp_up", T, N, K, q, "bf16", oracle, g=g)
    d_packed = packed_to_dev(packed)
    tiled = bcq.bcq_pack_decode(d_packed)
    _sync()
    assert tiled.numel() * 4 == bcq.decode_layout_bytes(N, K, q)
    assert np.array_equal(tiled.cpu().numpy().view(np.uint32), decode_layout(packed))
    a3 = alpha if alpha.ndim == 3 else alpha[:, :, None]
    y = bcq.bcq_linear_fwd_decode(tiled, to_dev(a3), to_dev(x, "bf16"), g=g, workspace=_ws(bcq, 1, T, N, K, g, q, 1))
    y_canon = bcq.bcq_linear_fwd_grouped(d_packed, to_dev(a3), to_dev(x, "bf16"), g, workspace=_ws(bcq, 1, T, N, K, g, q, 1))
    _sync()
    assert nmax_err(to_host(y), oracle.fwd(alpha, planes, x)) <= tol_for("bf16")
    if K % 128 == 0:  # same kernel, same order of sums (the canonical path of other K takes 4-byte plane loads)
        assert torch.equal(y, y_canon)


def test_decode_forward_rejects_what_it_does_not_take(bcq):
    import torch
    q, N, K = 2, 64, 1024
    tiled = torch.zeros((bcq.decode_layout_bytes(N, K, q) // 4,), dtype=torch.int32, device="cuda")
    alpha = torch.ones((q, N, 1), dtype=torch.float32, device="cuda")
    ws = torch.empty((1 << 20,), dtype=torch.uint8, device="cuda")
    for T, dt, g, w in ((81, torch.bfloat16, K, ws), (4, torch.float32, K, ws), (4, torch.bfloat16, 256, ws),
                        (4, torch.bfloat16, K, None)):
        x = torch.zeros((T, K), dtype=dt, device="cuda")
        a = alpha if g == K else torch.ones((q, N, K // g), dtype=torch.float32, device="cuda")
        with pytest.raises(bcq.BcqError):
            bcq.bcq_linear_fwd_decode(tiled, a, x, g=g, workspace=w)
