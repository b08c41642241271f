"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on seeded inputs.

Bar: sign planes, packed words and the transposed twin bit-exact; floating-point outputs within the
normalised max-abs error of _util (1e-5 for fp32 activations, 2e-2 for bf16 activations).
"""
import numpy as np
import pytest

from _util import (make_case, nmax_err, packed_to_dev, packed_to_host, to_dev, to_host, tol_for)
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


# ------------------------------------------------------------------ pack / unpack / transposed twin

@pytest.mark.parametrize("q,N,K", [(1, 1, 32), (3, 5, 96), (2, 67, 1280), (4, 1024, 1024), (1, 300, 4096)])
def test_pack_unpack_bit_exact(bcq, oracle, q, N, K):
    rng = np.random.default_rng(100 + N + K)
    planes = rng.choice(np.array([-1, 1], np.int8), size=(q, N, K))
    packed_ref = oracle.pack(planes)
    import torch
    d_planes = torch.from_numpy(planes).cuda()
    d_packed = bcq.bcq_pack(d_planes)
    _sync()
    assert np.array_equal(packed_to_host(d_packed), packed_ref)
    back = bcq.bcq_unpack(d_packed)
    _sync()
    assert np.array_equal(back.cpu().numpy(), planes)
    # only the sign of the byte counts
    odd = planes.astype(np.int16) * rng.integers(1, 128, size=planes.shape)
    odd[planes > 0] -= 1  # includes 0 -> +1
    d_packed2 = bcq.bcq_pack(torch.from_numpy(odd.astype(np.int8)).cuda())
    _sync()
    assert np.array_equal(packed_to_host(d_packed2), packed_ref)


@pytest.mark.parametrize("q,N,K", [(1, 32, 32), (3, 96, 160), (2, 1280, 5120), (4, 1024 + 32, 1024)])
def test_pack_transposed_bit_exact(bcq, oracle, q, N, K):
    rng = np.random.default_rng(200 + N + K)
    planes = rng.choice(np.array([-1, 1], np.int8), size=(q, N, K))
    twin_ref = oracle.pack(np.ascontiguousarray(planes.transpose(0, 2, 1)))  # bits along N
    d_twin = bcq.bcq_pack_transposed(packed_to_dev(oracle.pack(planes)))
    _sync()
    assert np.array_equal(packed_to_host(d_twin), twin_ref)


# ------------------------------------------------------------------ greedy quantizer

def _check_quantize(bcq, oracle, W, q, want_planes=True):
    import torch
    a_ref, b_ref, margin = oracle.quantize(W, q, with_margin=True)
    ws = torch.full((4,), 77, dtype=torch.int32, device="cuda")
    alpha, packed, planes = bcq.bcq_quantize(to_dev(W), q, want_planes=want_planes, workspace=ws)
    _sync()
    assert int(ws[0].item()) == 0
    alpha, packed = alpha.cpu().numpy(), packed_to_host(packed)
    planes_gpu = oracle.unpack(packed, W.shape[1])
    if want_planes:
        assert np.array_equal(planes.cpu().numpy(), planes_gpu)
    # rows where some fp64 mean sits on an fp32 rounding boundary may legitimately round either way
    fragile = (margin < 2.0 ** -40).any(axis=0)
    ok = ~fragile
    assert fragile.sum() <= max(1, W.shape[0] // 1000)
    assert np.array_equal(alpha[:, ok].view(np.uint32), a_ref[:, ok].view(np.uint32))
    assert np.array_equal(planes_gpu[:, ok], b_ref[:, ok])
    assert np.array_equal(packed[:, ok], oracle.pack(b_ref)[:, ok])
    for n in np.nonzero(fragile)[0]:
        for i in range(q):
            assert abs(float(alpha[i, n]) - float(a_ref[i, n])) <= np.spacing(a_ref[i, n]) or i > 0
        a_forced, b_forced = oracle.quantize_row_forced(W[n], q, alpha[:, n], np.ones(q, np.uint8))
        assert np.array_equal(b_forced, planes_gpu[:, n])


@pytest.mark.parametrize("q,N,K", [(3, 1024, 1024), (1, 8, 32), (4, 37, 1280), (2, 16, 96), (4, 64, 10240),
                                   (3, 9, 16384), (4, 200, 2560 + 32)])
def test_quantize_bit_exact(bcq, oracle, q, N, K):
    W = synth.weights(1, "out", N, K, extra=K)
    _check_quantize(bcq, oracle, W, q)


@pytest.mark.parametrize("K", [256, 512, 768, 1024, 1280, 1536, 2048, 2560, 3072, 4096, 5120, 6144, 8192, 10240])
def test_quantize_rows_of_256_column_chunks(bcq, oracle, K):
    # every chunk count of the form for rows of whole 256-column chunks (1, 2 or 4 waves per row), ragged N
    W = synth.weights(1, "out", 37, K, extra=K + 1)
    _check_quantize(bcq, oracle, W, 3)


@pytest.mark.parametrize("q,N,K", [(2, 6151, 512), (1, 3301, 5120), (3, 1001, 8192), (4, 3075, 2560)])
def test_quantize_more_rows_than_one_round_of_workgroups(bcq, oracle, q, N, K):
    W = synth.weights(1, "out", N, K, extra=N)
    _check_quantize(bcq, oracle, W, q, want_planes=False)


def test_quantize_residuals_that_hit_zero_exactly(bcq, oracle):
    # |w| constant along a row: the first mean equals every magnitude, all residuals become +0.0 and every later
    # plane is all +1; two magnitudes c and 3 c: zero after the second plane (Appendix C, Eq. ap1 - ap3)
    rng = np.random.default_rng(5)
    W = np.empty((24, 1024), dtype=np.float32)
    for n in range(24):
        sign = rng.choice(np.float32([-1.0, 1.0]), size=1024)
        c = np.float32(2.0 ** (n % 5 - 3) * 1.25)
        mag = np.full(1024, c, dtype=np.float32)
        if n % 2:
            mag[rng.permutation(1024)[:512]] = np.float32(3.0) * c
        W[n] = sign * mag
    a_ref, b_ref = oracle.quantize(W, 4)
    assert (b_ref[2:] == 1).all()  # the case is the one meant
    _check_quantize(bcq, oracle, W, 4)


def test_quantize_outliers_zero_rows_no_planes(bcq, oracle):
    W = synth.weights(4, "qkv", 2048, 2048, outliers=True)
    W[5] = 0.0
    W[6, ::2] = 0.0
    W[7, :3] = [-0.0, 0.0, 1.0]
    _check_quantize(bcq, oracle, W, 3, want_planes=False)


def test_quantize_reports_nonfinite_rows(bcq):
    import torch
    W = synth.weights(1, "out", 64, 256)
    W[3, 7] = np.inf
    W[40, 0] = np.nan
    ws = torch.zeros((4,), dtype=torch.int32, device="cuda")
    bcq.bcq_quantize(to_dev(W), 2, workspace=ws)
    _sync()
    assert int(ws[0].item()) == 2


# ------------------------------------------------------------------ forward / backward, full comparison

def _run_layer(bcq, oracle, config, kind, T, N, K, q, dtype, outliers=False, q_train=None, grad_scale=1.0,
               twin=True, workspace=False):
    import torch
    W, alpha, planes, packed, x, dy = make_case(config, kind, T, N, K, q, dtype, oracle, outliers)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_twin = bcq.bcq_pack_transposed(d_packed) if (twin and N % 32 == 0) else None
    code = 0 if dtype == "f32" else 1

    def ws(op):
        if not workspace:
            return None
        nbytes = bcq.workspace_bytes(op, T, N, K, q, code)
        return torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")

    y = bcq.bcq_linear_fwd(d_packed, d_alpha, d_x, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input(d_packed, d_alpha, d_dy, packed_t=d_twin, workspace=ws(2))
    da = bcq.bcq_linear_bwd_alpha(d_packed, d_x, d_dy, q_train=q_train, grad_scale=grad_scale, workspace=ws(3))
    _sync()
    tol = tol_for(dtype)
    e_y = nmax_err(to_host(y), oracle.fwd(alpha, planes, x))
    e_dx = nmax_err(to_host(dx), oracle.bwd_input(alpha, planes, dy))
    e_da = nmax_err(to_host(da), oracle.bwd_alpha(planes, x, dy, q_train=q_train, grad_scale=grad_scale))
    assert e_y <= tol, ("fwd", e_y)
    assert e_dx <= tol, ("bwd_input", e_dx)
    assert e_da <= tol, ("bwd_alpha", e_da)
    return e_y, e_dx, e_da


def test_config1_fp32_full(bcq, oracle):
    """N = K = 1024, q = 3, 32 fp32 tokens: quantize on the GPU, then fwd + dx + dalpha against the oracle."""
    import torch
    cfg = synth.CONFIGS[1]
    N, K = synth.layer_shape(cfg["h"], "out")
    T, q = cfg["tokens"][0], cfg["q"][0]
    W = synth.weights(1, "out", N, K)
    _check_quantize(bcq, oracle, W, q)
    for workspace in (False, True):
        _run_layer(bcq, oracle, 1, "out", T, N, K, q, "f32", workspace=workspace)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,N,K,q", [(1, 64, 64, 1), (4, 1280, 1280, 2), (8, 96, 160, 3), (33, 300, 416, 4),
                                     (300, 544, 1056, 3), (17, 35, 32, 8)])
def test_small_shapes_ragged(bcq, oracle, dtype, T, N, K, q):
    """Shapes that span several tiles with ragged tails in T, N and K; with and without workspace / twin."""
    for workspace, twin in ((False, False), (True, True), (True, False)):
        _run_layer(bcq, oracle, 3, "out", T, N, K, q, dtype, workspace=workspace, twin=twin)


@pytest.mark.parametrize("T,N,K,q", [
    (130, 8448, 256, 2),   # forward: 3 x 66 tiles of 64 x 128 tokens x outputs; input gradient: 64 x 64 tiles
    (130, 256, 8448, 3),   # the reverse
    (200, 2560, 2560, 4),  # 64 x 128 tiles in both, ragged last token tile
    (97, 1000, 4128, 4),   # N % 32 != 0 (no twin), K / 32 not a multiple of 4
])
def test_few_hundred_tokens_small_gemm_tiles(bcq, oracle, T, N, K, q):
    """At a few hundred tokens the matrix-core path picks 64-token tiles so that the compute units have work."""
    _run_layer(bcq, oracle, 3, "mlp_up", T, N, K, q, "bf16", workspace=True, twin=(N % 32 == 0))


def test_many_rows_eight_planes_without_workspace(bcq, oracle):
    """16384 rows and more put two row tiles into a wave of the workspace-free small-token kernel; with 5 .. 8 trained
    planes its cross-wave sum then needs more than 64 KiB of LDS, which the launcher must ask for."""
    _run_layer(bcq, oracle, 3, "mlp_up", 3, 16400, 4096, 8, "bf16", workspace=False, twin=False)


@pytest.mark.parametrize("T,N,K", [(100, 96, 96), (130, 160, 224), (257, 64, 32)])
def test_nonfinite_token_row_stays_in_its_row(bcq, oracle, T, N, K):
    """Tiled kernels pad the contraction to a multiple of 128 and the token tile to 64 or more rows: what they read
    for the padding must never bring another token's values into a row.  One token row of x and of dy is set to
    +inf; every other output row must still match the oracle (which never sees the poisoned rows)."""
    import torch
    q, bad = 3, 7
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, "bf16", oracle)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_twin = bcq.bcq_pack_transposed(d_packed)
    xp, dyp = x.copy(), dy.copy()
    xp[bad, :] = np.inf
    dyp[bad, :] = np.inf
    ws = lambda op: torch.empty((max(bcq.workspace_bytes(op, T, N, K, q, 1), 16),), dtype=torch.uint8, device="cuda")
    y = to_host(bcq.bcq_linear_fwd(d_packed, d_alpha, to_dev(xp, "bf16"), workspace=ws(1)))
    dx = to_host(bcq.bcq_linear_bwd_input(d_packed, d_alpha, to_dev(dyp, "bf16"), packed_t=d_twin, workspace=ws(2)))
    _sync()
    keep = np.arange(T) != bad
    assert np.isfinite(y[keep]).all() and np.isfinite(dx[keep]).all()
    assert not np.isfinite(y[bad]).any() and not np.isfinite(dx[bad]).any()
    tol = tol_for("bf16")
    assert nmax_err(y[keep], oracle.fwd(alpha, planes, x)[keep]) <= tol
    assert nmax_err(dx[keep], oracle.bwd_input(alpha, planes, dy)[keep]) <= tol


def test_q_train_and_grad_scale(bcq, oracle):
    _run_layer(bcq, oracle, 2, "out", 64, 256, 512, 4, "bf16", q_train=1, grad_scale=1.0 / 512, workspace=True)
    _run_layer(bcq, oracle, 2, "out", 64, 256, 512, 4, "f32", q_train=2, grad_scale=0.5)


def test_fp32_integer_case_is_exact(bcq, oracle):
    """Small-integer activations and power-of-two scales: every partial sum is exact in fp32, so the fp32
    path must reproduce the oracle exactly (zero tolerance catches any indexing slip)."""
    rng = np.random.default_rng(7)
    T, N, K, q = 19, 160, 224, 3
    planes = rng.choice(np.array([-1, 1], np.int8), size=(q, N, K))
    alpha = np.ldexp(1.0, rng.integers(-3, 3, size=(q, N))).astype(np.float32)
    x = rng.integers(-8, 9, size=(T, K)).astype(np.float32)
    dy = rng.integers(-4, 5, size=(T, N)).astype(np.float32)
    d_packed = packed_to_dev(oracle.pack(planes))
    y = bcq.bcq_linear_fwd(d_packed, to_dev(alpha), to_dev(x))
    dx = bcq.bcq_linear_bwd_input(d_packed, to_dev(alpha), to_dev(dy))
    da = bcq.bcq_linear_bwd_alpha(d_packed, to_dev(x), to_dev(dy))
    _sync()
    assert np.array_equal(to_host(y).astype(np.float64), oracle.fwd(alpha, planes, x))
    assert np.array_equal(to_host(dx).astype(np.float64), oracle.bwd_input(alpha, planes, dy))
    assert np.array_equal(to_host(da).astype(np.float64), oracle.bwd_alpha(planes, x, dy))


def test_bwd_alpha_is_deterministic(bcq, oracle):
    import torch
    W, alpha, planes, packed, x, dy = make_case(2, "qkv", 512, 768, 1024, 4, "bf16", oracle)
    d_packed, d_x, d_dy = packed_to_dev(packed), to_dev(x, "bf16"), to_dev(dy, "bf16")
    nbytes = bcq.workspace_bytes(3, 512, 768, 1024, 4, 1)
    ws = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
    a = bcq.bcq_linear_bwd_alpha(d_packed, d_x, d_dy, workspace=ws).clone()
    b = bcq.bcq_linear_bwd_alpha(d_packed, d_x, d_dy, workspace=ws)
    _sync()
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        q = int(rng.integers(1, 9))
        K = 32 * int(rng.integers(1, 50))
        N = int(rng.integers(1, 520))
        T = int(rng.choice([1, 2, 5, 8, 9, 16, 17, 31, 32, 33, 48, 49, 64, 80, 81, 100, 130]))
        divs = [g for g in range(32, K + 1, 32) if K % g == 0]
        g = int(rng.choice(divs))
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        cases.append((T, N, K, g, q, dtype, bool(rng.random() < 0.8), bool(rng.random() < 0.7)))
    return cases


@pytest.mark.parametrize("T,N,K,g,q,dtype,workspace,twin", _random_cases(36, 20221003858))
def test_random_shapes(bcq, oracle, T, N, K, g, q, dtype, workspace, twin):
    """Seeded random shapes, group sizes, plane counts and call options: every dispatch boundary of the library
    (token thresholds, tile shapes, ragged tails, with / without workspace and twin) against the oracle."""
    import torch
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, dtype, oracle, g=g)
    a3 = alpha if alpha.ndim == 3 else alpha[:, :, None]
    d_packed, d_alpha = packed_to_dev(packed), to_dev(a3)
    d_x, d_dy = to_dev(x, dtype), to_dev(dy, dtype)
    d_twin = bcq.bcq_pack_transposed(d_packed) if (twin and N % 32 == 0) else None
    code = 0 if dtype == "f32" else 1

    def ws(op):
        if not workspace:
            return None
        return torch.empty((max(bcq.workspace_bytes_grouped(op, T, N, K, g, q, code), 16),), dtype=torch.uint8, device="cuda")

    q_train = max(1, q - 1)
    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, d_x, g, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, d_dy, g, packed_t=d_twin, workspace=ws(2))
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, q_train=q_train, grad_scale=0.25, workspace=ws(3))
    _sync()
    tol = tol_for(dtype)
    ref_da = oracle.bwd_alpha(planes, x, dy, q_train=q_train, grad_scale=0.25, g=g)
    assert nmax_err(to_host(y), oracle.fwd(alpha, planes, x)) <= tol
    assert nmax_err(to_host(dx), oracle.bwd_input(alpha, planes, dy)) <= tol
    assert nmax_err(to_host(da).reshape(ref_da.shape), ref_da) <= tol


def _random_streaming_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        q = int(rng.integers(1, 9))
        K = int(rng.choice([512, 1024, 1536, 2048, 2560, 3072, 4096, 4608]))
        N = 32 * int(rng.integers(1, 90))
        T = int(rng.integers(1, 81))
        g = int(rng.choice([K] + [d for d in (512, 1024, 1536, 2048) if d < K and K % d == 0]))
        cases.append((T, N, K, g, q))
    return cases


@pytest.mark.parametrize("T,N,K,g,q", _random_streaming_cases(24, 2210))
def test_random_streaming_shapes(bcq, oracle, T, N, K, g, q):
    """Seeded random shapes the streaming kernels take (twin and workspace given, groups of whole segments): one to
    five token tiles, one or several segments per wave, every plane count."""
    import torch
    W, alpha, planes, packed, x, dy = make_case(3, "qkv", T, N, K, q, "bf16", oracle, g=g)
    a3 = alpha if alpha.ndim == 3 else alpha[:, :, None]
    d_packed, d_alpha = packed_to_dev(packed), to_dev(a3)
    d_x, d_dy = to_dev(x, "bf16"), to_dev(dy, "bf16")
    d_twin = bcq.bcq_pack_transposed(d_packed)

    def ws(op):
        return torch.empty((max(bcq.workspace_bytes_grouped(op, T, N, K, g, q, 1), 16),), dtype=torch.uint8, device="cuda")

    y = bcq.bcq_linear_fwd_grouped(d_packed, d_alpha, d_x, g, workspace=ws(1))
    yd = bcq.bcq_linear_fwd_decode(bcq.bcq_pack_decode(d_packed), d_alpha, d_x, g=g, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input_grouped(d_packed, d_alpha, d_dy, g, packed_t=d_twin, workspace=ws(2))
    da = bcq.bcq_linear_bwd_alpha_grouped(d_packed, d_x, d_dy, g, workspace=ws(3))
    _sync()
    tol = tol_for("bf16")
    ref_y, ref_da = oracle.fwd(alpha, planes, x), oracle.bwd_alpha(planes, x, dy, g=g)
    assert nmax_err(to_host(y), ref_y) <= tol
    assert nmax_err(to_host(yd), ref_y) <= tol
    assert nmax_err(to_host(dx), oracle.bwd_input(alpha, planes, dy)) <= tol
    assert nmax_err(to_host(da).reshape(ref_da.shape), ref_da) <= tol


# ------------------------------------------------------------------ streaming kernels: wide dynamic range, non-finite tokens

def _masked_rel_err(out, ref):
    """Largest element-wise relative error over the elements with |ref| > 1e-3 max|ref| (reported beside the
    normalised error, which never looks at small outputs)."""
    out, ref = np.asarray(out, np.float64), np.asarray(ref, np.float64)
    mask = np.abs(ref) > 1e-3 * np.abs(ref).max()
    return float((np.abs(out - ref)[mask] / np.abs(ref)[mask]).max())


def _outlier_activations(T, D, seed):
    """N(0,1) rounded to bf16 with, inside every 32-element block, one channel scaled by 2^10 and one by 2^-10, exact
    zeros and one bf16 subnormal: the block-scaled two-term FP8 re-coding is exact only within 2^-13 of a block's
    maximum, so the small channels lose bits next to the large one."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((T, D)).astype(np.float32)
    a[:, 3::32] *= np.float32(2.0 ** 10)
    a[:, 7::32] *= np.float32(2.0 ** -10)
    a[:, 11::32] = 0.0
    a[:, 13::32] = np.float32(2.0 ** -130)  # subnormal in bf16 (smallest normal: 2^-126)
    return synth.round_to_bf16(a)


@pytest.mark.parametrize("T", [1, 8, 16])
def test_streaming_activations_with_outlier_channels(bcq, oracle, T):
    """Single-layer streaming kernels and the batched kernel on activations with 2^20 of dynamic range inside every
    32-element block.  Bar: the normalised error as everywhere.  The masked element-wise relative error (elements above
    1e-3 of the largest output) is printed beside it as information, not as a bar: the absolute error of an output is
    set by the rounding of the products of the large channels (bf16 output rounding, and for the input gradient the
    8 significant bits kept of dy * alpha), so an output at 1e-3 of the maximum can be off by several per cent of
    itself (observed: forward 2.4e-2, input gradient 1.2e-1, scale gradient below 1e-5) while the normalised error stays
    at 2.7e-3."""
    import torch
    N, K, q = 640, 1536, 3
    W, alpha, planes, packed, _, _ = make_case(3, "out", T, N, K, q, "bf16", oracle)
    x, dy = _outlier_activations(T, K, 7), _outlier_activations(T, N, 8)
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_twin = bcq.bcq_pack_transposed(d_packed)
    d_x, d_dy = to_dev(x, "bf16"), to_dev(dy, "bf16")
    ws = lambda op: torch.empty((max(bcq.workspace_bytes(op, T, N, K, q, 1), 16),), dtype=torch.uint8, device="cuda")
    y = bcq.bcq_linear_fwd(d_packed, d_alpha, d_x, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input(d_packed, d_alpha, d_dy, packed_t=d_twin, workspace=ws(2))
    da = bcq.bcq_linear_bwd_alpha(d_packed, d_x, d_dy, workspace=ws(3))
    L = dict(N=N, K=K, tiled=bcq.bcq_pack_decode(d_packed), tiled_t=bcq.bcq_pack_decode(d_twin), alpha=d_alpha, x=d_x,
             dy=d_dy, y=torch.zeros_like(y), dx=torch.zeros_like(dx), dalpha=torch.zeros_like(da))
    for op in (1, 2, 3):
        bcq.bcq_linear_batched(bcq.batch_plan(op, [L], T, q))
    _sync()
    refs = (oracle.fwd(alpha, planes, x), oracle.bwd_input(alpha, planes, dy), oracle.bwd_alpha(planes, x, dy))
    for name, outs, ref in (("fwd", (y, L["y"]), refs[0]), ("bwd_input", (dx, L["dx"]), refs[1]),
                            ("bwd_alpha", (da, L["dalpha"]), refs[2])):
        for path, out in zip(("single", "batched"), outs):
            e, m = nmax_err(to_host(out), ref), _masked_rel_err(to_host(out), ref)
            assert e <= tol_for("bf16"), (name, path, e, m)
            print("outlier channels, T=%d %s %s: normalised %.2e, masked element-wise %.2e" % (T, name, path, e, m))
            assert np.isfinite(m)


@pytest.mark.parametrize("T", [3, 8, 16])
def test_streaming_nonfinite_token_stays_in_its_token(bcq, oracle, T):
    """What the streaming kernels promise for a non-finite activation: the outputs of that token are NaN, the outputs
    of every other token are those of the finite problem (tokens are separate columns of the matrix instruction and the
    re-coding gives a block with an Inf or NaN the NaN scale).  One token of x and of dy is poisoned (an Inf in one
    block, a NaN in another); single-layer and batched calls."""
    import torch
    N, K, q, bad = 320, 1024, 2, 1
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, "bf16", oracle)
    xp, dyp = x.copy(), dy.copy()
    xp[bad, 5], xp[bad, 700] = np.inf, np.nan
    dyp[bad, 17], dyp[bad, 300] = -np.inf, np.nan
    d_packed, d_alpha = packed_to_dev(packed), to_dev(alpha)
    d_twin = bcq.bcq_pack_transposed(d_packed)
    d_x, d_dy = to_dev(xp, "bf16"), to_dev(dyp, "bf16")
    ws = lambda op: torch.empty((max(bcq.workspace_bytes(op, T, N, K, q, 1), 16),), dtype=torch.uint8, device="cuda")
    y = bcq.bcq_linear_fwd(d_packed, d_alpha, d_x, workspace=ws(1))
    dx = bcq.bcq_linear_bwd_input(d_packed, d_alpha, d_dy, packed_t=d_twin, workspace=ws(2))
    L = dict(N=N, K=K, tiled=bcq.bcq_pack_decode(d_packed), tiled_t=bcq.bcq_pack_decode(d_twin), alpha=d_alpha, x=d_x,
             dy=d_dy, y=torch.zeros_like(y), dx=torch.zeros_like(dx))
    for op in (1, 2):
        bcq.bcq_linear_batched(bcq.batch_plan(op, [L], T, q))
    _sync()
    keep = np.arange(T) != bad
    ref_y, ref_dx = oracle.fwd(alpha, planes, x), oracle.bwd_input(alpha, planes, dy)
    for out, ref in ((y, ref_y), (L["y"], ref_y), (dx, ref_dx), (L["dx"], ref_dx)):
        o = to_host(out)
        assert np.isnan(o[bad]).all()
        assert np.isfinite(o[keep]).all()
        assert nmax_err(o[keep], ref[keep]) <= tol_for("bf16")
