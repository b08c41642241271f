"""Parity of bcq_quantize_alternating (Appendix C, Eq. ap4) with the CPU oracle, through the C ABI.

Sign planes, packed words and the fp32 scales are compared bit for bit on every vector whose decisions the oracle
reports as robust: the gap between the best and the second-best level of every element in every round is at least
1e-9 of sum_i |alpha_i| (the two sides add the same fp64 numbers in different orders, which moves alpha by about
1e-16), and no returned alpha sits within 2^-40 of an fp32 rounding boundary.  Fragile vectors must be rare."""
import numpy as np
import pytest

from _util import packed_to_host, to_dev
from paper_2210_03858_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


def _check(bcq, oracle, W, q, iters=15, g=None):
    import torch
    N, K = W.shape
    gg = K if g is None else g
    V = N * (K // gg)
    a_ref, b_ref, margin, done = oracle.quantize_alternating(W, q, iters=iters, g=g, with_margin=True)
    ws = torch.full((4,), 77, dtype=torch.int32, device="cuda")
    alpha, packed, planes = bcq.bcq_quantize_alternating(to_dev(W), q, iters=iters, g=g, want_planes=True, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[0].item()) == 0
    packed = packed_to_host(packed)
    planes_gpu = oracle.unpack(packed, K)
    assert np.array_equal(planes.cpu().numpy(), planes_gpu)
    alpha_v = alpha.cpu().numpy().reshape(q, V)
    a_ref = a_ref.reshape(q, V)
    pv, bv = planes_gpu.reshape(q, V, gg), b_ref.reshape(q, V, gg)
    robust = (margin[:, 0] >= 1e-9) & (margin[:, 1] >= 2.0 ** -40)
    assert (~robust).sum() <= max(1, V // 1000), (~robust).sum()
    assert np.array_equal(alpha_v[:, robust].view(np.uint32), a_ref[:, robust].view(np.uint32))
    assert np.array_equal(pv[:, robust], bv[:, robust])
    # fragile vectors: still a valid quantization whose error is as good as the oracle's, up to the flipped decision
    for v in np.nonzero(~robust)[0]:
        w = W.reshape(V, gg)[v].astype(np.float64)
        e_gpu = ((w - (alpha_v[:, v].astype(np.float64)[:, None] * pv[:, v]).sum(axis=0)) ** 2).sum()
        e_ref = ((w - (a_ref[:, v].astype(np.float64)[:, None] * bv[:, v]).sum(axis=0)) ** 2).sum()
        assert e_gpu <= e_ref * 1.05 + 1e-30
    return done


@pytest.mark.parametrize("q,N,K,g", [(1, 16, 128, None), (2, 40, 256, None), (3, 64, 1024, None), (4, 32, 1280, None),
                                     (3, 24, 1024, 256), (4, 10, 4096, None), (2, 6, 16384, None), (5, 8, 160, None),
                                     (8, 4, 256, 64), (3, 50, 96, 32)])
def test_alternating_bit_exact(bcq, oracle, q, N, K, g):
    W = synth.weights(1, "out", N, K, extra=7 * K + q)
    done = _check(bcq, oracle, W, q, g=g)
    if q > 1:
        assert done.max() > 1   # the refinement really runs


def test_alternating_zero_iterations_and_few(bcq, oracle):
    W = synth.weights(1, "out", 48, 512)
    _check(bcq, oracle, W, 3, iters=0)
    _check(bcq, oracle, W, 3, iters=1)
    _check(bcq, oracle, W, 3, iters=4)


def test_alternating_degenerate_rows_and_outliers(bcq, oracle):
    W = synth.weights(4, "qkv", 256, 512, outliers=True)
    W[5] = 0.0
    W[6, ::2] = 0.0
    W[7, :3] = [-0.0, 0.0, 1.0]
    W[8] = 0.25          # constant vector: every plane after the first has a zero residual
    W[9, :] = np.where(np.arange(512) % 2 == 0, 0.5, -0.25)
    _check(bcq, oracle, W, 3)


def test_alternating_reports_nonfinite_vectors(bcq):
    import torch
    W = synth.weights(1, "out", 64, 256)
    W[3, 7] = np.inf
    W[40, 0] = np.nan
    ws = torch.zeros((4,), dtype=torch.int32, device="cuda")
    bcq.bcq_quantize_alternating(to_dev(W), 2, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[0].item()) == 2


def test_alternating_gpt2_medium_layer(bcq, oracle):
    """One full (h, h) layer of the GPT-2-medium block, q = 3, 15 rounds."""
    W = synth.weights(2, "out", 1024, 1024)
    _check(bcq, oracle, W, 3)
