"""bcq_linear_fwd_lut (Section 6, "Inference Speed": forward by table look-up) against the oracle's Eq. 2."""
import numpy as np
import pytest

from paper_2210_03858_amd import synth
from _util import TOL_BF16, make_case, nmax_err, packed_to_dev, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bcq():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    return p


@pytest.mark.parametrize("T,N,K,q", [(1, 96, 512, 4), (2, 37, 1280, 3), (3, 200, 2560, 1), (4, 64, 4096, 2),
                                     (1, 33, 16384, 2), (4, 5, 32, 8), (1, 2560, 10240, 4), (2, 1000, 96, 4)])
def test_lut_forward_matches_oracle(bcq, oracle, T, N, K, q):
    import torch
    W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, "bf16", oracle)
    y = bcq.bcq_linear_fwd_lut(packed_to_dev(packed), to_dev(alpha), to_dev(x, "bf16"))
    torch.cuda.synchronize()
    ref = oracle.fwd(alpha, planes, x)
    assert nmax_err(to_host(y), ref) <= TOL_BF16


def test_lut_forward_equals_streaming_path_on_config5_block(bcq, oracle):
    # the four layer shapes of workload 5 at one token: both decode variants within tolerance of the oracle
    import torch
    for kind in synth.CONFIGS[5]["kinds"]:
        N, K = synth.layer_shape(synth.CONFIGS[5]["h"], kind)
        W, alpha, planes, packed, x, dy = make_case(5, kind, 1, N, K, 4, "bf16", oracle)
        d_packed, d_alpha, d_x = packed_to_dev(packed), to_dev(alpha), to_dev(x, "bf16")
        y_lut = bcq.bcq_linear_fwd_lut(d_packed, d_alpha, d_x)
        ws = torch.empty((bcq.workspace_bytes(1, 1, N, K, 4, 1),), dtype=torch.uint8, device="cuda")
        y_str = bcq.bcq_linear_fwd(d_packed, d_alpha, d_x, workspace=ws)
        torch.cuda.synchronize()
        ref = oracle.fwd(alpha, planes, x)
        assert nmax_err(to_host(y_lut), ref) <= TOL_BF16 and nmax_err(to_host(y_str), ref) <= TOL_BF16


def test_lut_rejects_what_it_does_not_take(bcq):
    import torch
    packed = torch.zeros((2, 64, 4128 // 32), dtype=torch.int32, device="cuda")
    alpha = torch.ones((2, 64), device="cuda")
    with pytest.raises(bcq.BcqError):
        bcq.bcq_linear_fwd_lut(packed, alpha, torch.zeros((4, 4128), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(bcq.BcqError):
        bcq.bcq_linear_fwd_lut(packed, alpha, torch.zeros((5, 4128), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(bcq.BcqError):
        bcq.bcq_linear_fwd_lut(packed, alpha, torch.zeros((1, 4128), dtype=torch.float32, device="cuda"))
