"""bcq_linear_fwd_static (scratch in the library's static device array, no allocation) against bcq_linear_fwd with a
caller's workspace and against the CPU oracle: two calls in a row, the second with a smaller input, both on shapes
whose forward goes through the scratch (pre-kernel + streaming kernel, not the single-kernel form)."""
import numpy as np
import pytest

from _util import TOL_BF16, make_case, nmax_err, packed_to_dev, to_dev, to_host

pytestmark = pytest.mark.gpu


def test_fwd_static_matches_workspace_call_twice(oracle):
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2210_03858_amd as p
    p.load()
    BF16 = p.binding.BCQ_BF16
    # (T, N, K, q): first 16 tokens (two operand halves) on a 4096 x 4096 layer, then 5 tokens on a ragged, smaller one
    for T, N, K, q in [(16, 4096, 4096, 3), (5, 1000, 8192 + 64, 2)]:
        assert 16 <= p.workspace_bytes(1, T, N, K, q, BF16) <= p.binding.STATIC_SCRATCH_BYTES
        W, alpha, planes, packed, x, dy = make_case(3, "out", T, N, K, q, "bf16", oracle)
        d_packed, d_alpha, d_x = packed_to_dev(packed), to_dev(alpha), to_dev(x, "bf16")
        ws = torch.empty((p.workspace_bytes(1, T, N, K, q, BF16),), dtype=torch.uint8, device="cuda")
        y_ws = p.bcq_linear_fwd(d_packed, d_alpha, d_x, workspace=ws)
        y = torch.full((T, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        p.bcq_linear_fwd_static(d_packed, d_alpha, d_x, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y.view(torch.int16), y_ws.view(torch.int16)), "differs from the workspace call"
        ref = oracle.fwd(alpha, planes, x)
        assert nmax_err(to_host(y), ref) <= TOL_BF16


def test_fwd_static_rejects_what_does_not_fit():
    import torch
    import paper_2210_03858_amd as p
    p.load()
    T, N, K, q = 80, 64, 12800, 1  # 25 segments x 5 token tiles x 2 halves: 2112000 bytes > 2 MiB
    packed = torch.zeros((q, N, K // 32), dtype=torch.int32, device="cuda")
    alpha = torch.ones((q, N), dtype=torch.float32, device="cuda")
    x = torch.zeros((T, K), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(p.BcqError) as e:
        p.bcq_linear_fwd_static(packed, alpha, x, y)
    assert e.value.status == 5
    with pytest.raises(p.BcqError) as e:
        p.bcq_linear_fwd_static(packed[:, :, :16].contiguous(), alpha, torch.zeros((81, 512), dtype=torch.bfloat16, device="cuda"),
                                torch.zeros((81, N), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == 2
