"""bcq_prepare / bcq_batch_prepare: after them the FIRST call of an operation in a process may sit inside a HIP graph
capture.  "First in the process" needs a fresh process, so the check runs in a child (one GPU process besides this one)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r'''
import sys
sys.path.insert(0, %r)
import torch
import paper_2210_03858_amd as p
p.load()
torch.manual_seed(0)
T, q = 8, 4
out = {}
# single-layer calls on shapes whose kernels need more than 64 KiB of LDS (the shared-activation streaming kernels)
N, K = 14336, 4096
packed = torch.randint(-2**31, 2**31 - 1, (q, N, K // 32), dtype=torch.int32, device="cuda")
twin = p.bcq_pack_transposed(packed)            # another kernel: not one of those prepared below
alpha = torch.rand((q, N), device="cuda") * 0.02
x = torch.randn((T, K), device="cuda").bfloat16()
dy = torch.randn((T, N), device="cuda").bfloat16()
ws = {op: torch.empty((max(p.workspace_bytes(op, T, N, K, q, 1), 16),), dtype=torch.uint8, device="cuda") for op in (1, 2, 3)}
y, dx, da = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda"), torch.zeros((T, K), dtype=torch.bfloat16, device="cuda"), torch.zeros((q, N), device="cuda")
L = dict(N=N, K=K, tiled=p.bcq_pack_decode(packed), tiled_t=p.bcq_pack_decode(twin), alpha=alpha, x=x, dy=dy,
         y=torch.zeros_like(y), dx=torch.zeros_like(dx), dalpha=torch.zeros_like(da))
plans = [p.batch_plan(op, [L], T, q) for op in (1, 2, 3)]
for op in (1, 2, 3):
    p.bcq_prepare(op, T, N, K, q)
for plan in plans:
    p.bcq_batch_prepare(plan)
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):       # the first launches of all these kernels in this process happen under capture
    p.bcq_linear_fwd(packed, alpha, x, y=y, workspace=ws[1])
    p.bcq_linear_bwd_input(packed, alpha, dy, packed_t=twin, dx=dx, workspace=ws[2])
    p.bcq_linear_bwd_alpha(packed, x, dy, dalpha=da, workspace=ws[3])
    for plan in plans:
        p.bcq_linear_batched(plan)
g.replay()
torch.cuda.synchronize()
g_out = [t.clone() for t in (y, dx, da, L["y"], L["dx"], L["dalpha"])]
for t in (y, dx, da, L["y"], L["dx"], L["dalpha"]):
    t.zero_()
p.bcq_linear_fwd(packed, alpha, x, y=y, workspace=ws[1])
p.bcq_linear_bwd_input(packed, alpha, dy, packed_t=twin, dx=dx, workspace=ws[2])
p.bcq_linear_bwd_alpha(packed, x, dy, dalpha=da, workspace=ws[3])
for plan in plans:
    p.bcq_linear_batched(plan)
torch.cuda.synchronize()
for a, b in zip(g_out, (y, dx, da, L["y"], L["dx"], L["dalpha"])):
    assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a, b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    assert a.float().abs().max().item() > 0
# single-layer and batched forward agree within the bf16 bar (different kernels, same arithmetic)
d = (y.float() - L["y"].float()).abs().max().item() / y.float().abs().max().item()
assert d <= 2e-2, d
print("PREPARE_OK")
'''


def test_first_call_inside_a_graph_capture_after_prepare():
    r = subprocess.run([sys.executable, "-c", CHILD % ROOT], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "PREPARE_OK" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
