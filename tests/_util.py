"""Shared helpers of the test-suite: tolerances, error measure, host<->device conversion."""
import numpy as np

from paper_2210_03858_amd import synth

# Normalised max-abs error per output tensor: max|out - ref| / max|ref|.
TOL_F32 = 1e-5   # fp32 activations, fp32 accumulation
TOL_BF16 = 2e-2  # bf16 activations and outputs, fp32 accumulation


def nmax_err(out, ref):
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(out)))
    return float(np.max(np.abs(out - ref))) / denom


def to_dev(a, dtype="f32"):
    """numpy fp32 array -> cuda tensor (bf16 values are assumed exactly representable)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.contiguous()


def to_host(t):
    import torch
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.detach().cpu().numpy()


def packed_to_dev(packed_u32):
    import torch
    return torch.from_numpy(np.ascontiguousarray(packed_u32).view(np.int32)).cuda().contiguous()


def packed_to_host(t):
    return t.detach().cpu().numpy().view(np.uint32)


def tol_for(dtype):
    return TOL_F32 if dtype == "f32" else TOL_BF16


def make_case(config, kind, T, N, K, q, dtype, oracle, outliers=False, extra=0, g=None):
    """Seeded layer + activations, quantized by the oracle (g: group size along K, None = row-wise)."""
    W = synth.weights(config, kind, N, K, outliers=outliers, extra=extra)
    alpha, planes = oracle.quantize(W, q, g=g)
    x = synth.activations(config, kind, T, K, 1, dtype, extra)
    dy = synth.activations(config, kind, T, N, 2, dtype, extra)
    return W, alpha, planes, oracle.pack(planes), x, dy


def decode_layout(packed):
    """Decode layout of include/bcq.h written out with numpy: [row tile][segment][plane][lane = row + 16 g][word j]
    holds canonical word packed[i][16 rt + row][16 seg + 4 g + j]; padding reads as 0."""
    import numpy as np
    q, N, cw = packed.shape
    rt, segs = -(-N // 16), -(-cw // 16)
    pad = np.zeros((q, rt * 16, segs * 16), dtype=np.uint32)
    pad[:, :N, :cw] = packed
    a = pad.reshape(q, rt, 16, segs, 4, 4).transpose(1, 3, 0, 4, 2, 5)  # rt, seg, plane, g, row, j
    return np.ascontiguousarray(a).reshape(-1)
