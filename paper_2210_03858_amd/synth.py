"""Seeded synthetic inputs for the BCQ linear layer (shapes only come from the paper).

This module serves both the GPU tests/benchmark and the CPU oracle's tests.  It
holds no arithmetic of the method itself: it draws random numbers, rounds
activations to bf16 where a configuration asks for bf16, and names the layer
shapes (AlphaTuning Table 1: (3h,h), (h,h), (4h,h), (h,4h)).

Stand-in statement: the paper adapts pretrained GPT-2 / OPT weights on WebNLG,
DART, E2E, MNLI and SAMSum.  None of those are available or needed for the
kernel; weights are N(0, 0.02^2) (the GPT-2 initialiser scale), activations and
output gradients are N(0, 1).
"""
import numpy as np

SEED_BASE = 221003858 * 1000

# layer kinds in one Transformer block, (N multiplier, K multiplier) of the hidden size h
LAYER_KINDS = ("qkv", "out", "mlp_up", "mlp_down")
_SHAPE_MULT = {"qkv": (3, 1), "out": (1, 1), "mlp_up": (4, 1), "mlp_down": (1, 4)}

# the five workloads (1-based, as in the configuration list of the benchmark definition)
CONFIGS = {
    1: dict(h=1024, q=(3,), tokens=(32,), dtype="f32", kinds=("out",), outliers=False),
    2: dict(h=1024, q=(4,), tokens=(8 * 512,), dtype="bf16", kinds=LAYER_KINDS, outliers=False),
    3: dict(h=1280, q=(1, 2, 3, 4), tokens=(1, 4, 8, 4 * 1024), dtype="bf16", kinds=LAYER_KINDS, outliers=False),
    4: dict(h=2048, q=(3,), tokens=(8 * 2048,), dtype="bf16", kinds=LAYER_KINDS, outliers=True),
    5: dict(h=2560, q=(4,), tokens=(1, 16, 256, 4096), dtype="bf16", kinds=LAYER_KINDS, outliers=False, layers=32),
}


def layer_shape(h, kind):
    """(N, K) = (h_out, h_in) of one linear layer of a block with hidden size h."""
    mn, mk = _SHAPE_MULT[kind]
    return mn * h, mk * h


def seed_for(config, kind, tensor_id, extra=0):
    """tensor_id: 0 = W, 1 = x, 2 = dy, 3 = outlier rows.  extra distinguishes replicas/layers."""
    return SEED_BASE + 100 * int(config) + 10 * LAYER_KINDS.index(kind) + int(tensor_id) + 100000 * int(extra)


def round_to_bf16(a):
    """Round fp32 values to the nearest bf16 (ties to even); returned as fp32 holding bf16 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of fp32 values that are already exactly representable in bf16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def weights(config, kind, N, K, outliers=False, extra=0, std=0.02):
    """W[N,K] fp32 ~ N(0, std^2); with outliers, max(1, round(0.001 N)) seeded rows are scaled by 10."""
    rng = np.random.default_rng(seed_for(config, kind, 0, extra))
    W = (std * rng.standard_normal((N, K))).astype(np.float32)
    if outliers:
        r = np.random.default_rng(seed_for(config, kind, 3, extra))
        n_out = max(1, int(round(0.001 * N)))
        rows = r.choice(N, size=n_out, replace=False)
        W[rows] *= np.float32(10.0)
    return W


def activations(config, kind, T, D, tensor_id, dtype="bf16", extra=0):
    """[T,D] ~ N(0,1) as fp32; for dtype 'bf16' the values are rounded to bf16 first."""
    rng = np.random.default_rng(seed_for(config, kind, tensor_id, extra))
    a = rng.standard_normal((T, D)).astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


def sample_indices(seed, T, D, count, full_rows=8, full_cols=8):
    """Output coordinates for sampled parity at sizes the oracle cannot sweep fully:
    `count` random entries plus `full_rows` complete rows and `full_cols` complete columns."""
    rng = np.random.default_rng(seed)
    tt = [rng.integers(0, T, size=count)]
    dd = [rng.integers(0, D, size=count)]
    for r in rng.choice(T, size=min(full_rows, T), replace=False):
        tt.append(np.full(D, r)); dd.append(np.arange(D))
    for c in rng.choice(D, size=min(full_cols, D), replace=False):
        tt.append(np.arange(T)); dd.append(np.full(T, c))
    return np.concatenate(tt).astype(np.int64), np.concatenate(dd).astype(np.int64)
