"""Thin ctypes binding of libbcq_hip.so (include/bcq.h): argument marshalling only.

Every function takes torch tensors that live on the GPU (PyTorch is used for device memory and streams
only), checks dtype/shape/contiguity on the host, passes raw device pointers and the current HIP stream to
the C entry point of the same name, and raises BcqError on a non-zero status.  There is no CPU fallback:
if the shared library is missing, load() raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbcq_hip.so")

BCQ_F32, BCQ_BF16 = 0, 1
OP_QUANTIZE, OP_FWD, OP_BWD_INPUT, OP_BWD_ALPHA = 0, 1, 2, 3
QUANTIZE_MAX_K = 16384

EXPORTS = ("bcq_status_string", "bcq_abi_version", "bcq_workspace_bytes", "bcq_quantize", "bcq_pack",
           "bcq_unpack", "bcq_pack_transposed", "bcq_linear_fwd", "bcq_linear_bwd_input", "bcq_linear_bwd_alpha",
           "bcq_workspace_bytes_grouped", "bcq_quantize_grouped", "bcq_linear_fwd_grouped",
           "bcq_linear_bwd_input_grouped", "bcq_linear_bwd_alpha_grouped", "bcq_quantize_alternating",
           "bcq_alpha_adamw_step", "bcq_linear_bwd_alpha_adamw", "bcq_decode_layout_bytes", "bcq_pack_decode",
           "bcq_linear_fwd_decode", "bcq_linear_fwd_static", "bcq_linear_fwd_lut", "bcq_batch_sizes", "bcq_batch_plan", "bcq_linear_batched",
           "bcq_prepare", "bcq_batch_prepare")

_lib = None


class AdamW(ctypes.Structure):
    """struct bcq_adamw of include/bcq.h."""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int64)]


class BatchLayer(ctypes.Structure):
    """struct bcq_batch_layer of include/bcq.h."""
    _fields_ = [("tiled", ctypes.c_void_p), ("tiled_t", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
                ("x", ctypes.c_void_p), ("dy", ctypes.c_void_p), ("y", ctypes.c_void_p), ("dx", ctypes.c_void_p),
                ("dalpha", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64)]


class BcqError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__("%s failed: status %d (%s)" % (what, self.status, status_string(self.status)))


def load():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run `python -m paper_2210_03858_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, sz, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    lib.bcq_status_string.restype = ctypes.c_char_p
    lib.bcq_status_string.argtypes = [i32]
    lib.bcq_abi_version.restype = i32
    lib.bcq_workspace_bytes.argtypes = [i32, i64, i64, i64, i32, i32, ctypes.POINTER(sz)]
    lib.bcq_quantize.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp, sz, vp]
    lib.bcq_pack.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.bcq_unpack.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.bcq_pack_transposed.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.bcq_linear_fwd.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.bcq_linear_bwd_input.argtypes = [vp, vp, vp, vp, i32, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.bcq_linear_bwd_alpha.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, i32, f32, vp, vp, sz, vp]
    lib.bcq_workspace_bytes_grouped.argtypes = [i32, i64, i64, i64, i64, i32, i32, ctypes.POINTER(sz)]
    lib.bcq_quantize_grouped.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, vp, sz, vp]
    lib.bcq_linear_fwd_grouped.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.bcq_linear_bwd_input_grouped.argtypes = [vp, vp, vp, vp, i32, i64, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.bcq_linear_bwd_alpha_grouped.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i32, i32, f32, vp, vp, sz, vp]
    lib.bcq_quantize_alternating.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
    ap = ctypes.POINTER(AdamW)
    lib.bcq_alpha_adamw_step.argtypes = [vp, vp, vp, vp, i64, ap, vp]
    lib.bcq_linear_bwd_alpha_adamw.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i32, i32, f32, vp, vp, vp, vp, ap,
                                               vp, sz, vp]
    lib.bcq_decode_layout_bytes.argtypes = [i64, i64, i32, ctypes.POINTER(sz)]
    lib.bcq_pack_decode.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.bcq_linear_fwd_decode.argtypes = [vp, vp, vp, i32, i64, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.bcq_linear_fwd_static.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp, vp]
    lib.bcq_linear_fwd_lut.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, vp, vp]
    bl = ctypes.POINTER(BatchLayer)
    lib.bcq_batch_sizes.argtypes = [i32, bl, i64, i64, i32, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.bcq_batch_plan.argtypes = [i32, bl, i64, i64, i32, i32, f32, i32, vp, sz]
    lib.bcq_linear_batched.argtypes = [vp, vp, sz, vp, sz, vp]
    lib.bcq_prepare.argtypes = [i32, i64, i64, i64, i64, i32, i32]
    lib.bcq_batch_prepare.argtypes = [vp, sz]
    for name in EXPORTS[2:]:
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def status_string(status):
    return load().bcq_status_string(int(status)).decode()


def abi_version():
    return int(load().bcq_abi_version())


def workspace_bytes(op, T, N, K, q, dtype):
    out = ctypes.c_size_t(0)
    st = load().bcq_workspace_bytes(op, T, N, K, q, dtype, ctypes.byref(out))
    if st:
        raise BcqError(st, "bcq_workspace_bytes")
    return int(out.value)


def workspace_bytes_grouped(op, T, N, K, g, q, dtype):
    out = ctypes.c_size_t(0)
    st = load().bcq_workspace_bytes_grouped(op, T, N, K, g, q, dtype, ctypes.byref(out))
    if st:
        raise BcqError(st, "bcq_workspace_bytes_grouped")
    return int(out.value)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _need(t, dtype, shape, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype
            and tuple(t.shape) == tuple(shape)):
        raise ValueError("%s must be a contiguous cuda tensor of dtype %s and shape %s" % (name, dtype, tuple(shape)))


def _act_dtype(t):
    if t.dtype == torch.float32:
        return BCQ_F32
    if t.dtype == torch.bfloat16:
        return BCQ_BF16
    raise ValueError("activations must be float32 or bfloat16")


def _ws(workspace):
    if workspace is None:
        return None, 0
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous cuda tensor")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _check(st, what):
    if st:
        raise BcqError(st, what)


def bcq_quantize(W, q, alpha=None, packed=None, planes_i8=None, want_planes=False, workspace=None):
    """Greedy BCQ of W[N,K] fp32 -> (alpha[q,N] f32, packed[q,N,K/32] int32 words, planes_i8 or None)."""
    N, K = W.shape
    _need(W, torch.float32, (N, K), "W")
    dev = W.device
    alpha = torch.empty((q, N), dtype=torch.float32, device=dev) if alpha is None else alpha
    packed = torch.empty((q, N, K // 32), dtype=torch.int32, device=dev) if packed is None else packed
    if planes_i8 is None and want_planes:
        planes_i8 = torch.empty((q, N, K), dtype=torch.int8, device=dev)
    _need(alpha, torch.float32, (q, N), "alpha")
    _need(packed, torch.int32, (q, N, K // 32), "packed")
    if planes_i8 is not None:
        _need(planes_i8, torch.int8, (q, N, K), "planes_i8")
    wp, wb = _ws(workspace)
    _check(load().bcq_quantize(_ptr(W), N, K, q, _ptr(alpha), _ptr(packed), _ptr(planes_i8), wp, wb, _stream()),
           "bcq_quantize")
    return alpha, packed, planes_i8


def bcq_pack(planes_i8, packed=None):
    q, N, K = planes_i8.shape
    _need(planes_i8, torch.int8, (q, N, K), "planes_i8")
    packed = torch.empty((q, N, K // 32), dtype=torch.int32, device=planes_i8.device) if packed is None else packed
    _need(packed, torch.int32, (q, N, K // 32), "packed")
    _check(load().bcq_pack(_ptr(planes_i8), N, K, q, _ptr(packed), _stream()), "bcq_pack")
    return packed


def bcq_unpack(packed, planes_i8=None):
    q, N, Kw = packed.shape
    _need(packed, torch.int32, (q, N, Kw), "packed")
    K = Kw * 32
    planes_i8 = torch.empty((q, N, K), dtype=torch.int8, device=packed.device) if planes_i8 is None else planes_i8
    _need(planes_i8, torch.int8, (q, N, K), "planes_i8")
    _check(load().bcq_unpack(_ptr(packed), N, K, q, _ptr(planes_i8), _stream()), "bcq_unpack")
    return planes_i8


def bcq_pack_transposed(packed, packed_t=None):
    q, N, Kw = packed.shape
    _need(packed, torch.int32, (q, N, Kw), "packed")
    K = Kw * 32
    if packed_t is None:
        packed_t = torch.empty((q, K, max(N // 32, 1)), dtype=torch.int32, device=packed.device)
    _check(load().bcq_pack_transposed(_ptr(packed), N, K, q, _ptr(packed_t), _stream()), "bcq_pack_transposed")
    return packed_t


def decode_layout_bytes(N, K, q):
    out = ctypes.c_size_t(0)
    _check(load().bcq_decode_layout_bytes(N, K, q, ctypes.byref(out)), "bcq_decode_layout_bytes")
    return int(out.value)


def bcq_pack_decode(packed, tiled=None):
    """canonical packed[q,N,K/32] -> decode layout (flat int32 tensor of decode_layout_bytes(N, K, q) bytes)."""
    q, N, Kw = packed.shape
    _need(packed, torch.int32, (q, N, Kw), "packed")
    K = Kw * 32
    words = decode_layout_bytes(N, K, q) // 4
    if tiled is None:
        tiled = torch.empty((words,), dtype=torch.int32, device=packed.device)
    _need(tiled, torch.int32, (words,), "tiled")
    _check(load().bcq_pack_decode(_ptr(packed), N, K, q, _ptr(tiled), _stream()), "bcq_pack_decode")
    return tiled


def bcq_linear_fwd_decode(tiled, alpha, x, g=None, y=None, workspace=None):
    """Forward from the decode layout; alpha[q,N] or [q,N,K/g]; at most 80 tokens of bf16; workspace required."""
    T, K = x.shape
    q, N = alpha.shape[0], alpha.shape[1]
    g = K if g is None else int(g)
    dt = _act_dtype(x)
    _need(tiled, torch.int32, (decode_layout_bytes(N, K, q) // 4,), "tiled")
    if alpha.dim() == 2:
        alpha = alpha.reshape(q, N, 1)
    _need(alpha, torch.float32, (q, N, K // max(g, 1)), "alpha")
    y = torch.empty((T, N), dtype=x.dtype, device=x.device) if y is None else y
    _need(y, x.dtype, (T, N), "y")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_fwd_decode(_ptr(tiled), _ptr(alpha), _ptr(x), dt, T, N, K, g, q, _ptr(y), wp, wb,
                                        _stream()), "bcq_linear_fwd_decode")
    return y


def bcq_linear_fwd(packed, alpha, x, y=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    dt = _act_dtype(x)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N), "alpha")
    _need(x, x.dtype, (T, K), "x")
    y = torch.empty((T, N), dtype=x.dtype, device=x.device) if y is None else y
    _need(y, x.dtype, (T, N), "y")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_fwd(_ptr(packed), _ptr(alpha), _ptr(x), dt, T, N, K, q, _ptr(y), wp, wb, _stream()),
           "bcq_linear_fwd")
    return y


LUT_MAX_TOKENS = 4
LUT_MAX_TABLE_BYTES = 128 * 1024


def bcq_linear_fwd_lut(packed, alpha, x, y=None):
    """Decode forward by table look-up (1 .. 4 tokens, bf16, row-wise scales, 8 * T * K <= 128 KiB); no workspace."""
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    dt = _act_dtype(x)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N), "alpha")
    _need(x, x.dtype, (T, K), "x")
    y = torch.empty((T, N), dtype=x.dtype, device=x.device) if y is None else y
    _need(y, x.dtype, (T, N), "y")
    _check(load().bcq_linear_fwd_lut(_ptr(packed), _ptr(alpha), _ptr(x), dt, T, N, K, q, _ptr(y), _stream()),
           "bcq_linear_fwd_lut")
    return y


STATIC_SCRATCH_BYTES = 2 * 1024 * 1024
STATIC_MAX_TOKENS = 80


def bcq_linear_fwd_static(packed, alpha, x, y):
    """Small-token forward into the caller's y, scratch in the library's static device array: no allocation anywhere
    (y is required for that reason)."""
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    dt = _act_dtype(x)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N), "alpha")
    _need(x, x.dtype, (T, K), "x")
    _need(y, x.dtype, (T, N), "y")
    _check(load().bcq_linear_fwd_static(_ptr(packed), _ptr(alpha), _ptr(x), dt, T, N, K, q, _ptr(y), _stream()),
           "bcq_linear_fwd_static")
    return y


def bcq_linear_bwd_input(packed, alpha, dy, packed_t=None, dx=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = dy.shape[0]
    dt = _act_dtype(dy)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N), "alpha")
    _need(dy, dy.dtype, (T, N), "dy")
    if packed_t is not None:
        _need(packed_t, torch.int32, (q, K, N // 32), "packed_t")
    dx = torch.empty((T, K), dtype=dy.dtype, device=dy.device) if dx is None else dx
    _need(dx, dy.dtype, (T, K), "dx")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_bwd_input(_ptr(packed), _ptr(packed_t), _ptr(alpha), _ptr(dy), dt, T, N, K, q,
                                       _ptr(dx), wp, wb, _stream()), "bcq_linear_bwd_input")
    return dx


def bcq_linear_bwd_alpha(packed, x, dy, q_train=None, grad_scale=1.0, dalpha=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    dt = _act_dtype(x)
    q_train = q if q_train is None else int(q_train)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(x, x.dtype, (T, K), "x")
    _need(dy, x.dtype, (T, N), "dy")
    dalpha = torch.empty((q_train, N), dtype=torch.float32, device=x.device) if dalpha is None else dalpha
    _need(dalpha, torch.float32, (q_train, N), "dalpha")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_bwd_alpha(_ptr(packed), _ptr(x), _ptr(dy), dt, T, N, K, q, q_train,
                                       float(grad_scale), _ptr(dalpha), wp, wb, _stream()), "bcq_linear_bwd_alpha")
    return dalpha


# ---- group-wise scales: alpha[q, N, K/g] (g = K gives the row-wise calls above) ----------------------------

def bcq_quantize_grouped(W, q, g, alpha=None, packed=None, planes_i8=None, want_planes=False, workspace=None):
    """Greedy BCQ of every length-g vector of W[N,K] -> (alpha[q,N,K/g] f32, packed[q,N,K/32], planes_i8 or None)."""
    N, K = W.shape
    g = int(g)
    G = K // max(g, 1)
    _need(W, torch.float32, (N, K), "W")
    dev = W.device
    alpha = torch.empty((q, N, G), dtype=torch.float32, device=dev) if alpha is None else alpha
    packed = torch.empty((q, N, K // 32), dtype=torch.int32, device=dev) if packed is None else packed
    if planes_i8 is None and want_planes:
        planes_i8 = torch.empty((q, N, K), dtype=torch.int8, device=dev)
    _need(alpha, torch.float32, (q, N, G), "alpha")
    _need(packed, torch.int32, (q, N, K // 32), "packed")
    if planes_i8 is not None:
        _need(planes_i8, torch.int8, (q, N, K), "planes_i8")
    wp, wb = _ws(workspace)
    _check(load().bcq_quantize_grouped(_ptr(W), N, K, g, q, _ptr(alpha), _ptr(packed), _ptr(planes_i8), wp, wb,
                                       _stream()), "bcq_quantize_grouped")
    return alpha, packed, planes_i8


def bcq_linear_fwd_grouped(packed, alpha, x, g, y=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    g = int(g)
    dt = _act_dtype(x)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N, K // max(g, 1)), "alpha")
    _need(x, x.dtype, (T, K), "x")
    y = torch.empty((T, N), dtype=x.dtype, device=x.device) if y is None else y
    _need(y, x.dtype, (T, N), "y")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_fwd_grouped(_ptr(packed), _ptr(alpha), _ptr(x), dt, T, N, K, g, q, _ptr(y), wp, wb,
                                         _stream()), "bcq_linear_fwd_grouped")
    return y


def bcq_linear_bwd_input_grouped(packed, alpha, dy, g, packed_t=None, dx=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = dy.shape[0]
    g = int(g)
    dt = _act_dtype(dy)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(alpha, torch.float32, (q, N, K // max(g, 1)), "alpha")
    _need(dy, dy.dtype, (T, N), "dy")
    if packed_t is not None:
        _need(packed_t, torch.int32, (q, K, N // 32), "packed_t")
    dx = torch.empty((T, K), dtype=dy.dtype, device=dy.device) if dx is None else dx
    _need(dx, dy.dtype, (T, K), "dx")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_bwd_input_grouped(_ptr(packed), _ptr(packed_t), _ptr(alpha), _ptr(dy), dt, T, N, K, g,
                                               q, _ptr(dx), wp, wb, _stream()), "bcq_linear_bwd_input_grouped")
    return dx


def bcq_linear_bwd_alpha_grouped(packed, x, dy, g, q_train=None, grad_scale=1.0, dalpha=None, workspace=None):
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    g = int(g)
    dt = _act_dtype(x)
    q_train = q if q_train is None else int(q_train)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(x, x.dtype, (T, K), "x")
    _need(dy, x.dtype, (T, N), "dy")
    G = K // max(g, 1)
    dalpha = torch.empty((q_train, N, G), dtype=torch.float32, device=x.device) if dalpha is None else dalpha
    _need(dalpha, torch.float32, (q_train, N, G), "dalpha")
    wp, wb = _ws(workspace)
    _check(load().bcq_linear_bwd_alpha_grouped(_ptr(packed), _ptr(x), _ptr(dy), dt, T, N, K, g, q, q_train,
                                               float(grad_scale), _ptr(dalpha), wp, wb, _stream()),
           "bcq_linear_bwd_alpha_grouped")
    return dalpha


def bcq_quantize_alternating(W, q, iters=15, g=None, alpha=None, packed=None, planes_i8=None, want_planes=False,
                             workspace=None):
    """Alternating quantizer (greedy start + `iters` rounds of least-squares refit and nearest-level re-assignment)
    -> (alpha[q,N,K/g] f32, packed[q,N,K/32], planes_i8 or None); g=None is row-wise (alpha[q,N,1])."""
    N, K = W.shape
    g = K if g is None else int(g)
    G = K // max(g, 1)
    _need(W, torch.float32, (N, K), "W")
    dev = W.device
    alpha = torch.empty((q, N, G), dtype=torch.float32, device=dev) if alpha is None else alpha
    packed = torch.empty((q, N, K // 32), dtype=torch.int32, device=dev) if packed is None else packed
    if planes_i8 is None and want_planes:
        planes_i8 = torch.empty((q, N, K), dtype=torch.int8, device=dev)
    _need(alpha, torch.float32, (q, N, G), "alpha")
    _need(packed, torch.int32, (q, N, K // 32), "packed")
    if planes_i8 is not None:
        _need(planes_i8, torch.int8, (q, N, K), "planes_i8")
    wp, wb = _ws(workspace)
    _check(load().bcq_quantize_alternating(_ptr(W), N, K, g, q, int(iters), _ptr(alpha), _ptr(packed),
                                           _ptr(planes_i8), wp, wb, _stream()), "bcq_quantize_alternating")
    return alpha, packed, planes_i8


def _adamw(step, lr, beta1, beta2, eps, weight_decay):
    return AdamW(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step))


def bcq_alpha_adamw_step(alpha, dalpha, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """AdamW step on the first dalpha.numel() scales of `alpha` (the trained planes), in place."""
    count = dalpha.numel()
    for t, name in ((alpha, "alpha"), (dalpha, "dalpha"), (m, "m"), (v, "v")):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32):
            raise ValueError("%s must be a contiguous float32 cuda tensor" % name)
    if alpha.numel() < count or m.numel() != count or v.numel() != count:
        raise ValueError("alpha must hold at least, and m, v exactly, dalpha.numel() elements")
    opt = _adamw(step, lr, beta1, beta2, eps, weight_decay)
    _check(load().bcq_alpha_adamw_step(_ptr(alpha), _ptr(dalpha), _ptr(m), _ptr(v), count, ctypes.byref(opt),
                                       _stream()), "bcq_alpha_adamw_step")
    return alpha


def bcq_linear_bwd_alpha_adamw(packed, x, dy, g, alpha, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                               weight_decay=0.0, q_train=None, grad_scale=1.0, dalpha=None, workspace=None):
    """Scale gradient + AdamW step on alpha[:q_train] in one call; returns dalpha."""
    q, N, Kw = packed.shape
    K = Kw * 32
    T = x.shape[0]
    g = int(g)
    dt = _act_dtype(x)
    q_train = q if q_train is None else int(q_train)
    G = K // max(g, 1)
    _need(packed, torch.int32, (q, N, Kw), "packed")
    _need(x, x.dtype, (T, K), "x")
    _need(dy, x.dtype, (T, N), "dy")
    _need(alpha, torch.float32, (q, N, G), "alpha")
    _need(m, torch.float32, (q_train, N, G), "m")
    _need(v, torch.float32, (q_train, N, G), "v")
    dalpha = torch.empty((q_train, N, G), dtype=torch.float32, device=x.device) if dalpha is None else dalpha
    _need(dalpha, torch.float32, (q_train, N, G), "dalpha")
    wp, wb = _ws(workspace)
    opt = _adamw(step, lr, beta1, beta2, eps, weight_decay)
    _check(load().bcq_linear_bwd_alpha_adamw(_ptr(packed), _ptr(x), _ptr(dy), dt, T, N, K, g, q, q_train,
                                             float(grad_scale), _ptr(dalpha), _ptr(alpha), _ptr(m), _ptr(v),
                                             ctypes.byref(opt), wp, wb, _stream()), "bcq_linear_bwd_alpha_adamw")
    return dalpha


# ---- batched small-token calls: one operation over many independent layers in two launches ---------------------

class BatchPlan:
    """A planned batch: the plan bytes on the host and their device copy, the workspace, and the tensors the plan
    points at (kept alive here).  Run it with bcq_linear_batched(plan), any number of times."""

    def __init__(self, op, T, q, q_train, table_host, table_dev, workspace, keep):
        self.op, self.T, self.q, self.q_train = op, T, q, q_train
        self.table_host, self.table_dev, self.workspace, self._keep = table_host, table_dev, workspace, keep


def batch_plan(op, layers, T, q, q_train=None, grad_scale=1.0, workspace=None):
    """layers: list of dicts with the tensors the op reads and writes (bcq_batch_layer of include/bcq.h: tiled,
    tiled_t, alpha, x, dy, y, dx, dalpha) plus N and K; tiled = bcq_pack_decode(packed), tiled_t =
    bcq_pack_decode(bcq_pack_transposed(packed)).  Builds the plan on the host, uploads it, allocates the
    workspace (or checks the one given)."""
    q_train = q if q_train is None else int(q_train)
    n = len(layers)
    arr = (BatchLayer * n)()
    keep = []
    for i, L in enumerate(layers):
        for name in ("tiled", "tiled_t", "alpha", "x", "dy", "y", "dx", "dalpha"):
            t = L.get(name)
            if t is not None:
                if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
                    raise ValueError("%s of layer %d must be a contiguous cuda tensor" % (name, i))
                keep.append(t)
            setattr(arr[i], name, None if t is None else t.data_ptr())
        arr[i].N, arr[i].K = int(L["N"]), int(L["K"])
    tb, wb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load().bcq_batch_sizes(op, arr, n, T, q, q_train, BCQ_BF16, ctypes.byref(tb), ctypes.byref(wb)),
           "bcq_batch_sizes")
    host = torch.empty((tb.value,), dtype=torch.uint8).pin_memory() if torch.cuda.is_available() else \
        torch.empty((tb.value,), dtype=torch.uint8)
    _check(load().bcq_batch_plan(op, arr, n, T, q, q_train, float(grad_scale), BCQ_BF16,
                                 ctypes.c_void_p(host.data_ptr()), tb.value), "bcq_batch_plan")
    dev = host.cuda()
    if workspace is None:
        workspace = torch.empty((max(wb.value, 16),), dtype=torch.uint8, device=dev.device)
    elif workspace.numel() * workspace.element_size() < wb.value:
        raise ValueError("workspace too small: %d bytes needed" % wb.value)
    return BatchPlan(op, T, q, q_train, host, dev, workspace, keep)


def bcq_linear_batched(plan):
    wp, wbytes = _ws(plan.workspace)
    _check(load().bcq_linear_batched(ctypes.c_void_p(plan.table_host.data_ptr()), _ptr(plan.table_dev),
                                     plan.table_host.numel(), wp, wbytes, _stream()), "bcq_linear_batched")


def bcq_batch_prepare(plan):
    """Host-side set-up of bcq_linear_batched for this plan (before a first call inside a graph capture)."""
    _check(load().bcq_batch_prepare(ctypes.c_void_p(plan.table_host.data_ptr()), plan.table_host.numel()),
           "bcq_batch_prepare")


def bcq_prepare(op, T, N, K, q, dtype=BCQ_BF16, g=None):
    """Host-side set-up for later calls of `op` with these shapes (before a first call inside a graph capture)."""
    _check(load().bcq_prepare(op, T, N, K, K if g is None else int(g), q, dtype), "bcq_prepare")
