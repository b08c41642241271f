"""ctypes front end of the CPU oracle (bcq_oracle.c).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's
cpu_baseline leg import this module; the GPU package never does, and this module
imports nothing from it.  All arithmetic lives in bcq_oracle.c (fp64, naive
loops, AlphaTuning Section 3 Eq. 1-2, Section 4.1 Eq. 3-4, Appendix C Eq. ap1-ap3 and its
group-wise paragraph);
this file only marshals numpy arrays and builds the shared object with gcc when
it is missing or older than its source.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcq_oracle.c")
_LIB = os.path.join(_HERE, "libbcq_oracle.so")
_lib = None


def build(force=False):
    """Compile bcq_oracle.c -> libbcq_oracle.so (plain -O2: no fast-math, no reassociation)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


_I64 = ctypes.c_int64
_INT = ctypes.c_int
_DBL = ctypes.c_double


def num_threads():
    return int(_load().orc_num_threads())


def _group(K, g):
    """Group size along K (Table 1 column g): None or K = row-wise; else g must divide K."""
    g = K if g is None else int(g)
    assert 1 <= g <= K and K % g == 0
    return g


def quantize(W, q, with_margin=False, g=None):
    """Greedy BCQ (Appendix C).  W[N,K] fp32 -> alpha[q,N] fp32, planes[q,N,K] int8 (+-1).
    With g < K (group-wise paragraph of Appendix C): alpha[q,N,K/g]."""
    W = _f32(W)
    N, K = W.shape
    g = _group(K, g)
    if g != K:
        alpha = np.empty((q, N, K // g), np.float32)
        planes = np.empty((q, N, K), np.int8)
        margin = np.empty((q, N, K // g), np.float64) if with_margin else None
        _load().orc_quantize_g(_p(W), _I64(N), _I64(K), _I64(g), _INT(q), _p(alpha), _p(planes),
                               _p(margin) if with_margin else None)
        return (alpha, planes, margin) if with_margin else (alpha, planes)
    alpha = np.empty((q, N), np.float32)
    planes = np.empty((q, N, K), np.int8)
    margin = np.empty((q, N), np.float64) if with_margin else None
    _load().orc_quantize(_p(W), _I64(N), _I64(K), _INT(q), _p(alpha), _p(planes),
                         _p(margin) if with_margin else None)
    return (alpha, planes, margin) if with_margin else (alpha, planes)


def quantize_row_forced(w, q, alpha_in, force):
    """Greedy BCQ of one row with alpha_i replaced by alpha_in[i] where force[i]."""
    w = _f32(w)
    K = w.shape[0]
    alpha_in = _f32(alpha_in)
    force = np.ascontiguousarray(force, dtype=np.uint8)
    alpha = np.empty((q,), np.float32)
    planes = np.empty((q, K), np.int8)
    _load().orc_quantize_row_forced(_p(w), _I64(K), _INT(q), _p(alpha_in), _p(force), _p(alpha), _p(planes))
    return alpha, planes


def pack(planes):
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    assert K % 32 == 0
    packed = np.empty((q, N, K // 32), np.uint32)
    _load().orc_pack(_p(planes), _I64(N), _I64(K), _INT(q), _p(packed))
    return packed


def unpack(packed, K):
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    q, N, Kw = packed.shape
    assert Kw * 32 == K
    planes = np.empty((q, N, K), np.int8)
    _load().orc_unpack(_p(packed), _I64(N), _I64(K), _INT(q), _p(planes))
    return planes


def _grouped(alpha, K):
    """Group size implied by the shape of alpha: [q,N] -> K (row-wise), [q,N,G] -> K/G."""
    if alpha.ndim == 2:
        return K
    assert alpha.ndim == 3 and K % alpha.shape[2] == 0
    return K // alpha.shape[2]


def dequant(alpha, planes):
    """Eq. 1: What = sum_i diag(alpha_i) B_i in fp64 (alpha[q,N], or alpha[q,N,K/g] group-wise)."""
    alpha = _f32(alpha)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    What = np.empty((N, K), np.float64)
    if alpha.ndim == 3:
        _load().orc_dequant_g(_p(alpha), _p(planes), _I64(N), _I64(K), _I64(_grouped(alpha, K)), _INT(q), _p(What))
        return What
    _load().orc_dequant(_p(alpha), _p(planes), _I64(N), _I64(K), _INT(q), _p(What))
    return What


def fwd(alpha, planes, x):
    """Eq. 2: y[T,N] fp64.  x[T,K] holds the exact input values as fp32."""
    alpha, x = _f32(alpha), _f32(x)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = x.shape[0]
    assert x.shape == (T, K) and alpha.shape[:2] == (q, N)
    y = np.empty((T, N), np.float64)
    if alpha.ndim == 3:
        _load().orc_fwd_g_at(_p(alpha), _p(planes), _p(x), _I64(T), _I64(N), _I64(K), _I64(_grouped(alpha, K)),
                             _INT(q), None, None, _I64(T * N), _p(y))
        return y
    _load().orc_fwd(_p(alpha), _p(planes), _p(x), _I64(T), _I64(N), _I64(K), _INT(q), _p(y))
    return y


def fwd_at(alpha, planes, x, tt, nn):
    alpha, x = _f32(alpha), _f32(x)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = x.shape[0]
    tt, nn = _i64(tt), _i64(nn)
    out = np.empty((tt.shape[0],), np.float64)
    if alpha.ndim == 3:
        _load().orc_fwd_g_at(_p(alpha), _p(planes), _p(x), _I64(T), _I64(N), _I64(K), _I64(_grouped(alpha, K)),
                             _INT(q), _p(tt), _p(nn), _I64(tt.shape[0]), _p(out))
        return out
    _load().orc_fwd_at(_p(alpha), _p(planes), _p(x), _I64(T), _I64(N), _I64(K), _INT(q),
                       _p(tt), _p(nn), _I64(tt.shape[0]), _p(out))
    return out


def bwd_input(alpha, planes, dy):
    """Eq. 3: dx[T,K] fp64."""
    alpha, dy = _f32(alpha), _f32(dy)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = dy.shape[0]
    assert dy.shape == (T, N)
    dx = np.empty((T, K), np.float64)
    if alpha.ndim == 3:
        _load().orc_bwd_input_g_at(_p(alpha), _p(planes), _p(dy), _I64(T), _I64(N), _I64(K),
                                   _I64(_grouped(alpha, K)), _INT(q), None, None, _I64(T * K), _p(dx))
        return dx
    _load().orc_bwd_input(_p(alpha), _p(planes), _p(dy), _I64(T), _I64(N), _I64(K), _INT(q), _p(dx))
    return dx


def bwd_input_at(alpha, planes, dy, tt, kk):
    alpha, dy = _f32(alpha), _f32(dy)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = dy.shape[0]
    tt, kk = _i64(tt), _i64(kk)
    out = np.empty((tt.shape[0],), np.float64)
    if alpha.ndim == 3:
        _load().orc_bwd_input_g_at(_p(alpha), _p(planes), _p(dy), _I64(T), _I64(N), _I64(K),
                                   _I64(_grouped(alpha, K)), _INT(q), _p(tt), _p(kk), _I64(tt.shape[0]), _p(out))
        return out
    _load().orc_bwd_input_at(_p(alpha), _p(planes), _p(dy), _I64(T), _I64(N), _I64(K), _INT(q),
                             _p(tt), _p(kk), _I64(tt.shape[0]), _p(out))
    return out


def bwd_alpha(planes, x, dy, q_train=None, grad_scale=1.0, g=None):
    """Eq. 4 read as the gradient of Eq. 2: dalpha[q_train,N] fp64; with g < K: dalpha[q_train,N,K/g]."""
    x, dy = _f32(x), _f32(dy)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = x.shape[0]
    q_train = q if q_train is None else q_train
    assert x.shape == (T, K) and dy.shape == (T, N) and 1 <= q_train <= q
    g = _group(K, g)
    if g != K:
        out = np.empty((q_train, N, K // g), np.float64)
        _load().orc_bwd_alpha_g_rows(_p(planes), _p(x), _p(dy), _I64(T), _I64(N), _I64(K), _I64(g), _INT(q),
                                     _INT(q_train), _DBL(grad_scale), None, _I64(N), _p(out))
        return out
    out = np.empty((q_train, N), np.float64)
    _load().orc_bwd_alpha(_p(planes), _p(x), _p(dy), _I64(T), _I64(N), _I64(K), _INT(q), _INT(q_train),
                          _DBL(grad_scale), _p(out))
    return out


def bwd_alpha_rows(planes, x, dy, rows, q_train=None, grad_scale=1.0, g=None):
    x, dy = _f32(x), _f32(dy)
    planes = np.ascontiguousarray(planes, dtype=np.int8)
    q, N, K = planes.shape
    T = x.shape[0]
    q_train = q if q_train is None else q_train
    rows = _i64(rows)
    g = _group(K, g)
    if g != K:
        out = np.empty((q_train, rows.shape[0], K // g), np.float64)
        _load().orc_bwd_alpha_g_rows(_p(planes), _p(x), _p(dy), _I64(T), _I64(N), _I64(K), _I64(g), _INT(q),
                                     _INT(q_train), _DBL(grad_scale), _p(rows), _I64(rows.shape[0]), _p(out))
        return out
    out = np.empty((q_train, rows.shape[0]), np.float64)
    _load().orc_bwd_alpha_rows(_p(planes), _p(x), _p(dy), _I64(T), _I64(N), _I64(K), _INT(q), _INT(q_train),
                               _DBL(grad_scale), _p(rows), _I64(rows.shape[0]), _p(out))
    return out


def storage_bytes(N, K, q, g=None):
    """Bytes of a BCQ matrix with 1-bit signs and fp32 scales: q*(N*K/8 + 4*N*K/g) (Table 1)."""
    g = K if g is None else g
    return q * (N * K // 8 + 4 * N * K // g)


def quantize_alternating(W, q, iters=15, g=None, with_margin=False):
    """Alternating quantizer (Appendix C, Eq. ap4): greedy start, then `iters` rounds of least-squares refit of
    alpha and nearest-level re-assignment of the signs.  Returns alpha[q,N] (or [q,N,K/g]) fp32, planes[q,N,K];
    with_margin also margin[N*K/g, 2] (decision gap, fp32 rounding margin) and the iterations done per vector."""
    W = _f32(W)
    N, K = W.shape
    g = _group(K, g)
    assert 1 <= q <= 8
    V = N * (K // g)
    alpha = np.empty((q, N, K // g), np.float32)
    planes = np.empty((q, N, K), np.int8)
    margin = np.empty((V, 2), np.float64) if with_margin else None
    done = np.empty((V,), np.int32) if with_margin else None
    _load().orc_quantize_alternating(_p(W), _I64(N), _I64(K), _I64(g), _INT(q), _INT(iters), _p(alpha), _p(planes),
                                     _p(margin) if with_margin else None, _p(done) if with_margin else None)
    if g == K:
        alpha = alpha[:, :, 0].copy()
    return (alpha, planes, margin, done) if with_margin else (alpha, planes)


def alternating_row_trace(w, q, iters=15):
    """One vector: (alpha[q], planes[q,n], err[iters,2], iterations done); err[it] = squared error before
    iteration it and after its refit (NaN where the loop had already stopped)."""
    w = _f32(w)
    n = w.shape[0]
    alpha = np.empty((q,), np.float32)
    planes = np.empty((q, n), np.int8)
    err = np.full((iters, 2), np.nan, np.float64)
    done = ctypes.c_int(0)
    _load().orc_alternating_row_trace(_p(w), _I64(n), _INT(q), _INT(iters), _p(alpha), _p(planes), _p(err),
                                      ctypes.byref(done))
    return alpha, planes, err, int(done.value)


def adamw_step(alpha, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One AdamW update of the scales (Appendix A: "AdamW optimizer"; the algorithm is that of the cited AdamW
    paper, decoupled weight decay), written out in fp64 numpy:
        m <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2,
        mhat = m / (1 - beta1^t),       vhat = v / (1 - beta2^t),
        alpha <- alpha - lr * (mhat / (sqrt(vhat) + eps) + weight_decay * alpha),      t = step >= 1.
    Returns (alpha, m, v) as new fp64 arrays; the inputs are not modified."""
    a = np.asarray(alpha, dtype=np.float64)
    g = np.asarray(grad, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    a = a - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * a)
    return a, m, v
