// C-ABI layer: argument validation, path selection, kernel enqueue.  See include/bcq.h for the contract.
#include "../../include/bcq.h"

#include "bcq_internal.h"

#include <math.h>
#include <string.h>

#include <atomic>

thread_local bool bcq::tl_dry_run = false;

// One capability probe per device, cached: 0 = unknown, 1 = gfx950, 2 = anything else.  Racing first calls store
// the same value.
bool bcq::host::device_ok() {
    static std::atomic<int> cache[64];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return false;
    }
    int c = cache[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        c = (strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : 2;
        cache[dev].store(c, std::memory_order_relaxed);
    }
    return c == 1;
}

namespace {

using bcq::host::kMaxElems;
using bcq::host::misaligned;

bcq_status check_shape(int64_t T, int64_t N, int64_t K, int q) {
    return bcq::host::shape_ok(T, N, K, q) ? BCQ_OK : BCQ_ERR_SHAPE;
}

// Group size along K: a multiple of 32 (a packed word never straddles two groups) that divides K.
bcq_status check_group(int64_t K, int64_t g) {
    if (g < 32 || g > K || g % 32 != 0 || K % g != 0) return BCQ_ERR_SHAPE;
    return BCQ_OK;
}

bcq_status check_device() { return bcq::host::device_ok() ? BCQ_OK : BCQ_ERR_DEVICE; }

inline bcq_status done(hipError_t e) { return e == hipSuccess ? BCQ_OK : BCQ_ERR_DEVICE; }

bcq_status check_workspace(const void* ws, size_t have, size_t need) {
    if (!ws) return BCQ_OK;
    if (misaligned(ws)) return BCQ_ERR_ALIGN;
    if (have < need) return BCQ_ERR_WORKSPACE;
    return BCQ_OK;
}

// Token count from which the tiled matrix-core kernels are used (bf16 activations, workspace given).
constexpr int64_t kMfmaMinTokens = 32;

// Small-token kernels: bf16, fewer tokens than the tiled kernels want, row-wise scales (they apply alpha after
// the contraction over all of K).  Group-wise scales take the tiled kernels at every token count.
bool small_fwd_ok(int64_t T, bool rowwise, int dtype) { return dtype == BCQ_BF16 && rowwise && T < kMfmaMinTokens; }
bool small_bwd_alpha_ok(int64_t T, bool rowwise, int dtype) { return dtype == BCQ_BF16 && rowwise && T <= 16; }

// Streaming kernels (need a workspace): row-wise scales, or group-wise scales whose groups are whole 512-column
// segments (forward, scale gradient); the input gradient takes any group size (one activation set per plane and
// group, at most kStreamMaxSets of them).  They take one pass over the planes per 16-token tile, and up to the
// token counts below that is still faster than expanding the weights for the tiled matrix-core kernels, whose few
// token tiles leave most of the chip idle (measured on 7680 x 2560, 10240 x 2560, 2560 x 10240: forward 17 - 39 us
// against 41 - 100 us at 32 - 80 tokens, input gradient 33 - 50 us against 43 - 102 us at 32 - 48 tokens).
constexpr int64_t kStreamMaxSets = 256;
constexpr int64_t kStreamFwdMaxTokens = 80;
constexpr int64_t kStreamDxMaxTokens = 48;
bool stream_group_ok(int64_t K, int64_t g) { return g == K || g % 512 == 0; }
bool stream_fwd_ok(int64_t T, int64_t K, int64_t g, int dtype) {
    return dtype == BCQ_BF16 && T <= kStreamFwdMaxTokens && stream_group_ok(K, g);
}
bool stream_bwd_alpha_ok(int64_t T, int64_t K, int64_t g, int dtype) {
    return dtype == BCQ_BF16 && T <= 16 && stream_group_ok(K, g);
}
bool stream_bwd_input_ok(int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype) {
    return dtype == BCQ_BF16 && T <= kStreamDxMaxTokens && N % 32 == 0 && q * (K / g) <= kStreamMaxSets;
}

bool mfma_fwd_ok(int64_t T, bool rowwise, int dtype) {
    return dtype == BCQ_BF16 && (T >= kMfmaMinTokens || !rowwise);
}
bool mfma_bwd_input_ok(int64_t T, int64_t N, bool rowwise, int dtype) {
    return dtype == BCQ_BF16 && (T >= kMfmaMinTokens || !rowwise) && N % 8 == 0;  // rows of dy 16-byte aligned
}
bool mfma_bwd_alpha_ok(int64_t T, int64_t N, int64_t K, bool rowwise, int dtype) {
    return dtype == BCQ_BF16 && (T > 16 || !rowwise) && N % 8 == 0 && N >= 8 && K >= 8;  // rows of dy 16-byte aligned
}

size_t workspace_need(int op, int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype) {
    const bool rowwise = (g == K);
    switch (op) {
        case BCQ_OP_QUANTIZE: return 16;  // status word
        case BCQ_OP_FWD:
            if (stream_fwd_ok(T, K, g, dtype)) return bcq::stream_fwd_workspace(T, K);
            return mfma_fwd_ok(T, rowwise, dtype) ? bcq::mfma_fwd_workspace(N, K) : 0;
        case BCQ_OP_BWD_INPUT: {
            // which path runs depends on the twin being passed, so the size covers both candidates
            const size_t a = stream_bwd_input_ok(T, N, K, g, q, dtype)
                                 ? bcq::stream_bwd_input_workspace(T, N, (int)(q * (K / g))) : 0;
            const size_t b = mfma_bwd_input_ok(T, N, rowwise, dtype) ? bcq::mfma_bwd_input_workspace(N, K) : 0;
            return a > b ? a : b;
        }
        case BCQ_OP_BWD_ALPHA:
            if (stream_bwd_alpha_ok(T, K, g, dtype)) return bcq::stream_bwd_alpha_workspace(T, K);
            return mfma_bwd_alpha_ok(T, N, K, rowwise, dtype) ? bcq::mfma_bwd_alpha_workspace(T, N, K, g, q) : 0;
        default: return 0;
    }
}

}  // namespace

extern "C" {

const char* bcq_status_string(bcq_status s) {
    switch (s) {
        case BCQ_OK: return "ok";
        case BCQ_ERR_NULL: return "a required pointer is NULL";
        case BCQ_ERR_SHAPE: return "unsupported shape (need N,K,T >= 1, 1 <= q <= 8, K % 32 == 0, sizes within limits)";
        case BCQ_ERR_DTYPE: return "unknown dtype or op code";
        case BCQ_ERR_ALIGN: return "pointer not 16-byte aligned";
        case BCQ_ERR_WORKSPACE: return "workspace smaller than bcq_workspace_bytes()";
        case BCQ_ERR_NONFINITE: return "non-finite weights";
        case BCQ_ERR_DEVICE: return "no usable gfx950 device or HIP failure";
    }
    return "unknown status";
}

int bcq_abi_version(void) { return 9; }

bcq_status bcq_workspace_bytes_grouped(int op, int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype,
                                       size_t* out) {
    if (!out) return BCQ_ERR_NULL;
    if (op < BCQ_OP_QUANTIZE || op > BCQ_OP_BWD_ALPHA) return BCQ_ERR_DTYPE;
    if (op == BCQ_OP_QUANTIZE) T = 1;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (dtype != BCQ_F32 && dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    *out = workspace_need(op, T, N, K, g, q, dtype);
    return BCQ_OK;
}

bcq_status bcq_workspace_bytes(int op, int64_t T, int64_t N, int64_t K, int q, int dtype, size_t* out) {
    return bcq_workspace_bytes_grouped(op, T, N, K, K, q, dtype, out);
}

bcq_status bcq_quantize_grouped(const float* W, int64_t N, int64_t K, int64_t g, int q, float* alpha,
                                uint32_t* packed, int8_t* planes_i8, void* workspace, size_t workspace_bytes,
                                void* stream) {
    if (!W || !alpha || !packed) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (g > BCQ_QUANTIZE_MAX_K) return BCQ_ERR_SHAPE;
    const int64_t vectors = N * (K / g);  // one workgroup each
    if (vectors > 0x7FFFFFFF) return BCQ_ERR_SHAPE;
    if (misaligned(W) || misaligned(alpha) || misaligned(packed) || misaligned(planes_i8)) return BCQ_ERR_ALIGN;
    s = check_workspace(workspace, workspace_bytes, workspace_need(BCQ_OP_QUANTIZE, 1, N, K, g, q, BCQ_F32));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    // W[N][K] row-major is also [N K / g][g] row-major, and alpha, packed and planes_i8 keep their layouts under
    // that view: group-wise quantization is the row-wise kernel on the reshaped matrix.
    return done(bcq::launch_quantize(W, vectors, g, q, alpha, packed, planes_i8, (int*)workspace, (hipStream_t)stream));
}

bcq_status bcq_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                        int8_t* planes_i8, void* workspace, size_t workspace_bytes, void* stream) {
    return bcq_quantize_grouped(W, N, K, K, q, alpha, packed, planes_i8, workspace, workspace_bytes, stream);
}

bcq_status bcq_quantize_alternating(const float* W, int64_t N, int64_t K, int64_t g, int q, int iters, float* alpha,
                                    uint32_t* packed, int8_t* planes_i8, void* workspace, size_t workspace_bytes,
                                    void* stream) {
    if (!W || !alpha || !packed) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (g > BCQ_QUANTIZE_MAX_K || iters < 0 || iters > BCQ_ALTERNATING_MAX_ITERS) return BCQ_ERR_SHAPE;
    const int64_t vectors = N * (K / g);
    if (vectors > 0x7FFFFFFF) return BCQ_ERR_SHAPE;
    if (misaligned(W) || misaligned(alpha) || misaligned(packed) || misaligned(planes_i8)) return BCQ_ERR_ALIGN;
    s = check_workspace(workspace, workspace_bytes, workspace_need(BCQ_OP_QUANTIZE, 1, N, K, g, q, BCQ_F32));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_quantize_alternating(W, vectors, g, q, iters, alpha, packed, planes_i8, (int*)workspace,
                                                 (hipStream_t)stream));
}

bcq_status bcq_pack(const int8_t* planes_i8, int64_t N, int64_t K, int q, uint32_t* packed, void* stream) {
    if (!planes_i8 || !packed) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    if (misaligned(planes_i8) || misaligned(packed)) return BCQ_ERR_ALIGN;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_pack(planes_i8, (int64_t)q * N * (K / 32), packed, (hipStream_t)stream));
}

bcq_status bcq_unpack(const uint32_t* packed, int64_t N, int64_t K, int q, int8_t* planes_i8, void* stream) {
    if (!planes_i8 || !packed) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    if (misaligned(planes_i8) || misaligned(packed)) return BCQ_ERR_ALIGN;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_unpack(packed, (int64_t)q * N * (K / 32), planes_i8, (hipStream_t)stream));
}

bcq_status bcq_pack_transposed(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* packed_t,
                               void* stream) {
    if (!packed || !packed_t) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    if (N % 32 != 0) return BCQ_ERR_SHAPE;
    if (misaligned(packed) || misaligned(packed_t)) return BCQ_ERR_ALIGN;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_pack_transposed(packed, N, K, q, packed_t, (hipStream_t)stream));
}

bcq_status bcq_linear_fwd_grouped(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                                  int64_t N, int64_t K, int64_t g, int q, void* y, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    if (!packed || !alpha || !x || !y) return BCQ_ERR_NULL;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (dtype != BCQ_F32 && dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (misaligned(packed) || misaligned(alpha) || misaligned(x) || misaligned(y)) return BCQ_ERR_ALIGN;
    s = check_workspace(workspace, workspace_bytes, workspace_need(BCQ_OP_FWD, T, N, K, g, q, dtype));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    const bool rowwise = (g == K);
    hipStream_t st = (hipStream_t)stream;
    if (workspace && stream_fwd_ok(T, K, g, dtype))
        return done(bcq::launch_fwd_stream(packed, alpha, x, T, N, K, g, q, y, workspace, st));
    if (small_fwd_ok(T, rowwise, dtype)) return done(bcq::launch_fwd_small(packed, alpha, x, T, N, K, q, y, st));
    if (workspace && mfma_fwd_ok(T, rowwise, dtype))
        return done(bcq::launch_fwd_mfma(packed, alpha, x, T, N, K, g, q, y, workspace, st));
    return done(bcq::launch_fwd_generic(packed, alpha, x, dtype, T, N, K, g, q, y, st));
}

bcq_status bcq_decode_layout_bytes(int64_t N, int64_t K, int q, size_t* out) {
    if (!out) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    *out = bcq::decode_layout_bytes(N, K, q);
    return BCQ_OK;
}

bcq_status bcq_pack_decode(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* tiled, void* stream) {
    if (!packed || !tiled) return BCQ_ERR_NULL;
    bcq_status s = check_shape(1, N, K, q);
    if (s != BCQ_OK) return s;
    if (misaligned(packed) || misaligned(tiled)) return BCQ_ERR_ALIGN;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_pack_decode(packed, N, K, q, tiled, (hipStream_t)stream));
}

bcq_status bcq_linear_fwd_decode(const uint32_t* tiled, const float* alpha, const void* x, int dtype, int64_t T,
                                 int64_t N, int64_t K, int64_t g, int q, void* y, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (!tiled || !alpha || !x || !y || !workspace) return BCQ_ERR_NULL;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (!stream_fwd_ok(T, K, g, dtype)) return BCQ_ERR_SHAPE;  // at most 80 tokens; row-wise or g % 512 == 0
    if (misaligned(tiled) || misaligned(alpha) || misaligned(x) || misaligned(y)) return BCQ_ERR_ALIGN;
    s = check_workspace(workspace, workspace_bytes, bcq::stream_fwd_workspace(T, K));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_fwd_stream_decode(tiled, alpha, x, T, N, K, g, q, y, workspace, (hipStream_t)stream));
}

bcq_status bcq_linear_fwd(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                          int64_t N, int64_t K, int q, void* y, void* workspace, size_t workspace_bytes,
                          void* stream) {
    return bcq_linear_fwd_grouped(packed, alpha, x, dtype, T, N, K, K, q, y, workspace, workspace_bytes, stream);
}

bcq_status bcq_linear_bwd_input_grouped(const uint32_t* packed, const uint32_t* packed_t, const float* alpha,
                                        const void* dy, int dtype, int64_t T, int64_t N, int64_t K, int64_t g,
                                        int q, void* dx, void* workspace, size_t workspace_bytes, void* stream) {
    if (!packed || !alpha || !dy || !dx) return BCQ_ERR_NULL;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (packed_t && N % 32 != 0) return BCQ_ERR_SHAPE;
    if (dtype != BCQ_F32 && dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (misaligned(packed) || misaligned(packed_t) || misaligned(alpha) || misaligned(dy) || misaligned(dx))
        return BCQ_ERR_ALIGN;
    s = check_workspace(workspace, workspace_bytes, workspace_need(BCQ_OP_BWD_INPUT, T, N, K, g, q, dtype));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    const bool rowwise = (g == K);
    hipStream_t st = (hipStream_t)stream;
    if (workspace && packed_t && stream_bwd_input_ok(T, N, K, g, q, dtype))
        return done(bcq::launch_bwd_input_stream(packed_t, alpha, dy, T, N, K, g, q, dx, workspace, st));
    if (workspace && mfma_bwd_input_ok(T, N, rowwise, dtype))
        return done(bcq::launch_bwd_input_mfma(packed, packed_t, alpha, dy, T, N, K, g, q, dx, workspace, st));
    return done(bcq::launch_bwd_input_generic(packed, alpha, dy, dtype, T, N, K, g, q, dx, st));
}

bcq_status bcq_linear_bwd_input(const uint32_t* packed, const uint32_t* packed_t, const float* alpha,
                                const void* dy, int dtype, int64_t T, int64_t N, int64_t K, int q, void* dx,
                                void* workspace, size_t workspace_bytes, void* stream) {
    return bcq_linear_bwd_input_grouped(packed, packed_t, alpha, dy, dtype, T, N, K, K, q, dx, workspace,
                                        workspace_bytes, stream);
}

namespace {

// Checks the optimizer arguments and turns them into the kernels' form.  Pure host arithmetic.
bcq_status make_adamw(const bcq_adamw* opt, float* alpha, float* m, float* v, bcq::AdamWArgs* out) {
    if (!opt || !alpha || !m || !v) return BCQ_ERR_NULL;
    if (!(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) || opt->step < 1 ||
        !(opt->eps >= 0.f) || !(opt->lr == opt->lr) || !(opt->weight_decay == opt->weight_decay))
        return BCQ_ERR_SHAPE;
    if (misaligned(alpha) || misaligned(m) || misaligned(v)) return BCQ_ERR_ALIGN;
    out->alpha = alpha;
    out->m = m;
    out->v = v;
    out->lr = opt->lr;
    out->beta1 = opt->beta1;
    out->beta2 = opt->beta2;
    out->eps = opt->eps;
    out->weight_decay = opt->weight_decay;
    out->inv_bc1 = (float)(1.0 / (1.0 - pow((double)opt->beta1, (double)opt->step)));
    out->inv_bc2 = (float)(1.0 / (1.0 - pow((double)opt->beta2, (double)opt->step)));
    return BCQ_OK;
}

bcq_status bwd_alpha_impl(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T, int64_t N,
                          int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                          const bcq_adamw* opt, float* alpha, float* m, float* v, bool with_opt, void* workspace,
                          size_t workspace_bytes, void* stream);

}  // namespace

bcq_status bcq_alpha_adamw_step(float* alpha, const float* dalpha, float* m, float* v, int64_t count,
                                const bcq_adamw* opt, void* stream) {
    if (!dalpha) return BCQ_ERR_NULL;
    bcq::AdamWArgs args;
    bcq_status s = make_adamw(opt, alpha, m, v, &args);
    if (s != BCQ_OK) return s;
    if (count < 1 || count > kMaxElems) return BCQ_ERR_SHAPE;
    if (misaligned(dalpha)) return BCQ_ERR_ALIGN;
    s = check_device();
    if (s != BCQ_OK) return s;
    return done(bcq::launch_adamw(dalpha, count, args, (hipStream_t)stream));
}

bcq_status bcq_linear_bwd_alpha_adamw(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                      int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                      float* dalpha, float* alpha, float* m, float* v, const bcq_adamw* opt,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_alpha_impl(packed, x, dy, dtype, T, N, K, g, q, q_train, grad_scale, dalpha, opt, alpha, m, v, true,
                          workspace, workspace_bytes, stream);
}

bcq_status bcq_linear_bwd_alpha_grouped(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                        int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                        float* dalpha, void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_alpha_impl(packed, x, dy, dtype, T, N, K, g, q, q_train, grad_scale, dalpha, nullptr, nullptr, nullptr,
                          nullptr, false, workspace, workspace_bytes, stream);
}

}  // extern "C"

namespace {

bcq_status bwd_alpha_impl(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T, int64_t N,
                          int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                          const bcq_adamw* opt, float* alpha, float* m, float* v, bool with_opt, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!packed || !x || !dy || !dalpha) return BCQ_ERR_NULL;
    bcq::AdamWArgs oargs = {};
    if (with_opt && (!opt || !alpha || !m || !v)) return BCQ_ERR_NULL;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (q_train < 1 || q_train > q) return BCQ_ERR_SHAPE;
    if (dtype != BCQ_F32 && dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (misaligned(packed) || misaligned(x) || misaligned(dy) || misaligned(dalpha)) return BCQ_ERR_ALIGN;
    if (with_opt) {
        s = make_adamw(opt, alpha, m, v, &oargs);
        if (s != BCQ_OK) return s;
    }
    s = check_workspace(workspace, workspace_bytes, workspace_need(BCQ_OP_BWD_ALPHA, T, N, K, g, q, dtype));
    if (s != BCQ_OK) return s;
    s = check_device();
    if (s != BCQ_OK) return s;
    const bool rowwise = (g == K);
    hipStream_t st = (hipStream_t)stream;
    if (workspace && stream_bwd_alpha_ok(T, K, g, dtype)) {
        hipError_t e = bcq::launch_bwd_alpha_stream(packed, x, dy, T, N, K, g, q, q_train, grad_scale, dalpha, workspace, st);
        if (e == hipSuccess && with_opt) e = bcq::launch_adamw(dalpha, (int64_t)q_train * N * (K / g), oargs, st);
        return done(e);
    }
    if (workspace && !stream_bwd_alpha_ok(T, K, g, dtype) && mfma_bwd_alpha_ok(T, N, K, rowwise, dtype))
        return done(bcq::launch_bwd_alpha_mfma(packed, x, dy, T, N, K, g, q, q_train, grad_scale, dalpha, workspace,
                                               with_opt ? &oargs : nullptr, st));
    hipError_t e;
    if (small_bwd_alpha_ok(T, rowwise, dtype))
        e = bcq::launch_bwd_alpha_small(packed, x, dy, T, N, K, q, q_train, grad_scale, dalpha, st);
    else
        e = bcq::launch_bwd_alpha_generic(packed, x, dy, dtype, T, N, K, g, q, q_train, grad_scale, dalpha, st);
    if (e == hipSuccess && with_opt) e = bcq::launch_adamw(dalpha, (int64_t)q_train * N * (K / g), oargs, st);
    return done(e);
}

}  // namespace

extern "C" {

bcq_status bcq_linear_bwd_alpha(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                int64_t N, int64_t K, int q, int q_train, float grad_scale, float* dalpha,
                                void* workspace, size_t workspace_bytes, void* stream) {
    return bcq_linear_bwd_alpha_grouped(packed, x, dy, dtype, T, N, K, K, q, q_train, grad_scale, dalpha, workspace,
                                        workspace_bytes, stream);
}

}  // extern "C"

namespace {
struct DryRun {  // sets the calling thread's dry-run flag for the lifetime of the object
    DryRun() { bcq::tl_dry_run = true; }
    ~DryRun() { bcq::tl_dry_run = false; }
};
}  // namespace

extern "C" bcq_status bcq_prepare(int op, int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype) {
    if (op < BCQ_OP_QUANTIZE || op > BCQ_OP_BWD_ALPHA) return BCQ_ERR_DTYPE;
    if (op == BCQ_OP_QUANTIZE) T = 1;
    bcq_status s = check_shape(T, N, K, q);
    if (s != BCQ_OK) return s;
    s = check_group(K, g);
    if (s != BCQ_OK) return s;
    if (dtype != BCQ_F32 && dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    s = check_device();
    if (s != BCQ_OK) return s;
    // Stand-in pointers: aligned, never dereferenced (no kernel is launched in a dry run).
    void* const p = reinterpret_cast<void*>((uintptr_t)1 << 20);
    const uint32_t* pu = static_cast<const uint32_t*>(p);
    float* pf = static_cast<float*>(p);
    const size_t ws = workspace_need(op, T, N, K, g, q, dtype);
    DryRun guard;
    const bool twin_ok = (N % 32 == 0);
    for (int with_ws = 0; with_ws < 2 && s == BCQ_OK; ++with_ws) {
        void* w = with_ws ? p : nullptr;
        const size_t wb = with_ws ? (ws > 16 ? ws : 16) : 0;
        switch (op) {
            case BCQ_OP_QUANTIZE:
                if (g <= BCQ_QUANTIZE_MAX_K) s = bcq_quantize_grouped(pf, N, K, g, q, pf, static_cast<uint32_t*>(p), nullptr, w, wb, nullptr);
                break;
            case BCQ_OP_FWD:
                s = bcq_linear_fwd_grouped(pu, pf, p, dtype, T, N, K, g, q, p, w, wb, nullptr);
                if (s == BCQ_OK && with_ws && g == K && dtype == BCQ_BF16 && T <= BCQ_STATIC_MAX_TOKENS &&
                    bcq::stream_fwd_workspace(T, K) <= (size_t)BCQ_STATIC_SCRATCH_BYTES)
                    s = bcq_linear_fwd_static(pu, pf, p, dtype, T, N, K, q, p, nullptr);
                if (s == BCQ_OK && with_ws && g == K && dtype == BCQ_BF16 && T <= BCQ_LUT_MAX_TOKENS &&
                    (size_t)T * (size_t)K * 8 <= (size_t)BCQ_LUT_MAX_TABLE_BYTES)
                    s = bcq_linear_fwd_lut(pu, pf, p, dtype, T, N, K, q, p, nullptr);
                break;
            case BCQ_OP_BWD_INPUT:
                s = bcq_linear_bwd_input_grouped(pu, nullptr, pf, p, dtype, T, N, K, g, q, p, w, wb, nullptr);
                if (s == BCQ_OK && twin_ok) s = bcq_linear_bwd_input_grouped(pu, pu, pf, p, dtype, T, N, K, g, q, p, w, wb, nullptr);
                break;
            default:
                for (int qt = 1; qt <= q && s == BCQ_OK; ++qt)  // the kernels are specialised by the number of trained planes
                    s = bcq_linear_bwd_alpha_grouped(pu, p, p, dtype, T, N, K, g, q, qt, 1.f, pf, w, wb, nullptr);
                break;
        }
    }
    return s;
}

