// Internal launch interface between the C-ABI layer (bcq_api.hip) and the gfx950 kernels.
// Nothing here is exported; every function enqueues work on `st` and returns the HIP status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace bcq {

// ---- element helpers shared by all kernels -------------------------------------------------
typedef uint16_t bf16_t;  // raw bf16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest even; NaN stays NaN (quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename XT> struct Elem;
template <> struct Elem<float> {
    __device__ static __forceinline__ float load(const float* p) { return *p; }
    __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ---- AdamW on the trained scales (Appendix A; decoupled weight decay) ---------------------------
// Device pointers to the scales and their two moment buffers (fp32, same shape as the scale gradient) plus the
// step's constants; alpha == nullptr means "no update".  inv_bc = 1 / (1 - beta^t), formed in fp64 on the host.
struct AdamWArgs {
    float* alpha;
    float* m;
    float* v;
    float lr, beta1, beta2, eps, weight_decay, inv_bc1, inv_bc2;
};

__device__ __forceinline__ void adamw_apply(const AdamWArgs& o, int64_t idx, float g) {
    const float m = o.beta1 * o.m[idx] + (1.f - o.beta1) * g;
    const float v = o.beta2 * o.v[idx] + (1.f - o.beta2) * g * g;
    o.m[idx] = m;
    o.v[idx] = v;
    const float a = o.alpha[idx];
    o.alpha[idx] = a - o.lr * ((m * o.inv_bc1) / (sqrtf(v * o.inv_bc2) + o.eps) + o.weight_decay * a);
}

// alpha, m, v <- AdamW(alpha, dalpha) over `count` scales
hipError_t launch_adamw(const float* dalpha, int64_t count, AdamWArgs args, hipStream_t st);

// The dynamic-LDS limit of a kernel is a property of (kernel, device).  One instance per kernel remembers, for every
// device of the process, the largest size already allowed there (64 KiB are allowed without asking).  Racing first
// calls from several host threads set the same attribute twice, which is harmless; the record itself is atomic.
struct LdsLimit {
    std::atomic<size_t> allowed[64] = {};
    hipError_t ensure(const void* kernel, size_t bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        const size_t seen = allowed[dev].load(std::memory_order_relaxed);
        const size_t have = seen > (size_t)(64 * 1024) ? seen : (size_t)(64 * 1024);
        if (bytes <= have) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        allowed[dev].store(bytes, std::memory_order_relaxed);
        return hipSuccess;
    }
};

// ---- dry runs ---------------------------------------------------------------------------------------------------
// bcq_prepare / bcq_batch_prepare walk through an entry point's host code with this flag set: path selection and the
// one-time host-side set-up (raising a kernel's dynamic-LDS limit) happen as in a real call, the launches are skipped.
extern thread_local bool tl_dry_run;
#define BCQ_LAUNCH(...)                                   \
    do {                                                  \
        if (!::bcq::tl_dry_run) hipLaunchKernelGGL(__VA_ARGS__); \
    } while (0)

// ---- host-side argument checks shared by the source files that hold C-ABI entry points ------------------
namespace host {
constexpr int64_t kMaxDim = (int64_t)1 << 17;     // N, K
constexpr int64_t kMaxTokens = (int64_t)1 << 24;  // T
constexpr int64_t kMaxElems = (int64_t)1 << 40;   // N*K, T*N, T*K
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline bool shape_ok(int64_t T, int64_t N, int64_t K, int q) {
    if (N < 1 || K < 1 || T < 1 || q < 1 || q > 8 || K % 32 != 0) return false;
    if (N > kMaxDim || K > kMaxDim || T > kMaxTokens) return false;
    return N * K <= kMaxElems && T * N <= kMaxElems && T * K <= kMaxElems;
}
// true when the calling thread's current device is a gfx950 (one probe per device, cached; thread-safe)
bool device_ok();
}  // namespace host

// ---- one-time kernels -----------------------------------------------------------------------
hipError_t launch_pack(const int8_t* planes, int64_t total_words, uint32_t* packed, hipStream_t st);
hipError_t launch_unpack(const uint32_t* packed, int64_t total_words, int8_t* planes, hipStream_t st);
hipError_t launch_pack_transposed(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* packed_t,
                                  hipStream_t st);
hipError_t launch_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                           int8_t* planes, int* status_word, hipStream_t st);

// Alternating quantizer over V vectors of length n (W viewed as [V][n]); alpha[q][V], packed[q][V][n/32].
hipError_t launch_quantize_alternating(const float* W, int64_t V, int64_t n, int q, int iters, float* alpha,
                                       uint32_t* packed, int8_t* planes, int* status_word, hipStream_t st);

// Scales are alpha[q][N][K / g] (g = group size along K, a multiple of 32 that divides K; g = K is the row-wise
// case alpha[q][N]); the scale gradient has the same shape.

// ---- any-shape kernels (plain vector ALU; need no workspace) --------------------------------
hipError_t launch_fwd_generic(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                              int64_t N, int64_t K, int64_t g, int q, void* y, hipStream_t st);
hipError_t launch_bwd_input_generic(const uint32_t* packed, const float* alpha, const void* dy, int dtype,
                                    int64_t T, int64_t N, int64_t K, int64_t g, int q, void* dx, hipStream_t st);
hipError_t launch_bwd_alpha_generic(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                    int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                    float* dalpha, hipStream_t st);

// ---- matrix-core kernels (bf16 activations, need the caller's workspace) ---------------------
size_t mfma_fwd_workspace(int64_t N, int64_t K);
size_t mfma_bwd_input_workspace(int64_t N, int64_t K);
hipError_t launch_fwd_mfma(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                           int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st);
hipError_t launch_bwd_input_mfma(const uint32_t* packed, const uint32_t* packed_t, const float* alpha, const void* dy,
                                 int64_t T, int64_t N, int64_t K, int64_t g, int q, void* dx, void* workspace,
                                 hipStream_t st);
size_t mfma_bwd_alpha_workspace(int64_t T, int64_t N, int64_t K, int64_t g, int q);
// opt != nullptr: the final reduction also applies the AdamW step to the trained scales
hipError_t launch_bwd_alpha_mfma(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                 int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                                 void* workspace, const AdamWArgs* opt, hipStream_t st);

// ---- small-token kernels without workspace (bf16, at most 16 tokens per tile; plane-by-plane, bf16 MFMA) ----
hipError_t launch_fwd_small(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                            int64_t K, int q, void* y, hipStream_t st);
hipError_t launch_bwd_alpha_small(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                  int64_t K, int q, int q_train, float grad_scale, float* dalpha, hipStream_t st);

// ---- small-token kernels on the block-scaled FP4 x FP8 matrix instruction (bf16; row-wise scales, or group-wise
// with g % 512 == 0 for forward / scale gradient; need a workspace for the activations re-coded as two FP8 terms) ----
size_t stream_fwd_workspace(int64_t T, int64_t K);
size_t stream_bwd_alpha_workspace(int64_t T, int64_t K);
size_t stream_bwd_input_workspace(int64_t T, int64_t N, int sets /* q * (K / g) */);
hipError_t launch_fwd_stream(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                             int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st);
hipError_t launch_fwd_stream_decode(const uint32_t* tiled, const float* alpha, const void* x, int64_t T, int64_t N,
                                    int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st);
size_t decode_layout_bytes(int64_t N, int64_t K, int q);
hipError_t launch_pack_decode(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* tiled, hipStream_t st);
hipError_t launch_bwd_alpha_stream(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                   int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                                   void* workspace, hipStream_t st);
hipError_t launch_bwd_input_stream(const uint32_t* packed_t, const float* alpha, const void* dy, int64_t T, int64_t N,
                                   int64_t K, int64_t g, int q, void* dx, void* workspace, hipStream_t st);

}  // namespace bcq
