// Any-shape kernels for the BCQ linear layer on the vector ALU (fp32 accumulation, fp32 or bf16 I/O).
// They evaluate AlphaTuning Eq. 2 (forward), Eq. 3 (input gradient) and Eq. 4 (scale gradient, read as the
// gradient of Eq. 2) directly on the packed sign planes, never forming W in memory, and need no workspace.
// The library uses them for fp32 activations, for shapes the tiled matrix-core kernels do not take, and
// whenever the caller passes no workspace.
#include "bcq_internal.h"

namespace bcq {

constexpr int GEN_TT = 8;  // tokens per pass

// sum_j (bit j of w ? +v[j] : -v[j]) over the 32 columns of one packed word
__device__ __forceinline__ float signed_sum32(uint32_t w, const float (&v)[32]) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 32; ++j) s += ((w >> j) & 1u) ? v[j] : -v[j];
    return s;
}

template <typename XT>
__device__ __forceinline__ void load32(const XT* p, float (&v)[32]) {
#pragma unroll
    for (int j = 0; j < 32; ++j) v[j] = Elem<XT>::load(p + j);
}

// Forward, Eq. 2.  One wave per output row n and tile of GEN_TT tokens; lanes stride over the packed words
// of the row, the alpha-weighted plane sum is formed per lane (it is linear), then one wave reduction.
template <typename XT>
__global__ __launch_bounds__(256) void fwd_generic_kernel(const uint32_t* __restrict__ packed,
                                                          const float* __restrict__ alpha, const XT* __restrict__ x,
                                                          XT* __restrict__ y, int64_t T, int64_t N, int64_t K,
                                                          int64_t g, int q) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
    const int64_t t0 = (int64_t)blockIdx.x * GEN_TT;
    if (n >= N) return;  // whole wave leaves together
    const int64_t Kw = K / 32, G = K / g, gw = g / 32;
    float acc[GEN_TT];
#pragma unroll
    for (int t = 0; t < GEN_TT; ++t) acc[t] = 0.f;
    for (int64_t w = lane; w < Kw; w += 64) {
        uint32_t bits[8];
        float a[8];  // scales of the group this word lies in (a word never straddles groups: g % 32 == 0)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            bits[i] = (i < q) ? packed[((int64_t)i * N + n) * Kw + w] : 0u;
            a[i] = (i < q) ? alpha[((int64_t)i * N + n) * G + w / gw] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < GEN_TT; ++t) {
            if (t0 + t < T) {
                float v[32];
                load32<XT>(x + (t0 + t) * K + 32 * w, v);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (i < q) acc[t] += a[i] * signed_sum32(bits[i], v);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < GEN_TT; ++t) {
        float s = acc[t];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0 && t0 + t < T) Elem<XT>::store(y + (t0 + t) * N + n, s);
    }
}

// Scale gradient, Eq. 4 as the gradient of Eq. 2.  One wave per row n; per lane
// g_i += dy[t][n] * (partial of sum_k B_i[n][k] x[t][k] over the lane's words), reduced once at the end.
template <typename XT>
__global__ __launch_bounds__(256) void bwd_alpha_generic_kernel(const uint32_t* __restrict__ packed,
                                                                const XT* __restrict__ x, const XT* __restrict__ dy,
                                                                float* __restrict__ dalpha, int64_t T, int64_t N,
                                                                int64_t K, int64_t g, int q_train, float grad_scale) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const int64_t Kw = K / 32, G = K / g, gw = g / 32;
    for (int64_t grp = 0; grp < G; ++grp) {  // one scale group at a time; the lanes stride over its words
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int64_t w = grp * gw + lane; w < (grp + 1) * gw; w += 64) {
            uint32_t bits[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) bits[i] = (i < q_train) ? packed[((int64_t)i * N + n) * Kw + w] : 0u;
            for (int64_t t = 0; t < T; ++t) {
                float v[32];
                load32<XT>(x + t * K + 32 * w, v);
                const float d = Elem<XT>::load(dy + t * N + n);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (i < q_train) acc[i] += d * signed_sum32(bits[i], v);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < q_train) {
                float s = acc[i];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
                if (lane == 0) dalpha[((int64_t)i * N + n) * G + grp] = grad_scale * s;
            }
        }
    }
}

// Input gradient, Eq. 3.  One thread per output column k and tile of GEN_TT tokens; the loop runs over the
// rows n of W, rebuilding What[n][k] = sum_i +-alpha_i[n] from the thread's bit of each plane.
template <typename XT>
__global__ __launch_bounds__(256) void bwd_input_generic_kernel(const uint32_t* __restrict__ packed,
                                                                const float* __restrict__ alpha,
                                                                const XT* __restrict__ dy, XT* __restrict__ dx,
                                                                int64_t T, int64_t N, int64_t K, int64_t g, int q) {
    const int64_t k = (int64_t)blockIdx.y * 256 + threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * GEN_TT;
    if (k >= K) return;
    const int64_t Kw = K / 32, G = K / g, grp = k / g;
    const int64_t w = k >> 5;
    const int j = (int)(k & 31);
    float acc[GEN_TT];
#pragma unroll
    for (int t = 0; t < GEN_TT; ++t) acc[t] = 0.f;
    for (int64_t n = 0; n < N; ++n) {
        float what = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < q) {
                const float a = alpha[((int64_t)i * N + n) * G + grp];
                const uint32_t b = packed[((int64_t)i * N + n) * Kw + w];
                what += ((b >> j) & 1u) ? a : -a;
            }
        }
#pragma unroll
        for (int t = 0; t < GEN_TT; ++t)
            if (t0 + t < T) acc[t] += Elem<XT>::load(dy + (t0 + t) * N + n) * what;
    }
#pragma unroll
    for (int t = 0; t < GEN_TT; ++t)
        if (t0 + t < T) Elem<XT>::store(dx + (t0 + t) * K + k, acc[t]);
}

hipError_t launch_fwd_generic(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                              int64_t N, int64_t K, int64_t g, int q, void* y, hipStream_t st) {
    dim3 grid((unsigned)((T + GEN_TT - 1) / GEN_TT), (unsigned)((N + 3) / 4));
    if (dtype == 0)
        BCQ_LAUNCH(fwd_generic_kernel<float>, grid, dim3(256), 0, st, packed, alpha, (const float*)x,
                           (float*)y, T, N, K, g, q);
    else
        BCQ_LAUNCH(fwd_generic_kernel<bf16_t>, grid, dim3(256), 0, st, packed, alpha, (const bf16_t*)x,
                           (bf16_t*)y, T, N, K, g, q);
    return hipGetLastError();
}

hipError_t launch_bwd_alpha_generic(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                    int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                    float* dalpha, hipStream_t st) {
    (void)q;
    dim3 grid((unsigned)((N + 3) / 4));
    if (dtype == 0)
        BCQ_LAUNCH(bwd_alpha_generic_kernel<float>, grid, dim3(256), 0, st, packed, (const float*)x,
                           (const float*)dy, dalpha, T, N, K, g, q_train, grad_scale);
    else
        BCQ_LAUNCH(bwd_alpha_generic_kernel<bf16_t>, grid, dim3(256), 0, st, packed, (const bf16_t*)x,
                           (const bf16_t*)dy, dalpha, T, N, K, g, q_train, grad_scale);
    return hipGetLastError();
}

hipError_t launch_bwd_input_generic(const uint32_t* packed, const float* alpha, const void* dy, int dtype,
                                    int64_t T, int64_t N, int64_t K, int64_t g, int q, void* dx, hipStream_t st) {
    dim3 grid((unsigned)((T + GEN_TT - 1) / GEN_TT), (unsigned)((K + 255) / 256));
    if (dtype == 0)
        BCQ_LAUNCH(bwd_input_generic_kernel<float>, grid, dim3(256), 0, st, packed, alpha, (const float*)dy,
                           (float*)dx, T, N, K, g, q);
    else
        BCQ_LAUNCH(bwd_input_generic_kernel<bf16_t>, grid, dim3(256), 0, st, packed, alpha,
                           (const bf16_t*)dy, (bf16_t*)dx, T, N, K, g, q);
    return hipGetLastError();
}

}  // namespace bcq
