// Greedy BCQ quantizer (AlphaTuning Appendix C: Eq. ap1 for the first plane, Eq. ap2-ap3 for the rest).
// One 256-thread workgroup per row of W.  The fp64 residual of the whole row stays in registers across the
// q planes, so W is read from HBM exactly once (4 N K bytes) and only alpha and the packed signs are
// written.  HBM bound; the fp64 abs-sum, compare and subtract are a few ALU operations per weight.
//
// Arithmetic (what makes the sign planes reproducible bit for bit): residual and abs-sum in fp64, mean
// rounded once to fp32, that fp32 value subtracted.  Only the ORDER of the fp64 sum is free.
#include "bcq_internal.h"

namespace bcq {

// Wave w of the block owns columns [w*C*64, (w+1)*C*64); lane l holds column w*C*64 + c*64 + l in r[c].
template <int CMAX>
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ W, int64_t N, int K, int q,
                                                       float* __restrict__ alpha, uint32_t* __restrict__ packed,
                                                       int8_t* __restrict__ planes, int* __restrict__ status_word) {
    __shared__ double wave_sum[4];
    const int64_t n = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int C = (K + 255) / 256;  // <= CMAX
    const int kbase = wave * C * 64;
    const float* wrow = W + n * (int64_t)K;
    const int Kw = K / 32;

    double r[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        int k = kbase + c * 64 + lane;
        r[c] = (c < C && k < K) ? (double)wrow[k] : 0.0;
    }

    for (int i = 0; i < q; ++i) {
        double s = 0.0;
        uint64_t mine = 0;  // lane c keeps the 64 sign bits of chunk c
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (c < C) {
                s += fabs(r[c]);
                uint64_t m = __ballot(r[c] >= 0.0);
                if (lane == c) mine = m;
            }
        }
        // workgroup sum of |r| in fp64
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        __syncthreads();  // wave_sum of the previous plane has been read by everyone
        if (lane == 0) wave_sum[wave] = s;
        __syncthreads();
        const double S = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
        const float a = (float)(S / (double)K);
        if (threadIdx.x == 0) {
            alpha[(int64_t)i * N + n] = a;
            if (i == 0 && status_word && !(fabs(S) <= 1.79769313486231570e308)) atomicAdd(status_word, 1);
        }
        // packed words: lane c writes the two words of chunk c (8 bytes, consecutive lanes are contiguous)
        if (lane < C) {
            int k0 = kbase + lane * 64;
            uint32_t* dst = packed + ((int64_t)i * N + n) * Kw + k0 / 32;
            if (k0 < K) dst[0] = (uint32_t)mine;
            if (k0 + 32 < K) dst[1] = (uint32_t)(mine >> 32);
        }
        const double ad = (double)a;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (c < C) {
                const bool pos = r[c] >= 0.0;
                const int k = kbase + c * 64 + lane;
                if (k < K) {  // padding lanes keep r = 0 so that they never add to the abs-sum
                    if (planes) planes[((int64_t)i * N + n) * K + k] = pos ? (int8_t)1 : (int8_t)-1;
                    r[c] = pos ? r[c] - ad : r[c] + ad;  // r - alpha * b with b = +-1
                }
            }
        }
    }
}

__global__ void zero_word_kernel(int* p) { *p = 0; }

template <int CMAX>
static hipError_t launch_q(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                           int8_t* planes, int* status_word, hipStream_t st) {
    hipLaunchKernelGGL(quantize_kernel<CMAX>, dim3((unsigned)N), dim3(256), 0, st, W, N, (int)K, q, alpha, packed,
                       planes, status_word);
    return hipGetLastError();
}

hipError_t launch_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                           int8_t* planes, int* status_word, hipStream_t st) {
    if (status_word) {
        hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, st, status_word);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const int C = (int)((K + 255) / 256);
    if (C <= 4) return launch_q<4>(W, N, K, q, alpha, packed, planes, status_word, st);
    if (C <= 8) return launch_q<8>(W, N, K, q, alpha, packed, planes, status_word, st);
    if (C <= 16) return launch_q<16>(W, N, K, q, alpha, packed, planes, status_word, st);
    if (C <= 24) return launch_q<24>(W, N, K, q, alpha, packed, planes, status_word, st);
    if (C <= 40) return launch_q<40>(W, N, K, q, alpha, packed, planes, status_word, st);
    return launch_q<64>(W, N, K, q, alpha, packed, planes, status_word, st);
}

}  // namespace bcq
