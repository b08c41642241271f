// Alternating BCQ quantizer (AlphaTuning Appendix C, "Alternating Method", Eq. ap4): greedy start (Eq. ap1-ap3),
// then `iters` rounds of
//   (1) alpha <- (B^T B)^{-1} B^T w      least-squares refit of the q scales of one vector (Eq. ap4),
//   (2) every element takes the sign pattern whose level sum_i +-alpha_i is nearest to its weight.
// One 256-thread workgroup per vector (a row, or one length-g group of a row).  The vector (fp32) and one byte of
// sign pattern per element stay in LDS for all rounds, so W is read from HBM once.  This is one-time PTQ work:
// the kernel is written for reproducibility, not speed.
//
// Arithmetic: every sum, the Cholesky solve and the level comparison are fp64; alpha is rounded to fp32 once at
// the end.  The loop stops early at a fixed point (round (2) changed nothing) and stops BEFORE a refit whose
// Gram matrix is singular (a Cholesky pivot <= 1e-9 n: two planes equal or opposite, e.g. an all-zero vector),
// keeping the current pair.  Ties between two levels go to the larger level, ties between equal levels to the
// larger pattern index (bit i of the pattern = plane i is +1).  Only the ORDER of the fp64 sums over the
// elements is free.
#include "bcq_internal.h"

namespace bcq {

constexpr int ALT_THREADS = 256;
constexpr int ALT_NRED = 8 + 28;  // right-hand side (q) + strict lower triangle of the Gram matrix (q (q - 1) / 2)

// Sum of `cnt` doubles per thread over the workgroup; every thread returns with all totals (same order in all).
__device__ __forceinline__ void block_sum(double* vals, int cnt, double* scratch /* [4][ALT_NRED] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = 0; i < cnt; ++i) {
        double s = vals[i];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        vals[i] = s;
    }
    __syncthreads();  // scratch of the previous call has been read by everyone
    if (lane == 0)
        for (int i = 0; i < cnt; ++i) scratch[wave * ALT_NRED + i] = vals[i];
    __syncthreads();
    for (int i = 0; i < cnt; ++i)
        vals[i] = (scratch[i] + scratch[ALT_NRED + i]) + (scratch[2 * ALT_NRED + i] + scratch[3 * ALT_NRED + i]);
}

__global__ __launch_bounds__(ALT_THREADS) void alternating_kernel(const float* __restrict__ W, int64_t V, int n, int q,
                                                                  int iters, float* __restrict__ alpha,
                                                                  uint32_t* __restrict__ packed,
                                                                  int8_t* __restrict__ planes,
                                                                  int* __restrict__ status_word) {
    extern __shared__ __attribute__((aligned(16))) unsigned char alt_smem[];
    double* scratch = reinterpret_cast<double*>(alt_smem);                 // [4][ALT_NRED]
    double* lv = scratch + 4 * ALT_NRED;                                    // [256] levels of the current alpha
    float* w = reinterpret_cast<float*>(lv + 256);                          // [n]
    uint8_t* code = reinterpret_cast<uint8_t*>(w + n);                      // [n]
    const int tid = threadIdx.x;
    const int64_t v = blockIdx.x;
    const float* wrow = W + v * (int64_t)n;
    for (int k = tid; k < n; k += ALT_THREADS) w[k] = wrow[k];
    __syncthreads();

    // ---- greedy start: plane i takes the sign of the residual w - sum_{j<i} alpha_j b_j (each element's residual
    // is rebuilt from its pattern so far, by the same chain of fp64 subtractions), alpha_i = fp32(mean |residual|)
    double a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = 0.0;
    for (int i = 0; i < q; ++i) {
        double s = 0.0;
        for (int k = tid; k < n; k += ALT_THREADS) {
            const uint8_t c = (i == 0) ? (uint8_t)0 : code[k];
            double r = (double)w[k];
            for (int j = 0; j < i; ++j) r = ((c >> j) & 1) ? r - a[j] : r + a[j];
            s += fabs(r);
            code[k] = (uint8_t)(c | ((r >= 0.0 ? 1u : 0u) << i));
        }
        block_sum(&s, 1, scratch);
        if (i == 0 && tid == 0 && status_word && !(fabs(s) <= 1.79769313486231570e308)) atomicAdd(status_word, 1);
        a[i] = (double)(float)(s / (double)n);
    }
    __syncthreads();

    const int levels = 1 << q;
    for (int it = 0; it < iters; ++it) {
        // ---- (1) Eq. ap4: right-hand side B^T w and Gram matrix B^T B (diagonal = n), summed over the workgroup
        double red[ALT_NRED];
#pragma unroll
        for (int i = 0; i < ALT_NRED; ++i) red[i] = 0.0;
        for (int k = tid; k < n; k += ALT_THREADS) {
            const uint8_t c = code[k];
            const double x = (double)w[k];
            int p = 8;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i < q) {
                    red[i] += ((c >> i) & 1) ? x : -x;
#pragma unroll
                    for (int j = 0; j < i; ++j) red[p + j] += (((c >> i) ^ (c >> j)) & 1) ? -1.0 : 1.0;
                }
                p += i;
            }
        }
        block_sum(red, ALT_NRED, scratch);
        // Cholesky of the Gram matrix, every thread on its own copy (identical values in all threads)
        double L[8][8], y[8];
        bool singular = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < q && !singular) {
                double d = (double)n;
                for (int p = 0; p < j; ++p) d -= L[j][p] * L[j][p];
                if (!(d > 1e-9 * (double)n)) {
                    singular = true;
                } else {
                    L[j][j] = sqrt(d);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        if (i > j && i < q) {
                            double s = red[8 + i * (i - 1) / 2 + j];
                            for (int p = 0; p < j; ++p) s -= L[i][p] * L[j][p];
                            L[i][j] = s / L[j][j];
                        }
                    }
                }
            }
        }
        if (singular) break;  // uniform: all threads hold the same numbers
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < q) {
                double s = red[i];
                for (int p = 0; p < i; ++p) s -= L[i][p] * y[p];
                y[i] = s / L[i][i];
            }
        }
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            if (i < q) {
                double s = y[i];
                for (int p = i + 1; p < q; ++p) s -= L[p][i] * a[p];
                a[i] = s / L[i][i];
            }
        }
        // ---- (2) levels of the new alpha, then the nearest level for every element
        __syncthreads();  // lv of the previous round has been read by everyone
        for (int c = tid; c < levels; c += ALT_THREADS) {
            double s = 0.0;
            for (int i = 0; i < q; ++i) s += ((c >> i) & 1) ? a[i] : -a[i];
            lv[c] = s;
        }
        __syncthreads();
        int changed = 0;
        for (int k = tid; k < n; k += ALT_THREADS) {
            const double x = (double)w[k];
            int best = levels - 1;
            double bl = lv[best], bd = fabs(x - bl);
            for (int c = levels - 2; c >= 0; --c) {
                const double l = lv[c], d = fabs(x - l);
                if (d < bd || (d == bd && l > bl)) {
                    best = c;
                    bd = d;
                    bl = l;
                }
            }
            if ((uint8_t)best != code[k]) {
                code[k] = (uint8_t)best;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }
    __syncthreads();

    // ---- outputs: alpha[i][v], packed[i][v][n / 32], planes[i][v][n]
    const int nw = n / 32;
    if (tid < q) alpha[(int64_t)tid * V + v] = (float)a[tid];
    for (int i = 0; i < q; ++i) {
        for (int wq = tid; wq < nw; wq += ALT_THREADS) {
            uint32_t word = 0u;
#pragma unroll 8
            for (int j = 0; j < 32; ++j) word |= (uint32_t)((code[32 * wq + j] >> i) & 1) << j;
            packed[((int64_t)i * V + v) * nw + wq] = word;
        }
        if (planes)
            for (int k = tid; k < n; k += ALT_THREADS)
                planes[((int64_t)i * V + v) * n + k] = ((code[k] >> i) & 1) ? (int8_t)1 : (int8_t)-1;
    }
}

__global__ void alt_zero_word_kernel(int* p) { *p = 0; }

hipError_t launch_quantize_alternating(const float* W, int64_t V, int64_t n, int q, int iters, float* alpha,
                                       uint32_t* packed, int8_t* planes, int* status_word, hipStream_t st) {
    if (status_word) {
        BCQ_LAUNCH(alt_zero_word_kernel, dim3(1), dim3(1), 0, st, status_word);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const size_t lds = (size_t)(4 * ALT_NRED + 256) * sizeof(double) + (size_t)n * 5;
    static LdsLimit limit;
    hipError_t ea = limit.ensure((const void*)alternating_kernel, lds);
    if (ea != hipSuccess) return ea;
    BCQ_LAUNCH(alternating_kernel, dim3((unsigned)V), dim3(ALT_THREADS), lds, st, W, V, (int)n, q, iters, alpha,
                       packed, planes, status_word);
    return hipGetLastError();
}

}  // namespace bcq
