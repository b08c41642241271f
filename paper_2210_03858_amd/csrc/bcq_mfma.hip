// Large-token path of the BCQ linear layer on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// AlphaTuning Eq. 2 / Eq. 3 are one dense contraction each once the q planes of a weight are summed:
//     y  = X  * What^T   (contraction over K),      dX = dY * What   (contraction over N),
// with What[n][k] = sum_i alpha_i[n] B_i[n][k] (Eq. 1).  Summing the planes BEFORE the contraction executes
// 2 T N K matrix-core flops instead of the 2 q T N K of a plane-by-plane product.
//
// Two kernels per call:
//   1. expand_*: reads the packed sign planes and alpha and writes What (or What^T) as bf16 into the caller's
//      workspace, already in the register order of the MFMA B operand ("fragment order"): for every tile of
//      32 output columns and every 16-long slice of the contraction, 64 lanes x 8 bf16 = 1 KiB contiguous.
//      This scratch is transient per call; persistent storage stays q bits per weight.
//   2. gemm_kernel: 256 x 256 output tile per workgroup, 4 waves in a 2 x 2 grid, each wave 128 x 128 =
//      4 x 4 MFMA tiles of v_mfma_f32_32x32x16_bf16.  The activation tile goes global -> registers -> LDS
//      (double buffered, rows padded by 16 B so that the 16-byte fragment reads are bank-conflict free); the
//      weight fragments are loaded straight from the workspace into registers (1 KiB coalesced per wave
//      load), so LDS carries only the activations.
#include "bcq_internal.h"

namespace bcq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROWB = BK * 2 + 16;         // bytes per LDS row of the activation tile (padded)
constexpr int STAGE = BM * ROWB;          // bytes per LDS stage

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---------------------------------------------------------------------------------------------------------
// expand for the forward: columns of the GEMM = rows n of W, contraction = k.
// thread = (c = n % 32, one group of up to 4 packed words); writes up to 16 fragment slots of 16 B.
__global__ __launch_bounds__(256) void expand_fwd_kernel(const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ alpha, int64_t N, int64_t K,
                                                         int q, int64_t R16 /* padded K / 16 */,
                                                         uint4* __restrict__ frag) {
    const int c = threadIdx.x & 31;
    const int64_t ct = blockIdx.x;
    const int64_t n = ct * 32 + c;
    const int64_t Kw = K / 32;
    const int64_t wq = (int64_t)blockIdx.y * 8 + (threadIdx.x >> 5);  // group of 4 words
    const int64_t Rw = R16 / 2;                                         // padded length in words
    if (wq * 4 >= Rw) return;
    float a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = (i < q && n < N) ? alpha[(int64_t)i * N + n] : 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
        const int64_t w = wq * 4 + ww;
        if (w >= Rw) break;
        uint32_t bits[8];
        const bool live = (n < N) && (w < Kw);
#pragma unroll
        for (int i = 0; i < 8; ++i) bits[i] = (i < q && live) ? packed[((int64_t)i * N + n) * Kw + w] : 0u;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {  // 8 columns of the word per fragment slot
            uint32_t out[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                float v[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int j = gg * 8 + p * 2 + e;
                    float s = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (i < q) s += ((bits[i] >> j) & 1u) ? a[i] : -a[i];
                    v[e] = live ? s : 0.f;
                }
                out[p] = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
            }
            const int64_t ks = w * 2 + (gg >> 1);
            const int lane = c + 32 * (gg & 1);
            frag[(ct * R16 + ks) * 64 + lane] = make_uint4(out[0], out[1], out[2], out[3]);
        }
    }
}

// expand for the input gradient: columns of the GEMM = columns k of W, contraction = n (transposed use of
// the canonical words: the 32 lanes of a column tile share one word and each takes its own bit).
__global__ __launch_bounds__(256) void expand_bwd_kernel(const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ alpha, int64_t N, int64_t K,
                                                         int q, int64_t R16 /* padded N / 16 */,
                                                         uint4* __restrict__ frag) {
    const int c = threadIdx.x & 31;
    const int64_t ct = blockIdx.x;  // K / 32 column tiles, exactly one packed word wide
    const int64_t Kw = K / 32;
    const int64_t slot = (int64_t)blockIdx.y * 8 + (threadIdx.x >> 5);  // = ks * 2 + g
    if (slot >= R16 * 2) return;
    const int64_t ks = slot >> 1;
    const int g = (int)(slot & 1);
    uint32_t out[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int64_t n = ks * 16 + g * 8 + p * 2 + e;
            float s = 0.f;
            if (n < N) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i < q) {
                        const float a = alpha[(int64_t)i * N + n];
                        const uint32_t b = packed[((int64_t)i * N + n) * Kw + ct];
                        s += ((b >> c) & 1u) ? a : -a;
                    }
                }
            }
            v[e] = s;
        }
        out[p] = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    }
    frag[(ct * R16 + ks) * 64 + c + 32 * g] = make_uint4(out[0], out[1], out[2], out[3]);
}

// ---------------------------------------------------------------------------------------------------------
// C[M][NC] = A[M][R] * Bfrag, A row-major bf16 with leading dimension lda, Bfrag in fragment order with R16
// slices per column tile (R16 * 16 >= R, a multiple of BK), C row-major bf16 with leading dimension ldc.
__global__ __launch_bounds__(256, 1) void gemm_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                      const uint4* __restrict__ Bfrag, bf16_t* __restrict__ C,
                                                      int64_t ldc, int64_t M, int64_t NC, int64_t R, int64_t R16,
                                                      int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroup -> tile: consecutive workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous
    // run of tiles that share weight columns so that its L2 sees every weight fragment once
    const int total = tiles_m * tiles_n;
    int bid = blockIdx.x;
    const int per_xcd = total / 8;
    int lid = (bid < per_xcd * 8) ? (bid % 8) * per_xcd + bid / 8 : bid;
    const int tile_n = lid / tiles_m, tile_m = lid % tiles_m;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t ct_count = (NC + 31) / 32;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // activation tile: 256 rows x 8 chunks of 16 B; thread handles chunk c of rows r0 + 32 * j
    const int lc = tid & 7, lr = tid >> 3;
    uint4 areg[8];
    auto load_a = [&](int64_t k0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t row = m0 + lr + 32 * j;
            const int64_t k = k0 + lc * 8;
            areg[j] = (row < M && k < R) ? *reinterpret_cast<const uint4*>(A + row * lda + k) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            *reinterpret_cast<uint4*>(smem + buf * STAGE + (lr + 32 * j) * ROWB + lc * 16) = areg[j];
    };

    // weight fragments of this wave: column tiles ct0 .. ct0+3
    const int64_t ct0 = (n0 + wn * 128) / 32;
    uint4 breg[4][4];  // [kk][j]
    auto load_b = [&](int64_t k0) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t ct = ct0 + j;
                breg[kk][j] = (ct < ct_count) ? Bfrag[(ct * R16 + (k0 / 16 + kk)) * 64 + lane] : make_uint4(0, 0, 0, 0);
            }
    };

    const int64_t steps = R16 * 16 / BK;
    load_a(0);
    load_b(0);
    store_a(0);
    __syncthreads();

    for (int64_t s = 0; s < steps; ++s) {
        const int buf = (int)(s & 1);
        uint4 bcur[4][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int j = 0; j < 4; ++j) bcur[kk][j] = breg[kk][j];
        if (s + 1 < steps) {
            load_a((s + 1) * BK);
            load_b((s + 1) * BK);
        }
        const unsigned char* sa = smem + buf * STAGE + (wm * 128 + (lane & 31)) * ROWB + (lane >> 5) * 16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * ROWB + kk * 32);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], as_bf16x8(bcur[kk][j]), acc[i][j], 0, 0, 0);
        }
        if (s + 1 < steps) store_a(buf ^ 1);
        __syncthreads();
    }

    // epilogue: acc register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its 32 x 32 tile
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = n0 + wn * 128 + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M && col < NC) C[row * ldc + col] = f32_to_bf16(acc[i][j][v]);
            }
        }
}

static inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

size_t mfma_fwd_workspace(int64_t N, int64_t K) { return (size_t)(round_up(N, 32) * round_up(K, BK) * 2); }
size_t mfma_bwd_input_workspace(int64_t N, int64_t K) { return (size_t)(round_up(K, 32) * round_up(N, BK) * 2); }

static hipError_t launch_gemm(const bf16_t* A, int64_t lda, const uint4* frag, bf16_t* C, int64_t ldc, int64_t M,
                              int64_t NC, int64_t R, int64_t R16, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           2 * STAGE);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((NC + BN - 1) / BN);
    hipLaunchKernelGGL(gemm_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 2 * STAGE, st, A, lda, frag, C,
                       ldc, M, NC, R, R16, tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_fwd_mfma(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                           int64_t K, int q, void* y, void* workspace, hipStream_t st) {
    const int64_t R16 = round_up(K, BK) / 16;
    const int64_t ct = (N + 31) / 32;
    dim3 grid((unsigned)ct, (unsigned)((R16 / 2 + 31) / 32));
    hipLaunchKernelGGL(expand_fwd_kernel, grid, dim3(256), 0, st, packed, alpha, N, K, q, R16, (uint4*)workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gemm((const bf16_t*)x, K, (const uint4*)workspace, (bf16_t*)y, N, T, N, K, R16, st);
}

hipError_t launch_bwd_input_mfma(const uint32_t* packed, const float* alpha, const void* dy, int64_t T, int64_t N,
                                 int64_t K, int q, void* dx, void* workspace, hipStream_t st) {
    const int64_t R16 = round_up(N, BK) / 16;
    dim3 grid((unsigned)(K / 32), (unsigned)((R16 * 2 + 7) / 8));
    hipLaunchKernelGGL(expand_bwd_kernel, grid, dim3(256), 0, st, packed, alpha, N, K, q, R16, (uint4*)workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gemm((const bf16_t*)dy, N, (const uint4*)workspace, (bf16_t*)dx, K, T, K, N, R16, st);
}

}  // namespace bcq
