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

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// two fp32 -> two bf16 (round to nearest even) in one v_cvt_pk_bf16_f32; `lo` lands in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---------------------------------------------------------------------------------------------------------
// expand for the forward: columns of the GEMM = rows n of W, contraction = k.
// thread = (c = n % 32, 8 consecutive k of one packed word) -> one 16-byte fragment slot.
__global__ __launch_bounds__(256) void expand_fwd_kernel(const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ alpha, int64_t N, int64_t K,
                                                         int q, int64_t R16 /* padded K / 16 */,
                                                         uint4* __restrict__ frag) {
    const int c = threadIdx.x & 31;
    const int64_t ct = blockIdx.x;
    const int64_t n = ct * 32 + c;
    const int64_t Kw = K / 32;
    const int64_t slot = (int64_t)blockIdx.y * 8 + (threadIdx.x >> 5);  // = ks * 2 + g, 8 columns each
    if (slot >= R16 * 2) return;
    const int64_t w = slot >> 2;
    const int sh = (int)(slot & 3) * 8;
    const bool live = (n < N) && (w < Kw);
    float a[8];
    uint32_t bits[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (i < q && live) ? alpha[(int64_t)i * N + n] : 0.f;
        bits[i] = (i < q && live) ? (packed[((int64_t)i * N + n) * Kw + w] >> sh) : 0u;
    }
    uint32_t out[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int j = p * 2 + e;
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < q) s += ((bits[i] >> j) & 1u) ? a[i] : -a[i];
            v[e] = s;
        }
        out[p] = pack_bf16x2(v[0], v[1]);
    }
    frag[(ct * R16 + (slot >> 1)) * 64 + c + 32 * (int)(slot & 1)] = make_uint4(out[0], out[1], out[2], out[3]);
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
        out[p] = pack_bf16x2(v[0], v[1]);
    }
    frag[(ct * R16 + ks) * 64 + c + 32 * g] = make_uint4(out[0], out[1], out[2], out[3]);
}

// ---------------------------------------------------------------------------------------------------------
// C[M][NC] = A[M][R] * Bfrag, A row-major bf16 with leading dimension lda, Bfrag in fragment order with R16
// slices per column tile (R16 * 16 >= R, a multiple of BK), C row-major bf16 with leading dimension ldc.
// Workgroup tile (64 TM) x (64 TN), 4 waves in a 2 x 2 grid, each wave TM x TN MFMA tiles.
// The weight fragment is the first MFMA operand, so one lane ends up with 4 consecutive output columns of
// one token.  Out-of-range rows, chunks and column tiles are clamped to valid addresses instead of branching:
// their products land in outputs that are never stored, or meet zero weights.
template <int TM, int TN>
struct GemmCfg {
    static constexpr int BMT = 64 * TM, BNT = 64 * TN;
    static constexpr int STAGE_B = BMT * ROWB;                 // one activation stage
    static constexpr int EPI_ROWB = 64 * TN + 8;               // epilogue row: 32 TN columns of bf16 + pad
    static constexpr int EPI_B = 4 * 64 * EPI_ROWB;            // 4 waves x 64 tokens
    static constexpr int LDS_B = (2 * STAGE_B > EPI_B) ? 2 * STAGE_B : EPI_B;
    static constexpr int OCC = (TM * TN >= 16) ? 1 : 2;
};

template <int TM, int TN>
__global__ __launch_bounds__(256, (TM * TN >= 16 ? 1 : 2)) void gemm_kernel(
    const bf16_t* __restrict__ A, int64_t lda, const u32x4* __restrict__ Bfrag, bf16_t* __restrict__ C, int64_t ldc,
    int64_t M, int64_t NC, int64_t R, int64_t R16, int tiles_m, int tiles_n) {
    using Cfg = GemmCfg<TM, TN>;
    constexpr int STAGE_B = Cfg::STAGE_B;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroup -> tile: consecutive workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous
    // run of tiles that share weight columns so that its L2 sees every weight fragment once
    const int total = tiles_m * tiles_n;
    const int bid = blockIdx.x;
    const int per_xcd = total / 8;
    const int lid = (bid < per_xcd * 8) ? (bid % 8) * per_xcd + bid / 8 : bid;
    const int tile_n = lid / tiles_m, tile_m = lid % tiles_m;
    const int64_t m0 = (int64_t)tile_m * Cfg::BMT, n0 = (int64_t)tile_n * Cfg::BNT;
    const int64_t ct_count = (NC + 31) / 32;

    f32x16 acc[TN][TM];  // [weight tile][token tile]
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // activation tile: 64 TM rows x 8 chunks of 16 B; thread handles chunk lc of rows lr + 32 * j
    constexpr int NA = 2 * TM;
    const int lc = tid & 7, lr = tid >> 3;
    const bf16_t* arow[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int64_t row = m0 + lr + 32 * j;
        row = row < M ? row : M - 1;
        arow[j] = A + row * lda;
    }
    const int64_t kmax = R - 8;
    u32x4 areg[NA];
    auto load_a = [&](int64_t k0) {
#ifdef BCQ_PROBE_NO_A
        if (k0 > 0) return;
#endif
        int64_t k = k0 + lc * 8;
        k = k < kmax ? k : kmax;
#pragma unroll
        for (int j = 0; j < NA; ++j) areg[j] = *reinterpret_cast<const u32x4*>(arow[j] + k);
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NA; ++j)
            *reinterpret_cast<u32x4*>(smem + buf * STAGE_B + (lr + 32 * j) * ROWB + lc * 16) = areg[j];
    };

    // weight fragments of this wave: column tiles ct0 .. ct0+TN-1
    const int64_t ct0 = (n0 + wn * 32 * TN) / 32;
    const u32x4* bptr[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int64_t ct = ct0 + j;
        ct = ct < ct_count ? ct : ct_count - 1;
        bptr[j] = Bfrag + ct * R16 * 64 + lane;
    }
    u32x4 b[4][TN];  // [kk][j]; slot kk is refilled for the next K-step right after its MFMAs are issued
    auto load_b = [&](int kk, int64_t step) {
#ifdef BCQ_PROBE_NO_B
        if (step > 0) return;
#endif
#pragma unroll
        for (int j = 0; j < TN; ++j) b[kk][j] = bptr[j][(step * 4 + kk) * 64];
    };
    bf16x8 xf[2][TM];  // activation fragments of two consecutive 16-slices
    auto read_x = [&](int buf, int kk) {
        const unsigned char* sa =
            smem + buf * STAGE_B + (wm * 32 * TM + (lane & 31)) * ROWB + (lane >> 5) * 16 + kk * 32;
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[kk & 1][i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * ROWB);
    };
    auto compute = [&](int buf, int64_t next_step) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) read_x(buf, kk + 1);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(b[kk][j]), xf[kk & 1][i], acc[j][i],
                                                                        0, 0, 0);
            load_b(kk, next_step);
            // issue order inside the slice: LDS reads of the next slice, the MFMAs, then the weight refill
            if (kk < 3) __builtin_amdgcn_sched_group_barrier(0x100, TM, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, TN, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int64_t steps = R16 * 16 / BK;
    const int64_t last = steps - 1;
    load_a(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) load_b(kk, 0);
    store_a(0);
    __syncthreads();
    read_x(0, 0);

    for (int64_t s = 0; s < steps; ++s) {
        const int buf = (int)(s & 1);
        const int64_t nx = s < last ? s + 1 : last;
        load_a(nx * BK);
        __builtin_amdgcn_sched_barrier(0);
        compute(buf, nx);
        store_a(buf ^ 1);
        __syncthreads();
        read_x(buf ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: acc register 4g+e of lane l is weight column 8g + 4*(l/32) + e, token l%32 of its 32 x 32 tile.
    // Pass the tile through LDS (64 tokens per wave at a time) so that global stores are 16 B per lane and
    // whole rows of 64 TN bytes are contiguous.
    constexpr int EROW = Cfg::EPI_ROWB;
#ifdef BCQ_PROBE_NO_STORE
    if (acc[0][0][0] != 123.456f) return;
#endif
    const bool vec_ok = (ldc % 8 == 0);
    if (vec_ok) {
        unsigned char* ew = smem + wave * 64 * EROW;
        constexpr int CH = 4 * TN;        // 16-byte chunks per row
        constexpr int RPI = 64 / CH;      // rows per store instruction
#pragma unroll
        for (int pass = 0; pass < (TM + 1) / 2; ++pass) {
            __syncthreads();
#pragma unroll
            for (int il = 0; il < 2; ++il) {
                const int it = pass * 2 + il;
                if (it < TM) {
#pragma unroll
                    for (int jw = 0; jw < TN; ++jw)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            uint2 o;
                            o.x = pack_bf16x2(acc[jw][it][4 * g], acc[jw][it][4 * g + 1]);
                            o.y = pack_bf16x2(acc[jw][it][4 * g + 2], acc[jw][it][4 * g + 3]);
                            *reinterpret_cast<uint2*>(ew + (il * 32 + (lane & 31)) * EROW +
                                                      (jw * 32 + 8 * g + 4 * (lane >> 5)) * 2) = o;
                        }
                }
            }
            __syncthreads();
            const int rows_here = (TM - pass * 2 >= 2) ? 64 : 32;
            const int ch = lane % CH, r0 = lane / CH;
#pragma unroll
            for (int rr = 0; rr < 64 / RPI; ++rr) {
                const int r = rr * RPI + r0;
                if (r < rows_here) {
                    const int64_t t = m0 + wm * 32 * TM + pass * 64 + r;
                    const int64_t n = n0 + wn * 32 * TN + ch * 8;
                    if (t < M) {
                        const u32x4 vv = *reinterpret_cast<const u32x4*>(ew + r * EROW + ch * 16);
                        if (n + 7 < NC) {
                            *reinterpret_cast<u32x4*>(C + t * ldc + n) = vv;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (n + e < NC) C[t * ldc + n + e] = (bf16_t)((vv[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
                        }
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < TM; ++it) {
            const int64_t t = m0 + wm * 32 * TM + it * 32 + (lane & 31);
            if (t >= M) continue;
            bf16_t* crow = C + t * ldc;
#pragma unroll
            for (int jw = 0; jw < TN; ++jw)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int64_t n = n0 + wn * 32 * TN + jw * 32 + 8 * g + 4 * (lane >> 5);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < NC) crow[n + e] = f32_to_bf16(acc[jw][it][4 * g + e]);
                }
        }
    }
}

static inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

size_t mfma_fwd_workspace(int64_t N, int64_t K) { return (size_t)(round_up(N, 32) * round_up(K, BK) * 2); }
size_t mfma_bwd_input_workspace(int64_t N, int64_t K) { return (size_t)(round_up(K, 32) * round_up(N, BK) * 2); }

template <int TM, int TN>
static hipError_t launch_gemm_cfg(const bf16_t* A, int64_t lda, const u32x4* frag, bf16_t* C, int64_t ldc, int64_t M,
                                  int64_t NC, int64_t R, int64_t R16, hipStream_t st) {
    using Cfg = GemmCfg<TM, TN>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<TM, TN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_B);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_m = (int)((M + Cfg::BMT - 1) / Cfg::BMT), tiles_n = (int)((NC + Cfg::BNT - 1) / Cfg::BNT);
    hipLaunchKernelGGL((gemm_kernel<TM, TN>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), Cfg::LDS_B, st, A, lda,
                       frag, C, ldc, M, NC, R, R16, tiles_m, tiles_n);
    return hipGetLastError();
}

// Tile choice: the largest tile that still gives every compute unit (256) a workgroup.
static hipError_t launch_gemm(const bf16_t* A, int64_t lda, const u32x4* frag, bf16_t* C, int64_t ldc, int64_t M,
                              int64_t NC, int64_t R, int64_t R16, hipStream_t st) {
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((NC + bn - 1) / bn); };
    if (tiles(256, 256) >= 192) return launch_gemm_cfg<4, 4>(A, lda, frag, C, ldc, M, NC, R, R16, st);
    if (tiles(256, 128) >= 192) return launch_gemm_cfg<4, 2>(A, lda, frag, C, ldc, M, NC, R, R16, st);
    return launch_gemm_cfg<2, 2>(A, lda, frag, C, ldc, M, NC, R, R16, st);
}

hipError_t launch_fwd_mfma(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                           int64_t K, int q, void* y, void* workspace, hipStream_t st) {
    const int64_t R16 = round_up(K, BK) / 16;
    const int64_t ct = (N + 31) / 32;
    dim3 grid((unsigned)ct, (unsigned)((R16 * 2 + 7) / 8));
    hipLaunchKernelGGL(expand_fwd_kernel, grid, dim3(256), 0, st, packed, alpha, N, K, q, R16, (uint4*)workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gemm((const bf16_t*)x, K, (const u32x4*)workspace, (bf16_t*)y, N, T, N, K, R16, st);
}

hipError_t launch_bwd_input_mfma(const uint32_t* packed, const float* alpha, const void* dy, int64_t T, int64_t N,
                                 int64_t K, int q, void* dx, void* workspace, hipStream_t st) {
    const int64_t R16 = round_up(N, BK) / 16;
    dim3 grid((unsigned)(K / 32), (unsigned)((R16 * 2 + 7) / 8));
    hipLaunchKernelGGL(expand_bwd_kernel, grid, dim3(256), 0, st, packed, alpha, N, K, q, R16, (uint4*)workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gemm((const bf16_t*)dy, N, (const u32x4*)workspace, (bf16_t*)dx, K, T, K, N, R16, st);
}


// =========================================================================================================
// Scale gradient on the matrix cores.  AlphaTuning Eq. 4, read as the gradient of Eq. 2, is
//     dalpha_i[n] = s * sum_t dY[t][n] * (X B_i^T)[t][n] = s * sum_k B_i[n][k] * G[n][k],   G = dY^T X.
// G is one dense contraction over the tokens (2 T N K matrix-core flops for ALL planes together, instead of
// 2 q T N K for q plane products); the sign planes only enter a signed row sum of the accumulators.
//
// Workgroup: 256 (k) x 256 (n) tile of G^T for one slice of the tokens; 4 waves in a 2 x 2 grid, each
// 128 x 128 = 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 with X^T as first and dY^T as second operand, so a lane
// holds one n and 16 k of every tile.  Both operands need the token index innermost: each thread loads an
// 8 (tokens) x 8 (columns) block with eight 16-byte loads, transposes it in registers (32 v_perm) and writes
// eight 16-byte rows into an XOR-swizzled LDS tile [column][64 tokens]; writes and fragment reads are
// bank-conflict free.  Partial sums per (token slice, k tile) go to the workspace; a second kernel adds them
// in a fixed order (no floating-point atomics, bit-reproducible).
constexpr int DA_TILE = 256;               // k and n extent of a workgroup tile
constexpr int DA_STAGE = DA_TILE * 128;    // bytes per operand per LDS stage: 256 columns x 64 tokens x 2 B

__device__ __forceinline__ int da_swz(int col, int chunk) { return col * 128 + ((chunk ^ (col & 7) ^ ((col >> 3) & 7)) << 4); }

__global__ __launch_bounds__(256, 1) void dalpha_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ DY,
                                                        const uint32_t* __restrict__ packed,
                                                        float* __restrict__ part, int64_t T, int64_t N, int64_t K,
                                                        int q_train, int tiles_k, int tiles_n, int64_t tokens_per_split) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;  // wm: k half, wn: n half
    const int tile_k = blockIdx.x % tiles_k, tile_n = blockIdx.x / tiles_k;
    const int split = blockIdx.y;
    const int64_t k0 = (int64_t)tile_k * DA_TILE, n0 = (int64_t)tile_n * DA_TILE;
    const int64_t t_begin = (int64_t)split * tokens_per_split;
    const int64_t t_end = (t_begin + tokens_per_split < T) ? t_begin + tokens_per_split : T;
    const int64_t steps = (t_end - t_begin + 63) / 64;

    f32x16 acc[4][4];  // [k tile][n tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // global -> register blocks: thread = (cb = column block of 8, tb = token block of 8)
    const int cb = tid & 31, tb = tid >> 5;
    int64_t xcol = k0 + cb * 8, dcol = n0 + cb * 8;
    xcol = xcol < K - 8 ? xcol : K - 8;  // clamped columns only feed outputs that are never stored
    dcol = dcol < N - 8 ? dcol : N - 8;
    u32x4 xr[8], dr[8];
    auto load_blocks = [&](int64_t step) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t t = t_begin + step * 64 + tb * 8 + r;
            const int64_t tc = t < T ? t : T - 1;
            u32x4 xv = *reinterpret_cast<const u32x4*>(X + tc * K + xcol);
            const u32x4 zero = {0u, 0u, 0u, 0u};
            xr[r] = t < t_end ? xv : zero;  // tokens outside the slice contribute nothing
            dr[r] = *reinterpret_cast<const u32x4*>(DY + tc * N + dcol);
        }
    };
    // 8 x 8 transpose of 16-bit elements, then 8 row writes of 16 B
    auto store_blocks = [&](int buf) {
        unsigned char* sx = smem + buf * 2 * DA_STAGE;
        unsigned char* sd = sx + DA_STAGE;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            u32x4 ox, od;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                ox[w] = __builtin_amdgcn_perm(xr[2 * w + 1][c >> 1], xr[2 * w][c >> 1], sel);
                od[w] = __builtin_amdgcn_perm(dr[2 * w + 1][c >> 1], dr[2 * w][c >> 1], sel);
            }
            *reinterpret_cast<u32x4*>(sx + da_swz(cb * 8 + c, tb)) = ox;
            *reinterpret_cast<u32x4*>(sd + da_swz(cb * 8 + c, tb)) = od;
        }
    };
    bf16x8 xf[2][4], df[2][4];
    auto read_frags = [&](int buf, int kk) {
        const unsigned char* sx = smem + buf * 2 * DA_STAGE;
        const unsigned char* sd = sx + DA_STAGE;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xf[kk & 1][i] = *reinterpret_cast<const bf16x8*>(sx + da_swz(wm * 128 + i * 32 + (lane & 31), kk * 2 + (lane >> 5)));
            df[kk & 1][i] = *reinterpret_cast<const bf16x8*>(sd + da_swz(wn * 128 + i * 32 + (lane & 31), kk * 2 + (lane >> 5)));
        }
    };

    load_blocks(0);
    store_blocks(0);
    __syncthreads();
    read_frags(0, 0);
    for (int64_t s = 0; s < steps; ++s) {
        const int buf = (int)(s & 1);
        const int64_t nx = s + 1 < steps ? s + 1 : s;
        load_blocks(nx);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) read_frags(buf, kk + 1);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[kk & 1][i], df[kk & 1][j], acc[i][j], 0, 0, 0);
            if (kk < 3) __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < steps) store_blocks(buf ^ 1);
        __syncthreads();
        if (s + 1 < steps) read_frags(buf ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: signed sums over this wave's 128 k for each plane; lane owns n = n_base + j*32 + lane%32
    float* red = reinterpret_cast<float*>(smem);  // [plane][wm][256 n]; the loop above ended with a barrier
    const int64_t Kw = K / 32;
    for (int p = 0; p < q_train; ++p) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
            const int64_t nc = n < N ? n : N - 1;
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t kt = (k0 + wm * 128 + i * 32) / 32;
                if (kt < Kw) {
                    const uint32_t word = packed[((int64_t)p * N + nc) * Kw + kt] >> (4 * (lane >> 5));
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int bit = 8 * (v >> 2) + (v & 3);
                        s += ((word >> bit) & 1u) ? acc[i][j][v] : -acc[i][j][v];
                    }
                }
            }
            s += __shfl_xor(s, 32);
            if (lane < 32) red[(p * 2 + wm) * 256 + wn * 128 + j * 32 + lane] = s;
        }
    }
    __syncthreads();
    const int64_t part_id = (int64_t)split * tiles_k + tile_k;
    for (int p = 0; p < q_train; ++p) {
        const int64_t n = n0 + tid;
        if (n < N) part[(part_id * q_train + p) * N + n] = red[(p * 2 + 0) * 256 + tid] + red[(p * 2 + 1) * 256 + tid];
    }
}

__global__ __launch_bounds__(256) void dalpha_reduce_kernel(const float* __restrict__ part, float* __restrict__ dalpha,
                                                            int64_t count /* q_train * N */, int parts, float scale) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    float s = 0.f;
    for (int p = 0; p < parts; ++p) s += part[(int64_t)p * count + idx];
    dalpha[idx] = scale * s;
}

static void dalpha_plan(int64_t T, int64_t N, int64_t K, int* tiles_k, int* tiles_n, int* splits, int64_t* per_split) {
    *tiles_k = (int)((K + DA_TILE - 1) / DA_TILE);
    *tiles_n = (int)((N + DA_TILE - 1) / DA_TILE);
    const int64_t tiles = (int64_t)*tiles_k * *tiles_n;
    int64_t s = (512 + tiles - 1) / tiles;            // aim at two workgroups per compute unit
    const int64_t max_s = (T + 255) / 256;            // at least 256 tokens (4 steps) per slice
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    int64_t per = ((T + s - 1) / s + 63) / 64 * 64;
    *per_split = per;
    *splits = (int)((T + per - 1) / per);
}

size_t mfma_bwd_alpha_workspace(int64_t T, int64_t N, int64_t K, int q) {
    int tk, tn, sp;
    int64_t per;
    dalpha_plan(T, N, K, &tk, &tn, &sp, &per);
    return (size_t)sp * tk * q * N * sizeof(float);
}

hipError_t launch_bwd_alpha_mfma(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                 int64_t K, int q_train, float grad_scale, float* dalpha, void* workspace,
                                 hipStream_t st) {
    static bool attr_set = false;
    const int lds = 4 * DA_STAGE;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)dalpha_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int tk, tn, sp;
    int64_t per;
    dalpha_plan(T, N, K, &tk, &tn, &sp, &per);
    hipLaunchKernelGGL(dalpha_kernel, dim3((unsigned)(tk * tn), (unsigned)sp), dim3(256), lds, st, (const bf16_t*)x,
                       (const bf16_t*)dy, packed, (float*)workspace, T, N, K, q_train, tk, tn, per);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t count = (int64_t)q_train * N;
    hipLaunchKernelGGL(dalpha_reduce_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                       (const float*)workspace, dalpha, count, sp * tk, grad_scale);
    return hipGetLastError();
}

}  // namespace bcq
