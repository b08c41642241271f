// Small-token path (up to 16 tokens per pass, bf16): streams the packed sign planes from HBM exactly once and
// feeds them to the matrix cores plane by plane, as AlphaTuning Eq. 2 is written:
//     y[t][n]      = sum_i alpha_i[n] * C_i[n][t]           C_i[n][t] = sum_k B_i[n][k] x[t][k]      (Eq. 2)
//     dalpha_i[n]  = s * sum_t dy[t][n] * C_i[n][t]                                                    (Eq. 4)
//     dx[t][k]     = sum_i sum_n B_i[n][k] * (alpha_i[n] dy[t][n])                                     (Eq. 3)
// In this regime the work per weight BIT is what matters (the planes are the only large operand), so nothing
// is dequantised: a lane turns 8 sign bits into 8 bf16 values of +-1 with 8 vector-ALU operations (one shift
// and one three-input bit operation per register pair) and v_mfma_f32_16x16x32_bf16 multiplies them with a
// 32 x 16 slice of the activations (tokens padded to 16 in registers only).
//
// Work split: a workgroup owns 16 R rows of the plane matrix and all tokens of one 16-token tile; its W waves
// split the contraction range and add their partial 16 x 16 tiles through LDS in a fixed order (deterministic).
// Each lane reads its own 8 bytes of every plane row per 256-column segment, so a plane word is fetched by
// exactly one lane of one wave.  The contraction index is permuted inside the MFMA (lane group g owns columns
// 64 g .. 64 g + 63 of the segment, and a register pair holds columns c and c + 16 of a word) - legal because
// both operands use the same permutation - which is what makes the one-shift expansion possible.
//
// The input gradient uses the transposed twin (rows = columns k of W, bits along n) and activations
// pre-multiplied per plane, dy * alpha_i, rounded to bf16 by a small pre-kernel into the workspace.
#include "bcq_internal.h"

namespace bcq {

typedef __attribute__((ext_vector_type(8))) __bf16 s_bf16x8;
typedef __attribute__((ext_vector_type(4))) float s_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t s_u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t s_u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 s_bf16x2;
typedef __attribute__((ext_vector_type(2))) float s_f32x2;

enum { SMALL_FWD = 0, SMALL_DALPHA = 1, SMALL_DX = 2 };

__device__ __forceinline__ uint32_t s_pack_bf16x2(float lo, float hi) {
    s_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, s_bf16x2));
}

// 8 signs of one packed word -> MFMA operand: register p holds columns c = 4u + p (low half) and c + 16 (high).
__device__ __forceinline__ s_bf16x8 expand_signs(uint32_t word, int u) {
    s_u32x4 r;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int c = 4 * u + p;
        r[p] = ((word << (15 - c)) & 0x80008000u) ^ 0xBF80BF80u;  // bit 1 -> +1.0, bit 0 -> -1.0
    }
    return __builtin_bit_cast(s_bf16x8, r);
}

// Activation fragment matching expand_signs: columns (4u+p, 4u+p+16) of the 32-column word starting at `p32`.
__device__ __forceinline__ s_bf16x8 load_act_frag(const bf16_t* p32, int u, bool live) {
    s_u32x4 r = {0u, 0u, 0u, 0u};
    if (live) {
        const s_u32x2 lo = *reinterpret_cast<const s_u32x2*>(p32 + 4 * u);
        const s_u32x2 hi = *reinterpret_cast<const s_u32x2*>(p32 + 16 + 4 * u);
        r[0] = __builtin_amdgcn_perm(hi[0], lo[0], 0x05040100u);
        r[1] = __builtin_amdgcn_perm(hi[0], lo[0], 0x07060302u);
        r[2] = __builtin_amdgcn_perm(hi[1], lo[1], 0x05040100u);
        r[3] = __builtin_amdgcn_perm(hi[1], lo[1], 0x07060302u);
    }
    return __builtin_bit_cast(s_bf16x8, r);
}

// planes: [q][rows][cw] words (canonical for FWD / DALPHA, twin for DX).  act: FWD, DALPHA: x[T][C];
// DX: scaled activations [q][T][C].  rows x C is the plane matrix seen by this kernel (C = 32 cw).
template <int MODE, int R>
__global__ __launch_bounds__(R == 2 ? 256 : 1024) void small_kernel(const uint32_t* __restrict__ planes, const bf16_t* __restrict__ act,
                                                     const float* __restrict__ alpha, const bf16_t* __restrict__ dy,
                                                     void* __restrict__ out, int64_t T, int64_t rows, int64_t cw,
                                                     int q, int q_used, float scale, int segs_per_wave) {
    extern __shared__ __attribute__((aligned(16))) float red[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int rl = lane & 15, g = lane >> 4;                 // row (or token) within the tile, contraction group
    const int64_t row0 = (int64_t)blockIdx.x * 16 * R;
    const int64_t t0 = (int64_t)blockIdx.y * 16;
    const int64_t C = cw * 32;
    const bool tok_live = (t0 + rl) < T;
    const int64_t tok = tok_live ? t0 + rl : T - 1;
    constexpr int NACC = (MODE == SMALL_DX) ? 1 : 8;

    s_f32x4 acc[R][NACC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[r][i] = s_f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's plane rows (clamped: rows beyond the matrix produce outputs that are never stored)
    const uint32_t* prow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t rr = row0 + 16 * r + rl;
        rr = rr < rows ? rr : rows - 1;
        prow[r] = planes + rr * cw;
    }
    const int64_t plane_stride = rows * cw;

    const int seg_begin = wave * segs_per_wave;
    for (int s = 0; s < segs_per_wave; ++s) {
        const int64_t w0 = ((int64_t)(seg_begin + s) * 8) + 2 * g;  // first of this lane's two words
        if ((int64_t)(seg_begin + s) * 8 >= cw) break;               // whole wave leaves together
        const bool w_live0 = w0 < cw, w_live1 = (w0 + 1) < cw;
        const int64_t wc0 = w_live0 ? w0 : cw - 1, wc1 = w_live1 ? w0 + 1 : cw - 1;
        uint32_t bits[R][8][2];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < q_used) {
                    bits[r][i][0] = prow[r][(int64_t)i * plane_stride + wc0];
                    bits[r][i][1] = prow[r][(int64_t)i * plane_stride + wc1];
                }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bool live = tok_live && (j == 0 ? w_live0 : w_live1);
            const int64_t col = (j == 0 ? wc0 : wc1) * 32;
#pragma unroll 1
            for (int u = 0; u < 4; ++u) {
                if (MODE == SMALL_DX) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (i < q_used) {
                            const s_bf16x8 v = load_act_frag(act + ((int64_t)i * T + tok) * C + col, u, live);
#pragma unroll
                            for (int r = 0; r < R; ++r)
                                acc[r][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(expand_signs(bits[r][i][j], u), v,
                                                                                    acc[r][0], 0, 0, 0);
                        }
                } else {
                    const s_bf16x8 v = load_act_frag(act + tok * C + col, u, live);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (i < q_used)
                                acc[r][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(expand_signs(bits[r][i][j], u), v,
                                                                                    acc[r][i], 0, 0, 0);
                }
            }
        }
    }

    // Accumulator register v of lane l: plane-matrix row 4 * (l / 16) + v of the tile, token l % 16.
    // FWD folds alpha into one tile per row block before the cross-wave sum; DALPHA keeps the planes apart.
    constexpr int NOUT = (MODE == SMALL_DALPHA) ? 8 : 1;
    const int nout = (MODE == SMALL_DALPHA) ? q_used : 1;
    s_f32x4 part[R][NOUT];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (MODE == SMALL_FWD) {
            s_f32x4 y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < q_used) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        int64_t n = row0 + 16 * r + 4 * g + v;
                        n = n < rows ? n : rows - 1;
                        y[v] += alpha[(int64_t)i * rows + n] * acc[r][i][v];
                    }
                }
            part[r][0] = y;
        } else if (MODE == SMALL_DX) {
            part[r][0] = acc[r][0];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) part[r][i < NOUT ? i : 0] = acc[r][i < NACC ? i : 0];
        }
    }
    // cross-wave sum in wave order: red[w][r][o][lane][4]
    if (W > 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) *reinterpret_cast<s_f32x4*>(&red[(((wave * R + r) * nout + o) * 64 + lane) * 4]) = part[r][o];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) {
                    s_f32x4 s = part[r][o];
                    for (int w = 1; w < W; ++w) s += *reinterpret_cast<const s_f32x4*>(&red[(((w * R + r) * nout + o) * 64 + lane) * 4]);
                    part[r][o] = s;
                }
    }

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t n = row0 + 16 * r + 4 * g;  // first of this lane's 4 rows
        if (MODE == SMALL_DALPHA) {
            float d[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) d[v] = (tok_live && n + v < rows) ? bf16_to_f32(dy[tok * rows + n + v]) : 0.f;
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) {
                    s_f32x4 s;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float x = d[v] * part[r][o][v];
                        x += __shfl_xor(x, 1);
                        x += __shfl_xor(x, 2);
                        x += __shfl_xor(x, 4);
                        x += __shfl_xor(x, 8);
                        s[v] = x * scale;
                    }
                    // token tiles beyond the first accumulate in a later pass; this kernel is launched with one
                    if (rl == 0)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (n + v < rows) reinterpret_cast<float*>(out)[(int64_t)o * rows + n + v] = s[v];
                }
        } else {
            bf16_t* o = reinterpret_cast<bf16_t*>(out);
            if (tok_live) {
                if (n + 3 < rows && (rows & 3) == 0) {
                    s_u32x2 pk;
                    pk[0] = s_pack_bf16x2(part[r][0][0], part[r][0][1]);
                    pk[1] = s_pack_bf16x2(part[r][0][2], part[r][0][3]);
                    *reinterpret_cast<s_u32x2*>(o + tok * rows + n) = pk;
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (n + v < rows) o[tok * rows + n + v] = f32_to_bf16(part[r][0][v]);
                }
            }
        }
    }
}

// dys[i][t][n] = bf16(dy[t][n] * alpha_i[n])
__global__ __launch_bounds__(256) void scale_dy_kernel(const bf16_t* __restrict__ dy, const float* __restrict__ alpha,
                                                       bf16_t* __restrict__ dys, int64_t T, int64_t N, int q) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= T * N) return;
    const int64_t n = idx % N;
    const float d = bf16_to_f32(dy[idx]);
    for (int i = 0; i < q; ++i) dys[(int64_t)i * T * N + idx] = f32_to_bf16(d * alpha[(int64_t)i * N + n]);
}

struct SmallPlan {
    int R, W, segs_per_wave;
    unsigned grid_x;
};

static SmallPlan small_plan(int64_t rows, int64_t cw) {
    SmallPlan p;
    const int64_t segs = (cw + 7) / 8;
    // enough waves for the 1024 SIMDs of the chip: prefer two row tiles per wave, split the contraction more
    // (up to 16 waves per workgroup) when the matrix has few rows
    p.R = (rows / 32) * 4 >= 2048 ? 2 : 1;
    const int64_t blocks = (rows + 16 * p.R - 1) / (16 * p.R);
    int W = 4;
    while (W < 16 && blocks * W < 2048 && segs >= 2 * W) W *= 2;
    if (W > segs) W = (int)(segs < 1 ? 1 : segs);
    p.W = W;
    p.segs_per_wave = (int)((segs + W - 1) / W);
    p.grid_x = (unsigned)blocks;
    return p;
}

template <int MODE>
static hipError_t launch_small(const uint32_t* planes, const bf16_t* act, const float* alpha, const bf16_t* dy,
                               void* out, int64_t T, int64_t rows, int64_t cw, int q, int q_used, float scale,
                               hipStream_t st) {
    const SmallPlan p = small_plan(rows, cw);
    const dim3 grid(p.grid_x, (unsigned)((T + 15) / 16));
    const dim3 block((unsigned)(64 * p.W));
    const int nout = (MODE == SMALL_DALPHA) ? q_used : 1;
    const size_t lds = (size_t)p.W * p.R * nout * 64 * 4 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {  // up to 16 waves x 8 planes x 1 KiB of partial tiles
        hipError_t e = hipFuncSetAttribute((const void*)small_kernel<MODE, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void*)small_kernel<MODE, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (p.R == 2)
        hipLaunchKernelGGL((small_kernel<MODE, 2>), grid, block, lds, st, planes, act, alpha, dy, out, T, rows, cw, q,
                           q_used, scale, p.segs_per_wave);
    else
        hipLaunchKernelGGL((small_kernel<MODE, 1>), grid, block, lds, st, planes, act, alpha, dy, out, T, rows, cw, q,
                           q_used, scale, p.segs_per_wave);
    return hipGetLastError();
}

size_t small_bwd_input_workspace(int64_t T, int64_t N, int q) { return (size_t)q * T * N * 2; }

hipError_t launch_fwd_small(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                            int64_t K, int q, void* y, hipStream_t st) {
    return launch_small<SMALL_FWD>(packed, (const bf16_t*)x, alpha, nullptr, y, T, N, K / 32, q, q, 1.f, st);
}

hipError_t launch_bwd_alpha_small(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                  int64_t K, int q, int q_train, float grad_scale, float* dalpha, hipStream_t st) {
    return launch_small<SMALL_DALPHA>(packed, (const bf16_t*)x, nullptr, (const bf16_t*)dy, dalpha, T, N, K / 32, q,
                                      q_train, grad_scale, st);
}

hipError_t launch_bwd_input_small(const uint32_t* packed_t, const float* alpha, const void* dy, int64_t T, int64_t N,
                                  int64_t K, int q, void* dx, void* workspace, hipStream_t st) {
    const int64_t total = T * N;
    hipLaunchKernelGGL(scale_dy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t*)dy,
                       alpha, (bf16_t*)workspace, T, N, q);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_small<SMALL_DX>(packed_t, (const bf16_t*)workspace, nullptr, nullptr, dx, T, K, N / 32, q, q, 1.f, st);
}

}  // namespace bcq
