// Small-token path without a workspace (up to 16 tokens per pass, bf16, forward and scale gradient): streams the
// packed sign planes from HBM exactly once and feeds them to the matrix cores plane by plane, as AlphaTuning
// Eq. 2 is written:
//     y[t][n]      = sum_i alpha_i[n] * C_i[n][t]           C_i[n][t] = sum_k B_i[n][k] x[t][k]      (Eq. 2)
//     dalpha_i[n]  = s * sum_t dy[t][n] * C_i[n][t]                                                    (Eq. 4)
// (With a workspace the library uses the FP4 x FP8 kernels of bcq_stream.hip instead, which also cover Eq. 3.)
// In this regime the work per weight BIT is what matters (the planes are the only large operand), so nothing
// is dequantised: a lane turns 8 sign bits into 8 bf16 values of +-1 with 8 vector-ALU operations (one shift
// and one three-input bit operation per register pair) and v_mfma_f32_16x16x32_bf16 multiplies them with a
// 32 x 16 slice of the activations (tokens padded to 16 in registers only).
//
// Work split: a workgroup owns 16 R rows of the plane matrix and all tokens of one 16-token tile; its W waves
// split the contraction range and add their partial 16 x 16 tiles through LDS in a fixed order (deterministic).
// Each lane reads its own 16 bytes of every plane row per 512-column segment (four lanes cover 64 contiguous
// bytes of a row), so a plane word is fetched by exactly one lane of one wave.  The contraction index is permuted inside the MFMA (lane group g owns columns
// 128 g .. 128 g + 127 of a 512-column segment, and a register pair holds columns c and c + 16 of a word) - legal because
// both operands use the same permutation - which is what makes the one-shift expansion possible.
#include "bcq_internal.h"

namespace bcq {

typedef __attribute__((ext_vector_type(8))) __bf16 s_bf16x8;
typedef __attribute__((ext_vector_type(4))) float s_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t s_u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t s_u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 s_bf16x2;
typedef __attribute__((ext_vector_type(2))) float s_f32x2;

enum { SMALL_FWD = 0, SMALL_DALPHA = 1 };

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

// planes: [q][rows][cw] words (canonical layout); act: x[T][C].  rows x C is the plane matrix (C = 32 cw).
template <int MODE, int R, int QP>
__global__ __launch_bounds__(512) void small_kernel(const uint32_t* __restrict__ planes, const bf16_t* __restrict__ act,
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
    constexpr int NACC = QP;  // planes beyond q_used read plane q_used-1 again and are dropped

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

    // epilogue operands, requested before the main loop so that their latency is covered by it
    float ep[R][QP][4];  // FWD: alpha_i of this lane's 4 rows; DALPHA: dy of this lane's token and 4 rows (plane 0 slot)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int64_t n = row0 + 16 * r + 4 * g + v;
            const bool n_live = n < rows;
            n = n_live ? n : rows - 1;
            if (MODE == SMALL_FWD) {
#pragma unroll
                for (int i = 0; i < QP; ++i) ep[r][i][v] = (i < q_used) ? alpha[(int64_t)i * rows + n] : 0.f;
            } else if (MODE == SMALL_DALPHA) {
                ep[r][0][v] = (tok_live && n_live) ? bf16_to_f32(dy[tok * rows + n]) : 0.f;
            }
        }

    // raw halves of an activation fragment (see load_act_frag), loaded early and permuted at use
    struct ActRaw { s_u32x2 lo, hi; };
    auto load_act_raw = [&](const bf16_t* p32, int u, bool live) {
        ActRaw a;
        a.lo = s_u32x2{0u, 0u};
        a.hi = s_u32x2{0u, 0u};
        if (live) {
            a.lo = *reinterpret_cast<const s_u32x2*>(p32 + 4 * u);
            a.hi = *reinterpret_cast<const s_u32x2*>(p32 + 16 + 4 * u);
        }
        return a;
    };
    auto act_frag = [&](const ActRaw& a) {
        s_u32x4 r;
        r[0] = __builtin_amdgcn_perm(a.hi[0], a.lo[0], 0x05040100u);
        r[1] = __builtin_amdgcn_perm(a.hi[0], a.lo[0], 0x07060302u);
        r[2] = __builtin_amdgcn_perm(a.hi[1], a.lo[1], 0x05040100u);
        r[3] = __builtin_amdgcn_perm(a.hi[1], a.lo[1], 0x07060302u);
        return __builtin_bit_cast(s_bf16x8, r);
    };

    const int seg_begin = wave * segs_per_wave;
    constexpr int PPP = QP;  // planes per pass
    {
        const bf16_t* act_row = act + tok * C;
        const uint32_t* pbase = planes;
        for (int s = 0; s < segs_per_wave; ++s) {
            if ((int64_t)(seg_begin + s) * 16 >= cw) break;                // whole wave leaves together
            const int64_t w0 = ((int64_t)(seg_begin + s) * 16) + 4 * g;  // first of this lane's four words
            // one 16-byte load per plane row when the four words exist (cw % 4 == 0 keeps it aligned)
            const bool quad = (w0 + 3 < cw) && ((cw & 3) == 0);
            int64_t wc[4];
            bool wl[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wl[j] = (w0 + j) < cw;
                wc[j] = wl[j] ? w0 + j : cw - 1;
            }
            uint32_t bits[R][PPP][4];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < PPP; ++i) {
                    const int ic = i < q_used ? i : q_used - 1;
                    const uint32_t* pr = pbase + (prow[r] - planes) + (int64_t)ic * plane_stride;
                    if (quad) {
                        const s_u32x4 v4 = *reinterpret_cast<const s_u32x4*>(pr + w0);
#pragma unroll
                        for (int j = 0; j < 4; ++j) bits[r][i][j] = v4[j];
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) bits[r][i][j] = pr[wc[j]];
                    }
                }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                ActRaw araw[2][4];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        araw[jj][u] = load_act_raw(act_row + wc[2 * half + jj] * 32, u, tok_live && wl[2 * half + jj]);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int j = 2 * half + jj;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const s_bf16x8 v = act_frag(araw[jj][u]);
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int i = 0; i < PPP; ++i) {
                                acc[r][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(expand_signs(bits[r][i][j], u), v,
                                                                                    acc[r][i], 0, 0, 0);
                            }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    }

    // Accumulator register v of lane l: plane-matrix row 4 * (l / 16) + v of the tile, token l % 16.
    // FWD folds alpha into one tile per row block before the cross-wave sum; DALPHA keeps the planes apart.
    constexpr int NOUT = (MODE == SMALL_DALPHA) ? QP : 1;
    const int nout = (MODE == SMALL_DALPHA) ? q_used : 1;
    s_f32x4 part[R][NOUT];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (MODE == SMALL_FWD) {
            s_f32x4 y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < QP; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) y[v] += ep[r][i][v] * acc[r][i][v];  // alpha of unused planes is 0
            part[r][0] = y;
        } else {
#pragma unroll
            for (int i = 0; i < NOUT; ++i) part[r][i] = acc[r][i < NACC ? i : 0];
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
            for (int v = 0; v < 4; ++v) d[v] = ep[r][0][v];
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

struct SmallPlan {
    int R, W, segs_per_wave;
    unsigned grid_x;
};

static SmallPlan small_plan(int64_t rows, int64_t cw) {
    SmallPlan p;
    const int64_t segs = (cw + 15) / 16;  // 512-column segments
    // two row tiles per wave (half the activation traffic per plane byte) only when there are rows to spare
    p.R = rows >= 16384 ? 2 : 1;
    const int64_t blocks = (rows + 16 * p.R - 1) / (16 * p.R);
    // waves per workgroup: aim at about two waves per SIMD (2048 on the chip); among the candidates from there
    // up to 8 take the first that keeps every wave at least 80 % loaded, else the best balanced
    const int wmax = (int)(segs < 8 ? segs : 8);
    int w0 = (int)((2048 + blocks - 1) / blocks);
    w0 = w0 < 1 ? 1 : (w0 > wmax ? wmax : w0);
    int best_w = w0;
    double best_eff = 0.0;
    for (int w = w0; w <= wmax; ++w) {
        const int64_t spw = (segs + w - 1) / w;
        const double eff = (double)segs / (double)(w * spw);
        if (eff >= 0.8) { best_w = w; break; }
        if (eff > best_eff + 1e-9) { best_eff = eff; best_w = w; }
    }
    p.W = best_w;
    p.segs_per_wave = (int)((segs + best_w - 1) / best_w);
    p.grid_x = (unsigned)((rows + 16 * p.R - 1) / (16 * p.R));
    return p;
}

template <int MODE>
static hipError_t launch_small(const uint32_t* planes, const bf16_t* act, const float* alpha, const bf16_t* dy,
                               void* out, int64_t T, int64_t rows, int64_t cw, int q, int q_used, float scale,
                               hipStream_t st) {
    const SmallPlan p = small_plan(rows, cw);
    const dim3 grid(p.grid_x, (unsigned)((T + 15) / 16));
    const dim3 block((unsigned)(64 * p.W));
    if (p.W < 1 || p.W > 8) return hipErrorInvalidConfiguration;  // the kernel is compiled for at most 512 threads
    const int nout = (MODE == SMALL_DALPHA) ? q_used : 1;
    const size_t lds = (size_t)p.W * p.R * nout * 64 * 4 * sizeof(float);
    const int qp = q_used <= 4 ? q_used : 8;
    // more than 64 KiB of dynamic LDS (many rows, 5 .. 8 trained planes) needs the kernel's limit raised first
#define BCQ_SMALL_LAUNCH(RR, QQ)                                                                                   \
    {                                                                                                              \
        static LdsLimit limit;                                                                                     \
        const hipError_t le = limit.ensure((const void*)small_kernel<MODE, RR, QQ>, lds);                          \
        if (le != hipSuccess) return le;                                                                           \
        BCQ_LAUNCH((small_kernel<MODE, RR, QQ>), grid, block, lds, st, planes, act, alpha, dy, out, T, rows, cw, q, \
                           q_used, scale, p.segs_per_wave);                                                        \
    }
#define BCQ_SMALL_Q(RR)                                          \
    switch (qp) {                                                \
        case 1: BCQ_SMALL_LAUNCH(RR, 1); break;                  \
        case 2: BCQ_SMALL_LAUNCH(RR, 2); break;                  \
        case 3: BCQ_SMALL_LAUNCH(RR, 3); break;                  \
        case 4: BCQ_SMALL_LAUNCH(RR, 4); break;                  \
        default: BCQ_SMALL_LAUNCH(RR, 8); break;                 \
    }
    if (p.R == 2) {
        BCQ_SMALL_Q(2)
    } else {
        BCQ_SMALL_Q(1)
    }
#undef BCQ_SMALL_Q
#undef BCQ_SMALL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_fwd_small(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                            int64_t K, int q, void* y, hipStream_t st) {
    return launch_small<SMALL_FWD>(packed, (const bf16_t*)x, alpha, nullptr, y, T, N, K / 32, q, q, 1.f, st);
}

hipError_t launch_bwd_alpha_small(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                  int64_t K, int q, int q_train, float grad_scale, float* dalpha, hipStream_t st) {
    return launch_small<SMALL_DALPHA>(packed, (const bf16_t*)x, nullptr, (const bf16_t*)dy, dalpha, T, N, K / 32, q,
                                      q_train, grad_scale, st);
}

}  // namespace bcq
