// Greedy BCQ quantizer (AlphaTuning Appendix C: Eq. ap1 for the first plane, Eq. ap2-ap3 for the rest).
// The fp64 residual of a whole row stays in registers across the q planes, so W is read from HBM exactly once
// (4 N K bytes) and only alpha and the packed signs are written.  Two forms:
//   quantize_rows_kernel  rows of whole 256-column chunks (every layer shape of the workloads): 16-byte loads, four
//                         ALU instructions per weight and plane, the sign bits packed inside the lane and
//                         transposed between 8 lanes; one wave per row up to 2560 columns, 2 or 4 waves above.
//   quantize_kernel       any K % 32 == 0 up to 16384: one column per lane and chunk of 64, ballots gathered with
//                         v_writelane; one wave per row up to 4096 columns, else one workgroup per row.
// With q = 1 the first form streams W at 0.77 of the HBM peak; each further plane adds its ALU time (four fp64
// or bit instructions per weight), which the loads of other waves only partly hide.
//
// Arithmetic (what makes the sign planes reproducible bit for bit): residual and abs-sum in fp64, mean
// rounded once to fp32, that fp32 value subtracted.  Only the ORDER of the fp64 sum is free.
#include "bcq_internal.h"

#include <type_traits>

namespace bcq {

// compile-time loop: f(std::integral_constant<int, C>) for C = BEGIN .. END - 1
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

// dst[lane L] = v (v wave-uniform); the lane index must be an instruction constant.  The scalar operand is usually
// the result of a vector compare issued just before; inside inline assembly the compiler cannot see that
// dependency, so the wait states the hardware wants between a vector write of a scalar register and its use here
// are spelled out.
template <int L>
__device__ __forceinline__ void write_lane(uint32_t& dst, uint32_t v) {
    asm volatile("s_nop 4\n\tv_writelane_b32 %0, %1, %2" : "+v"(dst) : "s"(v), "n"(L));
}

// The same for four chunks at once: four sign-bit compares (sign bit clear <=> high word > -1 as an integer), then
// the eight lane writes.  Written out so that every lane write comes at least four issue slots after the compare
// whose scalar result it reads - the compares of the other chunks and one s_nop fill them - instead of five idle
// slots before each of the eight.  Both blocks are volatile, so nothing moves between or across them in a way that
// shortens those distances.
template <int L0>
__device__ __forceinline__ void ballots4(int h0, int h1, int h2, int h3, uint32_t& lo, uint32_t& hi) {
    uint64_t m0, m1, m2, m3;
    asm volatile(
        "v_cmp_gt_i32 %0, %4, -1\n\t"
        "v_cmp_gt_i32 %1, %5, -1\n\t"
        "v_cmp_gt_i32 %2, %6, -1\n\t"
        "v_cmp_gt_i32 %3, %7, -1"
        : "=s"(m0), "=s"(m1), "=s"(m2), "=s"(m3)
        : "v"(h0), "v"(h1), "v"(h2), "v"(h3));
    asm volatile(
        "s_nop 0\n\t"
        "v_writelane_b32 %0, %2, %10\n\t"
        "v_writelane_b32 %1, %3, %10\n\t"
        "v_writelane_b32 %0, %4, %11\n\t"
        "v_writelane_b32 %1, %5, %11\n\t"
        "v_writelane_b32 %0, %6, %12\n\t"
        "v_writelane_b32 %1, %7, %12\n\t"
        "v_writelane_b32 %0, %8, %13\n\t"
        "v_writelane_b32 %1, %9, %13"
        : "+v"(lo), "+v"(hi)
        : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)),
          "s"((uint32_t)m2), "s"((uint32_t)(m2 >> 32)), "s"((uint32_t)m3), "s"((uint32_t)(m3 >> 32)),
          "n"(L0), "n"(L0 + 1), "n"(L0 + 2), "n"(L0 + 3));
}

// Chunk cc of a row = columns 64 cc .. 64 cc + 63.  WAVE_ROW = true: wave w owns the whole row 4 blockIdx.x + w,
// register r[c] of lane l holds column 64 c + l.  WAVE_ROW = false: the four waves of the block share row
// blockIdx.x, wave w takes chunks 4 c + w.  Either way every chunk of a wave is entirely inside the row except
// at most one (K % 64 == 32), so all guards are wave-uniform but one lane mask.
//
// Signs come from the sign bit of the residual: the weights are normalised with + 0.0 on load (-0.0 -> +0.0) and
// x - x = +0.0 afterwards, so "sign bit clear" is exactly r >= 0 (rows with NaN have unspecified outputs).
// The wave-uniform ballot of chunk c goes into lane c with v_writelane, so that the packed words leave as one
// coalesced store per plane; the subtraction r -= alpha * b is r - copysign(alpha, r) on the high word.
// EXACT: every wave has exactly CMAX whole chunks (K == 64 NW CMAX), so no guard is needed at all.
template <int CMAX, bool WAVE_ROW, bool EXACT>
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ W, int64_t N, int K, int q,
                                                       float* __restrict__ alpha, uint32_t* __restrict__ packed,
                                                       int8_t* __restrict__ planes, int* __restrict__ status_word) {
    __shared__ double wave_sum[4];
    constexpr int NW = WAVE_ROW ? 1 : 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n = WAVE_ROW ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    if (WAVE_ROW && n >= N) return;  // whole wave leaves; this form has no barrier
    const int wv = WAVE_ROW ? 0 : wave;
    const float* wrow = W + n * (int64_t)K;
    const int Kw = K / 32;
    // chunks of this wave that reach into the row (uniform), and whether the last of them is only half inside
    const int chunks_row = (K + 63) / 64;
    const int nch = EXACT ? CMAX : (chunks_row > wv ? (chunks_row - wv + NW - 1) / NW : 0);  // <= CMAX
    const int last = nch - 1;
    const bool last_half = !EXACT && (nch > 0) && (((last * NW + wv) * 64 + 64) > K);
    const bool lane_in_last = !last_half || lane < 32;

    double r[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        r[c] = 0.0;
        if (EXACT || c < nch) {
            const int k = (c * NW + wv) * 64 + lane;
            if (EXACT || c < last || lane_in_last) r[c] = (double)wrow[k] + 0.0;
        }
    }

    for (int i = 0; i < q; ++i) {
        double s = 0.0;
        uint32_t mine_lo = 0u, mine_hi = 0u;
        if constexpr (CMAX % 4 == 0) {
            // chunks beyond the row hold +0.0: they add nothing to the sum, and their ballots land in lanes that
            // store nothing, so no guard is needed here
            static_for<0, CMAX / 4>([&](auto gg) {
                constexpr int c = 4 * decltype(gg)::value;
                s += (fabs(r[c]) + fabs(r[c + 1])) + (fabs(r[c + 2]) + fabs(r[c + 3]));
                ballots4<c>(__double2hiint(r[c]), __double2hiint(r[c + 1]), __double2hiint(r[c + 2]),
                            __double2hiint(r[c + 3]), mine_lo, mine_hi);
            });
        } else {
            static_for<0, CMAX>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                if (EXACT || c < nch) {
                    s += fabs(r[c]);
                    const uint64_t m = __ballot((int)__double2hiint(r[c]) >= 0);  // sign bit clear <=> +1
                    write_lane<c>(mine_lo, (uint32_t)m);                          // the ballot is wave-uniform
                    write_lane<c>(mine_hi, (uint32_t)(m >> 32));
                }
            });
        }
        // sum of |r| over the row in fp64
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        double S = s;
        if (!WAVE_ROW) {
            __syncthreads();  // wave_sum of the previous plane has been read by everyone
            if (lane == 0) wave_sum[wave] = s;
            __syncthreads();
            S = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
        }
        const float a = (float)(S / (double)K);
        if (WAVE_ROW ? (lane == 0) : (threadIdx.x == 0)) {
            alpha[(int64_t)i * N + n] = a;
            if (i == 0 && status_word && !(fabs(S) <= 1.79769313486231570e308)) atomicAdd(status_word, 1);
        }
        // packed words: lane c writes the two words of its chunk (8 bytes; consecutive lanes are 8 NW bytes apart)
        if (lane < nch) {
            const int k0 = (lane * NW + wv) * 64;
            uint32_t* dst = packed + ((int64_t)i * N + n) * Kw + k0 / 32;
            dst[0] = mine_lo;
            if (k0 + 32 < K) dst[1] = mine_hi;
        }
        if (planes) {
#pragma unroll
            for (int c = 0; c < CMAX; ++c) {
                if (EXACT || (c < nch && (c < last || lane_in_last))) {
                    const int k = (c * NW + wv) * 64 + lane;
                    planes[((int64_t)i * N + n) * K + k] = ((int)__double2hiint(r[c]) >= 0) ? (int8_t)1 : (int8_t)-1;
                }
            }
        }
        // r -= alpha * b, b = sign of r: subtract alpha carrying r's sign bit.  Lanes of the half chunk that lie beyond
        // the row subtract 0, so they stay +0.0 and never add to the abs-sum.
        const double ad = (double)a;
        const double ad_last = lane_in_last ? ad : 0.0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (EXACT || c < nch) {
                const double sub = (!EXACT && c == last) ? ad_last : ad;
                const int hi = __double2hiint(sub) | (__double2hiint(r[c]) & (int)0x80000000);
                r[c] -= __hiloint2double(hi, __double2loint(sub));
            }
        }
    }
}

__global__ void zero_word_kernel(int* p) { *p = 0; }

// ---- rows whose length is a multiple of 256: the fast form ------------------------------------------------------
// One wave-load of 16 bytes per lane covers a CHUNK of 256 columns (lane l holds columns 4 l .. 4 l + 3), so the
// weights arrive as 1 KiB per instruction.  NW waves share a row (wave `sub` takes chunks c NW + sub, c < C) and a
// workgroup holds 4 / NW rows and ends with them: many short workgroups, started by the hardware as others end,
// overlap the loads of some rows with the arithmetic of others better than persistent workgroups that request
// their next row ahead did (measured on the 10240 x 2560 and 2560 x 10240 layers).
//
// Per weight and plane the ALU work is four instructions: |r| into the fp64 sum, the sign bit shifted into a word
// of the lane (v_alignbit), alpha with r's sign bit (v_and_or), and the fp64 subtraction.  The word a lane has
// collected after 8 chunks holds one nibble per chunk; the 32-column words of the canonical layout need one nibble
// from each of 8 neighbouring lanes instead, which is an 8 x 8 nibble transpose inside every group of 8 lanes:
// three exchange steps per 2048 columns and plane.
// Cross-lane moves inside a row of 16 lanes (data-parallel primitives of the vector ALU: a few cycles, where a trip
// through the LDS crossbar costs a hundred).  Every pattern used here is a permutation, so all lanes receive a value.
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1, 0, 3, 2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2, 3, 0, 1]
constexpr int DPP_QUAD_REVERSE = 0x1B; // quad_perm [3, 2, 1, 0]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i of each 8 takes lane 7 - i
constexpr int DPP_MIRROR = 0x140;      // lane i of each 16 takes lane 15 - i

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    return __hiloint2double((int)dpp_move<CTRL>((uint32_t)__double2hiint(v)), (int)dpp_move<CTRL>((uint32_t)__double2loint(v)));
}

// sum over the 64 lanes of a wave, the same value in every lane: four exchange steps inside each row of 16, then
// the four row sums through scalar registers
__device__ __forceinline__ double wave_sum_f64(double s) {
    s += dpp_move<DPP_XOR1>(s);
    s += dpp_move<DPP_XOR2>(s);
    s += dpp_move<DPP_HALF_MIRROR>(s);
    s += dpp_move<DPP_MIRROR>(s);
    auto row = [&](int l) {
        return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(s), l), __builtin_amdgcn_readlane(__double2loint(s), l));
    };
    return (row(0) + row(16)) + (row(32) + row(48));
}

template <int D>
__device__ __forceinline__ uint32_t nibble_exchange(uint32_t x, bool upper) {
    constexpr uint32_t LOW = D == 4 ? 0x0000FFFFu : D == 2 ? 0x00FF00FFu : 0x0F0F0F0Fu;
    constexpr int S = 4 * D;
    // the value of lane ^ D (for D = 4: mirror the 8 lanes, then reverse each 4 of them)
    const uint32_t p = D == 1 ? dpp_move<DPP_XOR1>(x) : D == 2 ? dpp_move<DPP_XOR2>(x)
                                                               : dpp_move<DPP_QUAD_REVERSE>(dpp_move<DPP_HALF_MIRROR>(x));
    // lanes with bit D clear keep their LOW nibbles and take the partner's LOW nibbles into the high places (the
    // partner rotated left by S); the others keep the high ones and take the partner's high nibbles into the LOW
    // places (rotated right by S).  The bits a rotation wraps around fall outside the places taken.
    const uint32_t keep = upper ? ~LOW : LOW;
    const uint32_t rot = __builtin_amdgcn_alignbit(p, p, upper ? S : 32 - S);
    return (x & keep) | (rot & ~keep);
}

template <int C, int NW>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const float* __restrict__ W, int64_t N, int q,
                                                            float* __restrict__ alpha, uint32_t* __restrict__ packed,
                                                            int8_t* __restrict__ planes, int* __restrict__ status_word) {
    constexpr int K = 256 * C * NW, Kw = K / 32, RPB = 4 / NW;
    constexpr int G = (C + 7) / 8;  // groups of up to 8 chunks, one collected word each
    __shared__ double wave_sum[2][4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = wave % NW, rib = wave / NW;
    const int j = lane & 7;
    const float4* W4 = reinterpret_cast<const float4*>(W);

    const int64_t n = (int64_t)blockIdx.x * RPB + rib;
    const bool valid = n < N;  // wave-uniform; a wave without a row works on zeros, joins the barriers and stores nothing
    double r[C][4];
    {
        float4 w[C];
        const float4* src = W4 + n * (K / 4) + lane;
#pragma unroll
        for (int c = 0; c < C; ++c) w[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (valid) {  // one branch around all requests, so that they are in flight together
#pragma unroll
            for (int c = 0; c < C; ++c) w[c] = src[(c * NW + sub) * 64];
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            // + 0.0 turns -0.0 into +0.0, so "sign bit clear" below is exactly r >= 0
            r[c][0] = (double)w[c].x + 0.0;
            r[c][1] = (double)w[c].y + 0.0;
            r[c][2] = (double)w[c].z + 0.0;
            r[c][3] = (double)w[c].w + 0.0;
        }
    }
    int par = 0;  // which of the two sets of wave sums the next plane uses
    {
        for (int i = 0; i < q; ++i) {
            double s0 = 0.0, s1 = 0.0;
            uint32_t X[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                uint32_t x = 0u;
#pragma unroll
                for (int c = (g * 8 + 7 < C ? g * 8 + 7 : C - 1); c >= g * 8; --c) {
                    s0 += fabs(r[c][0]) + fabs(r[c][1]);
                    s1 += fabs(r[c][2]) + fabs(r[c][3]);
#pragma unroll
                    for (int e = 3; e >= 0; --e)
                        x = __builtin_amdgcn_alignbit(x, (uint32_t)__double2hiint(r[c][e]), 31);  // x = x << 1 | sign
                }
                // x: nibble c - 8 g holds the four sign bits of this lane's columns of chunk c (1 = negative).  After
                // the exchange lane 8 w + j holds word w of chunk 8 g + j: the nibble of lane 8 w + t at bits 4 t .. 4 t + 3.
                // (Done here, not at the store, so that it fills the waits of the sum and the division below.)
                x = nibble_exchange<4>(x, (j & 4) != 0);
                x = nibble_exchange<2>(x, (j & 2) != 0);
                X[g] = ~nibble_exchange<1>(x, (j & 1) != 0);  // 1 <=> +1 <=> sign bit clear
            }
            const double s = wave_sum_f64(s0 + s1);
            double S = s;
            if constexpr (NW > 1) {
                double* ws = wave_sum[par];  // two sets in turn: one barrier per plane is enough
                par ^= 1;
                if (lane == 0) ws[wave] = s;
                __syncthreads();
                S = ws[rib * NW];
#pragma unroll
                for (int w = 1; w < NW; ++w) S += ws[rib * NW + w];
            }
            const float a = (float)(S / (double)K);
            if (valid) {
                if (lane == 0 && sub == 0) {
                    alpha[(int64_t)i * N + n] = a;
                    if (i == 0 && status_word && !(fabs(S) <= 1.79769313486231570e308)) atomicAdd(status_word, 1);
                }
                uint32_t* prow = packed + ((int64_t)i * N + n) * Kw;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const int c = g * 8 + j;
                    if (c < C) prow[(c * NW + sub) * 8 + (lane >> 3)] = X[g];
                }
                if (planes) {
                    int8_t* drow = planes + ((int64_t)i * N + n) * K + 4 * lane;
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        uint32_t v = 0u;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            v |= (__double2hiint(r[c][e]) >= 0 ? 0x01u : 0xFFu) << (8 * e);
                        *reinterpret_cast<uint32_t*>(drow + (c * NW + sub) * 256) = v;
                    }
                }
            }
            // r -= alpha * b with b = sign of r,
            // as one fused multiply-add with b = +-1.0 built from r's sign bit (the product is exact, so the result is
            // the correctly rounded r -+ alpha): the low word of b is 0 for every weight, unlike that of alpha
            // (nothing reads the residual of the last plane)
            if (i + 1 < q) {
                const double na = -(double)a;
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int bhi = 0x3FF00000 | (__double2hiint(r[c][e]) & (int)0x80000000);
                        r[c][e] = fma(__hiloint2double(bhi, 0), na, r[c][e]);
                    }
            }
        }
    }
}

template <int C, int NW>
static hipError_t launch_rows(const float* W, int64_t N, int q, float* alpha, uint32_t* packed, int8_t* planes,
                              int* status_word, hipStream_t st) {
    constexpr int RPB = 4 / NW;
    const unsigned blocks = (unsigned)((N + RPB - 1) / RPB);
    BCQ_LAUNCH((quantize_rows_kernel<C, NW>), dim3(blocks), dim3(256), 0, st, W, N, q, alpha, packed, planes, status_word);
    return hipGetLastError();
}

template <int CMAX, bool WAVE_ROW>
static hipError_t launch_q(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                           int8_t* planes, int* status_word, hipStream_t st) {
    const unsigned blocks = (unsigned)(WAVE_ROW ? (N + 3) / 4 : N);
    if (K == (int64_t)64 * (WAVE_ROW ? 1 : 4) * CMAX)
        BCQ_LAUNCH((quantize_kernel<CMAX, WAVE_ROW, true>), dim3(blocks), dim3(256), 0, st, W, N, (int)K, q,
                           alpha, packed, planes, status_word);
    else
        BCQ_LAUNCH((quantize_kernel<CMAX, WAVE_ROW, false>), dim3(blocks), dim3(256), 0, st, W, N, (int)K, q,
                           alpha, packed, planes, status_word);
    return hipGetLastError();
}


hipError_t launch_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                           int8_t* planes, int* status_word, hipStream_t st) {
    if (status_word) {
        BCQ_LAUNCH(zero_word_kernel, dim3(1), dim3(1), 0, st, status_word);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (K % 256 == 0) {  // the fast form, where the row splits into 1, 2 or 4 waves of a supported chunk count
        const int chunks = (int)(K / 256);
#define BCQ_ROWS(CC, NWW) \
    if (chunks == CC * NWW) return launch_rows<CC, NWW>(W, N, q, alpha, packed, planes, status_word, st);
        BCQ_ROWS(1, 1) BCQ_ROWS(2, 1) BCQ_ROWS(3, 1) BCQ_ROWS(4, 1) BCQ_ROWS(5, 1) BCQ_ROWS(6, 1) BCQ_ROWS(8, 1)
        BCQ_ROWS(10, 1) BCQ_ROWS(6, 2) BCQ_ROWS(8, 2) BCQ_ROWS(10, 2) BCQ_ROWS(6, 4) BCQ_ROWS(8, 4) BCQ_ROWS(10, 4)
#undef BCQ_ROWS
    }
#define BCQ_Q_PICK(MODE)                                                                        \
    if (C <= 2) return launch_q<2, MODE>(W, N, K, q, alpha, packed, planes, status_word, st);   \
    if (C <= 4) return launch_q<4, MODE>(W, N, K, q, alpha, packed, planes, status_word, st);   \
    if (C <= 8) return launch_q<8, MODE>(W, N, K, q, alpha, packed, planes, status_word, st);   \
    if (C <= 16) return launch_q<16, MODE>(W, N, K, q, alpha, packed, planes, status_word, st); \
    if (C <= 20) return launch_q<20, MODE>(W, N, K, q, alpha, packed, planes, status_word, st); \
    if (C <= 32) return launch_q<32, MODE>(W, N, K, q, alpha, packed, planes, status_word, st); \
    if (C <= 40) return launch_q<40, MODE>(W, N, K, q, alpha, packed, planes, status_word, st); \
    return launch_q<64, MODE>(W, N, K, q, alpha, packed, planes, status_word, st);
    if (K <= 4096) {  // one wave per row
        const int C = (int)((K + 63) / 64);
        BCQ_Q_PICK(true)
    }
    const int C = (int)((K + 255) / 256);
    BCQ_Q_PICK(false)
#undef BCQ_Q_PICK
}

}  // namespace bcq
