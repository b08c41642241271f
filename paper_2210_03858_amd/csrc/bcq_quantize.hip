// Greedy BCQ quantizer (AlphaTuning Appendix C: Eq. ap1 for the first plane, Eq. ap2-ap3 for the rest).
// The fp64 residual of a whole row stays in registers across the q planes, so W is read from HBM exactly once
// (4 N K bytes) and only alpha and the packed signs are written.  HBM bound; the fp64 abs-sum, compare and
// subtract are a few ALU operations per weight.  Rows of up to 4096 columns take one WAVE each (four rows per
// workgroup, no LDS, no barrier: the per-plane sum is a wave reduction); longer rows take one 256-thread
// workgroup each with the four waves' sums combined through LDS.
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
