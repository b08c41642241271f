// Look-up-table forward for decode (AlphaTuning Section 6, "Inference Speed": the paper's route to fast small-batch
// inference is a GEMM that never dequantises but indexes tables of partial activation sums with the weight bits).
// A selectable variant of Eq. 2 for 1 .. 4 tokens, next to the default small-token path on the FP4 x FP8 matrix
// instruction, so that the two can be measured against each other on this hardware.
//
// For every group of 4 consecutive columns and every token the 16 signed sums  +-x[4g] +-x[4g+1] +-x[4g+2] +-x[4g+3]
// are a table; a nibble of a packed plane word is the index.  Since the table is odd under complementing the
// nibble, only the 8 entries with bit 3 clear are stored (8 K bytes per token) and bit 3 flips the sign.  A workgroup
// builds the tables of the whole row length in LDS once (fp32, exact sums of four bf16 up to rounding) and then
// serves 32 rows of W: 8 lanes share a row, each walking every 8th packed word of each plane, the lane sums meet
// by shuffles and alpha is applied once per plane and row.
#include "../../include/bcq.h"

#include "bcq_internal.h"

namespace bcq {

constexpr int LUT_ROWS = 32;   // rows of W per workgroup
constexpr int LUT_PARTS = 8;   // lanes per row

template <int T>
__global__ __launch_bounds__(256) void lut_fwd_kernel(const uint32_t* __restrict__ packed, const float* __restrict__ alpha,
                                                      const bf16_t* __restrict__ x, int64_t N, int K, int q,
                                                      bf16_t* __restrict__ y) {
    extern __shared__ __attribute__((aligned(16))) float tab[];  // [T][K / 4][8]
    const int tid = threadIdx.x;
    const int G = K / 4, Kw = K / 32;

    // tables: a thread takes whole groups (one 8-byte load of four bf16, 8 entries = two 16-byte LDS stores); four groups'
    // loads are requested before the first is used.  Entry v = the three low index bits; column 4 g + 3 enters with a
    // minus sign.
    const int groups = T * G;  // (t, g) flattened: x is [T][K], the table [T][G][8]
    for (int g0 = tid; g0 < groups; g0 += 4 * 256) {
        uint2 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gi = g0 + u * 256;
            raw[u] = gi < groups ? *reinterpret_cast<const uint2*>(x + (int64_t)gi * 4) : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int gi = g0 + u * 256;
            if (gi < groups) {
                const float x0 = __uint_as_float(raw[u].x << 16), x1 = __uint_as_float(raw[u].x & 0xFFFF0000u);
                const float x2 = __uint_as_float(raw[u].y << 16), x3 = __uint_as_float(raw[u].y & 0xFFFF0000u);
                float4 lo, hi;  // v = 0 .. 3 and 4 .. 7
                lo.x = -x0 - x1 - x2 - x3;
                lo.y = x0 - x1 - x2 - x3;
                lo.z = -x0 + x1 - x2 - x3;
                lo.w = x0 + x1 - x2 - x3;
                hi.x = -x0 - x1 + x2 - x3;
                hi.y = x0 - x1 + x2 - x3;
                hi.z = -x0 + x1 + x2 - x3;
                hi.w = x0 + x1 + x2 - x3;
                reinterpret_cast<float4*>(tab)[gi * 2] = lo;
                reinterpret_cast<float4*>(tab)[gi * 2 + 1] = hi;
            }
        }
    }
    __syncthreads();

    const int r = tid >> 3, part = tid & 7;
    const int64_t n = (int64_t)blockIdx.x * LUT_ROWS + r;
    const int64_t nc = n < N ? n : N - 1;  // rows beyond the matrix repeat the last one and store nothing
    float yacc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) yacc[t] = 0.f;
    // two independent sums per token (even and odd nibbles), so that consecutive look-ups do not wait for each other
    float s[T], s2[T];
    auto clear_sums = [&]() {
#pragma unroll
        for (int t = 0; t < T; ++t) s[t] = s2[t] = 0.f;
    };
    auto word_sums = [&](uint32_t word, int w) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t nib = (word >> (4 * j)) & 15u;
            const uint32_t flip = 0u - (nib >> 3);           // all ones when bit 3 is set
            const uint32_t idx = (nib ^ flip) & 7u;          // the complement's low bits then
            const int base = (w * 8 + j) * 8 + (int)idx;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float v = __uint_as_float(__float_as_uint(tab[t * G * 8 + base]) ^ (flip & 0x80000000u));
                if (j & 1) s2[t] += v; else s[t] += v;
            }
        }
    };
    auto plane_done = [&](int i) {  // lane sums of the row meet; alpha once per plane and row
        const float a = alpha[(int64_t)i * N + nc];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float v = s[t] + s2[t];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            yacc[t] += a * v;
        }
    };
    if ((Kw & 3) == 0) {
        // 16-byte loads: lane `part` takes words 4 part .. 4 part + 3 of every 32.  The loads of a plane go out in
        // batches of up to 8, and the next batch (of this plane or the next) is requested before the current one is used.
        constexpr int BATCH = 8;
        const int quads = (Kw / 4 - part + LUT_PARTS - 1) / LUT_PARTS;  // of this lane, per plane (lanes beyond Kw / 4: 0)
        const int bpp = (Kw / 4 + LUT_PARTS * BATCH - 1) / (LUT_PARTS * BATCH);  // batches per plane, the same for all lanes
        uint4 cur[BATCH], nxt[BATCH];
        auto request = [&](int b) {
            const int i = b / bpp, h = b - i * bpp;
            const uint32_t* prow = packed + ((int64_t)i * N + nc) * Kw;
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int k = h * BATCH + u;
                nxt[u] = k < quads ? *reinterpret_cast<const uint4*>(prow + 4 * (part + k * LUT_PARTS)) : make_uint4(0u, 0u, 0u, 0u);
            }
        };
        request(0);
        for (int b = 0; b < q * bpp; ++b) {
            const int i = b / bpp, h = b - i * bpp;
#pragma unroll
            for (int u = 0; u < BATCH; ++u) cur[u] = nxt[u];
            if (b + 1 < q * bpp) request(b + 1);
            if (h == 0) clear_sums();
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int k = h * BATCH + u;
                if (k < quads) {
                    const int w = 4 * (part + k * LUT_PARTS);
                    word_sums(cur[u].x, w);
                    word_sums(cur[u].y, w + 1);
                    word_sums(cur[u].z, w + 2);
                    word_sums(cur[u].w, w + 3);
                }
            }
            if (h == bpp - 1) plane_done(i);
        }
    } else {
        for (int i = 0; i < q; ++i) {
            const uint32_t* prow = packed + ((int64_t)i * N + nc) * Kw;
            clear_sums();
            for (int w = part; w < Kw; w += LUT_PARTS) word_sums(prow[w], w);
            plane_done(i);
        }
    }
    if (part == 0 && n < N) {
#pragma unroll
        for (int t = 0; t < T; ++t) y[(int64_t)t * N + n] = f32_to_bf16(yacc[t]);
    }
}

template <int T>
static hipError_t launch_lut_t(const uint32_t* packed, const float* alpha, const bf16_t* x, int64_t N, int64_t K, int q,
                               bf16_t* y, hipStream_t st) {
    const size_t lds = (size_t)T * (size_t)K * 8;
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)lut_fwd_kernel<T>, lds);
    if (e != hipSuccess) return e;
    BCQ_LAUNCH((lut_fwd_kernel<T>), dim3((unsigned)((N + LUT_ROWS - 1) / LUT_ROWS)), dim3(256), lds, st, packed, alpha, x,
               N, (int)K, q, y);
    return hipGetLastError();
}

}  // namespace bcq

extern "C" bcq_status bcq_linear_fwd_lut(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                                         int64_t N, int64_t K, int q, void* y, void* stream) {
    using namespace bcq::host;
    if (!packed || !alpha || !x || !y) return BCQ_ERR_NULL;
    if (!shape_ok(T, N, K, q)) return BCQ_ERR_SHAPE;
    if (T > BCQ_LUT_MAX_TOKENS || (size_t)T * (size_t)K * 8 > (size_t)BCQ_LUT_MAX_TABLE_BYTES) return BCQ_ERR_SHAPE;
    if (N > (int64_t)0x7FFFFFFF * bcq::LUT_ROWS) return BCQ_ERR_SHAPE;
    if (dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (misaligned(packed) || misaligned(alpha) || misaligned(x) || misaligned(y)) return BCQ_ERR_ALIGN;
    if (!device_ok()) return BCQ_ERR_DEVICE;
    const bcq::bf16_t* xb = static_cast<const bcq::bf16_t*>(x);
    bcq::bf16_t* yb = static_cast<bcq::bf16_t*>(y);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    switch (T) {
        case 1: e = bcq::launch_lut_t<1>(packed, alpha, xb, N, K, q, yb, st); break;
        case 2: e = bcq::launch_lut_t<2>(packed, alpha, xb, N, K, q, yb, st); break;
        case 3: e = bcq::launch_lut_t<3>(packed, alpha, xb, N, K, q, yb, st); break;
        default: e = bcq::launch_lut_t<4>(packed, alpha, xb, N, K, q, yb, st); break;
    }
    return e == hipSuccess ? BCQ_OK : BCQ_ERR_DEVICE;
}
