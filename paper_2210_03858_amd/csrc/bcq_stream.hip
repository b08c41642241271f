// Host side of the small-token streaming kernels (bcq_stream_kernels.h): launch plans and the single-layer launchers.
#include "bcq_stream_kernels.h"

namespace bcq {

// ---------------------------------------------------------------------------------------------------------
// gsegs > 0: the contraction axis carries scale groups of gsegs segments each and every wave must own whole groups
static StreamPlan stream_plan(int64_t T, int64_t rows, int64_t cw, int gsegs = 0) {
    StreamPlan p;
    p.segs = (cw + 15) / 16;
    p.halves = T <= 8 ? 1 : 2;
    p.tiles = (int)((T + 15) / 16);
    // One 16-row tile per wave: measured faster than two at every size (more waves keep more plane bytes in flight,
    // which is what bounds the stream; the activation operand is L2-resident either way).
    p.R = 1;
    const int64_t blocks = (rows + 16 * p.R - 1) / (16 * p.R);
    // waves per workgroup: aim at about two waves per SIMD (2048 on the chip); among the candidates from there up to
    // 8 take the first that keeps every wave at least 80 % loaded, else the best balanced
    const int wmax = (int)(p.segs < 8 ? p.segs : 8);
    int w0 = (int)((2048 + blocks - 1) / blocks);
    w0 = w0 < 1 ? 1 : (w0 > wmax ? wmax : w0);
    int best_w = w0;
    double best_eff = 0.0;
    for (int w = w0; w <= wmax; ++w) {
        const int64_t spw = (p.segs + w - 1) / w;
        const double eff = (double)p.segs / (double)(w * spw);
        if (eff >= 0.8) {
            best_w = w;
            break;
        }
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            best_w = w;
        }
    }
    p.W = best_w;
    p.segs_per_wave = (int)((p.segs + best_w - 1) / best_w);
    if (gsegs > 0) {  // whole groups per wave
        const int64_t groups = p.segs / gsegs;
        if (p.W > groups) p.W = (int)groups;
        const int64_t gpw = (groups + p.W - 1) / p.W;
        p.W = (int)((groups + gpw - 1) / gpw);
        p.segs_per_wave = (int)(gpw * gsegs);
    }
    p.grid_x = (unsigned)((rows + 16 * p.R - 1) / (16 * p.R));
    p.xq_bytes = (size_t)p.tiles * p.segs * 4 * p.halves * QBLK;
    p.sq_bytes = (size_t)p.tiles * p.segs * p.halves * QSCL;
    return p;
}

size_t stream_workspace(int64_t T, int64_t contraction, int sets) {
    const StreamPlan p = stream_plan(T, 16, contraction / 32);
    return (size_t)sets * (p.xq_bytes + p.sq_bytes);
}

// Plan of stream_lds_kernel: KW = 0 means "use stream_kernel".  It pays when the workgroups (8 / KW row tiles each)
// still fill the chip, i.e. for plane matrices with many rows (at least min_wgs workgroups).
struct LdsPlan {
    int KW, spp;
    bool exact;
    unsigned grid_x;
};
static LdsPlan lds_plan(int64_t rows, int64_t segs, int halves, int gsegs, int q_used, int min_wgs = 224) {
    LdsPlan p = {0, 0, false, 0};
    if (q_used > 4) return p;  // the ring of plane registers is sized for up to 4 planes
    const int64_t rt = (rows + 15) / 16;
    int kw = 0;
    if ((rt + 7) / 8 >= min_wgs)
        kw = 1;
    else if (halves == 1 && (rt + 3) / 4 >= min_wgs)
        kw = 2;
    if (kw == 0 || segs < 2 * LCS * kw) return p;
    int64_t spp = (segs + kw - 1) / kw;
    if (gsegs > 0) spp = (spp + gsegs - 1) / gsegs * gsegs;  // whole scale groups per part
    p.KW = kw;
    p.spp = (int)spp;
    p.exact = (spp * kw == segs) && (spp % LCS == 0);
    p.grid_x = (unsigned)((rt + (8 / kw) - 1) / (8 / kw));
    return p;
}

template <int MODE, int QP, bool TWO, bool GROUPED, int KW, bool EXACT, bool TILED>
static hipError_t launch_lds_cfg(const uint32_t* planes, const unsigned char* xq, const unsigned char* sq,
                                 const float* alpha, const bf16_t* dy, void* out, int64_t T, int64_t rows, int64_t cw,
                                 int q_used, float scale, const LdsPlan& lp, int64_t segs, int tiles, int gsegs, int G,
                                 hipStream_t st, int64_t xq_plane = 0, int64_t sq_plane = 0, uint32_t seg_magic = 0,
                                 int segs_n = 0) {
    constexpr int H = TWO ? 2 : 1;
    constexpr int LDS_B = 2 * KW * LCS * H * (4 * QBLK + QSCL);
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)stream_lds_kernel<MODE, QP, TWO, GROUPED, KW, EXACT, TILED>, LDS_B);
    if (e != hipSuccess) return e;
    BCQ_LAUNCH((stream_lds_kernel<MODE, QP, TWO, GROUPED, KW, EXACT, TILED>), dim3(lp.grid_x, (unsigned)tiles), dim3(512),
                       LDS_B, st, planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale, lp.spp, segs, gsegs, G, xq_plane,
                       sq_plane, seg_magic, segs_n);
    return hipGetLastError();
}

// input gradient through stream_lds_kernel: one virtual plane over q * segs_n segments
static hipError_t launch_lds_dx(const uint32_t* twin, const unsigned char* xq, const unsigned char* sq, void* out, int64_t T,
                                int64_t rows, int64_t cw, const LdsPlan& lp, int64_t vsegs, int tiles, int halves,
                                int64_t xq_plane, int64_t sq_plane, int segs_n, int G, hipStream_t st) {
    const uint32_t magic = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)segs_n - 1) / (uint64_t)segs_n);
#define BCQ_LDS_DX(TT, KW, EX)                                                                                          \
    return launch_lds_cfg<STREAM_DX, 1, TT, false, KW, EX, false>(twin, xq, sq, nullptr, nullptr, out, T, rows, cw, 1, 1.f, lp, \
                                                                  vsegs, tiles, 1, G, st, xq_plane, sq_plane, magic, segs_n)
    if (halves == 2) {
        if (lp.exact) BCQ_LDS_DX(true, 1, true);
        BCQ_LDS_DX(true, 1, false);
    }
    if (lp.KW == 2) {
        if (lp.exact) BCQ_LDS_DX(false, 2, true);
        BCQ_LDS_DX(false, 2, false);
    }
    if (lp.exact) BCQ_LDS_DX(false, 1, true);
    BCQ_LDS_DX(false, 1, false);
#undef BCQ_LDS_DX
}

template <int MODE, int QP, bool TWO, bool GROUPED, bool TILED>
static hipError_t launch_lds_kw(const uint32_t* planes, const unsigned char* xq, const unsigned char* sq,
                                const float* alpha, const bf16_t* dy, void* out, int64_t T, int64_t rows, int64_t cw,
                                int q_used, float scale, const LdsPlan& lp, int64_t segs, int tiles, int gsegs, int G,
                                hipStream_t st) {
#define BCQ_LDS_GO(KW, EX) \
    return launch_lds_cfg<MODE, QP, TWO, GROUPED, KW, EX, TILED>(planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale, lp, \
                                                          segs, tiles, gsegs, G, st)
    if (!TWO && lp.KW == 2) {
        if (lp.exact) BCQ_LDS_GO((TWO ? 1 : 2), true);
        BCQ_LDS_GO((TWO ? 1 : 2), false);
    }
    if (lp.exact) BCQ_LDS_GO(1, true);
    BCQ_LDS_GO(1, false);
#undef BCQ_LDS_GO
}

template <int MODE, bool TILED>
static hipError_t launch_lds(const uint32_t* planes, const unsigned char* xq, const unsigned char* sq, const float* alpha,
                             const bf16_t* dy, void* out, int64_t T, int64_t rows, int64_t cw, int q_used, float scale,
                             const LdsPlan& lp, int64_t segs, int tiles, int halves, bool grouped, int gsegs, int G,
                             hipStream_t st) {
#define BCQ_LDS_ARGS planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale, lp, segs, tiles, gsegs, G, st
#define BCQ_LDS_Q(QQ)                                                                          \
    if (halves == 2) {                                                                         \
        if (grouped) return launch_lds_kw<MODE, QQ, true, true, TILED>(BCQ_LDS_ARGS);          \
        return launch_lds_kw<MODE, QQ, true, false, TILED>(BCQ_LDS_ARGS);                      \
    } else {                                                                                   \
        if (grouped) return launch_lds_kw<MODE, QQ, false, true, TILED>(BCQ_LDS_ARGS);         \
        return launch_lds_kw<MODE, QQ, false, false, TILED>(BCQ_LDS_ARGS);                     \
    }
    switch (q_used) {
        case 1: BCQ_LDS_Q(1)
        case 2: BCQ_LDS_Q(2)
        case 3: BCQ_LDS_Q(3)
        default: BCQ_LDS_Q(4)
    }
#undef BCQ_LDS_Q
#undef BCQ_LDS_ARGS
}

// g = group size of the scales along the columns of W (K of the layer); g == layer K means row-wise.
// The single-kernel form is used when a wave has one segment and all waves of the launch are resident at once
// (every wave repeats the re-coding of its segment, about 2.5 us of vector-ALU work; measured: 2560 x 2560 and
// 5120 x 1280 gain 2.3 - 2.7 us per call, 7680 x 2560 loses 1.7 us, 10240 x 2560 loses 8 us)
constexpr int FUSED_MAX_SEGS = 1;
constexpr int64_t FUSED_MAX_WAVES = 1024;

template <int MODE, int QP, bool TWO>
static hipError_t launch_fused_cfg(const uint32_t* planes, const bf16_t* act, const float* alpha, const bf16_t* dy,
                                   void* out, int64_t T, int64_t rows, int64_t cw, int q_used, float scale,
                                   const StreamPlan& p, int gsegs, int G, hipStream_t st) {
    constexpr int H = TWO ? 2 : 1;
    const int nout = (MODE == STREAM_DALPHA) ? q_used : 1;
    const size_t stage = (size_t)p.W * (4 * H * QBLK + H * QSCL), red = (size_t)p.W * nout * 1024;
    const size_t lds = stage > red ? stage : red;
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)stream_fused_kernel<MODE, QP, TWO>, lds);
    if (e != hipSuccess) return e;
    BCQ_LAUNCH((stream_fused_kernel<MODE, QP, TWO>), dim3(p.grid_x, (unsigned)p.tiles), dim3((unsigned)(64 * p.W)),
                       lds, st, planes, act, alpha, dy, out, T, rows, cw, q_used, scale, p.segs_per_wave, p.segs, gsegs, G);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_fused(const uint32_t* planes, const bf16_t* act, const float* alpha, const bf16_t* dy, void* out,
                               int64_t T, int64_t rows, int64_t cw, int q_used, float scale, const StreamPlan& p,
                               int gsegs, int G, hipStream_t st) {
#define BCQ_FUSED_Q(QQ)                                                                                                \
    if (p.halves == 2)                                                                                                 \
        return launch_fused_cfg<MODE, QQ, true>(planes, act, alpha, dy, out, T, rows, cw, q_used, scale, p, gsegs, G, st); \
    return launch_fused_cfg<MODE, QQ, false>(planes, act, alpha, dy, out, T, rows, cw, q_used, scale, p, gsegs, G, st);
    switch (q_used <= 4 ? q_used : 8) {
        case 1: BCQ_FUSED_Q(1)
        case 2: BCQ_FUSED_Q(2)
        case 3: BCQ_FUSED_Q(3)
        case 4: BCQ_FUSED_Q(4)
        default: BCQ_FUSED_Q(8)
    }
#undef BCQ_FUSED_Q
}

template <int MODE, bool TILED = false>
static hipError_t launch_stream(const uint32_t* planes, const bf16_t* act, const float* alpha, const bf16_t* dy, void* out,
                                int64_t T, int64_t rows, int64_t cw, int q, int q_used, float scale, void* workspace,
                                int64_t g, int64_t layer_k, hipStream_t st) {
    const bool grouped = (g != layer_k);
    const int G = (int)(layer_k / g);
    const int gsegs = (grouped && MODE != STREAM_DX) ? (int)(g / 512) : 0;  // needs g % 512 == 0 (checked by the caller)
    const StreamPlan p = stream_plan(T, rows, cw, gsegs);
    if (p.W < 1 || p.W > 8 || p.R != 1) return hipErrorInvalidConfiguration;  // compiled for at most 512 threads, R = 1
    if constexpr (MODE != STREAM_DX && !TILED) {
        int fused_max = FUSED_MAX_SEGS;
        if (p.segs_per_wave <= fused_max && p.R == 1 && (int64_t)p.grid_x * p.tiles * p.W <= FUSED_MAX_WAVES)
            return launch_fused<MODE>(planes, act, alpha, dy, out, T, rows, cw, q_used, scale, p, gsegs, G, st);
    }
    const int sets = (MODE == STREAM_DX) ? q * G : 1;
    unsigned char* xq = reinterpret_cast<unsigned char*>(workspace);
    unsigned char* sq = xq + (size_t)sets * p.xq_bytes;
    {
        const int64_t threads = (int64_t)p.tiles * p.segs * 256;
        const dim3 grid((unsigned)((threads + 255) / 256), (unsigned)sets);
        BCQ_LAUNCH((quant_act_kernel<MODE>), grid, dim3(256), 0, st, act, alpha, T, cw * 32, p.segs, p.halves,
                           p.tiles, xq, sq, p.xq_bytes, p.sq_bytes, G);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if constexpr (MODE == STREAM_DX) {
        if (cw % 16 == 0) {  // whole segments
            const int64_t vsegs = (int64_t)q_used * p.segs;
            // the per-wave kernel fetches one activation set per plane and row tile, so sharing pays from fewer
            // workgroups than for the forward (measured at 8 tokens: 10240 rows 18.0 -> 14.9 us, 12288 rows equal,
            // 6144 rows 3 % slower)
            const LdsPlan lp = lds_plan(rows, vsegs, p.halves, 0, 1, p.halves == 1 ? 160 : 224);
            // group-wise scales: a workgroup (8 / KW row tiles of the twin) takes ONE activation set, so its rows must
            // lie in one scale group; other group sizes keep the per-wave kernel (16 rows per workgroup, g % 32 == 0)
            const bool one_group = (G == 1) || (lp.KW > 0 && g % (16 * (8 / lp.KW)) == 0);
            if (lp.KW > 0 && one_group)
                return launch_lds_dx(planes, xq, sq, out, T, rows, cw, lp, vsegs, p.tiles, p.halves, (int64_t)p.xq_bytes,
                                     (int64_t)p.sq_bytes, (int)p.segs, G, st);
        }
    }
    if constexpr (MODE != STREAM_DX) {
        if (TILED || cw % 4 == 0) {
            const LdsPlan lp = lds_plan(rows, p.segs, p.halves, gsegs, q_used);
            if (lp.KW > 0)
                return launch_lds<MODE, TILED>(planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale, lp, p.segs, p.tiles,
                                        p.halves, grouped, gsegs > 0 ? gsegs : 1, G, st);
        }
    }
    const dim3 grid(p.grid_x, (unsigned)p.tiles);
    const dim3 block((unsigned)(64 * p.W));
    const int nout = (MODE == STREAM_DALPHA) ? q_used : 1;
    const size_t lds = (size_t)p.W * p.R * nout * 64 * 4 * sizeof(float);
    const int qp = q_used <= 4 ? q_used : 8;
    const bool quad = TILED || (cw % 4 == 0);  // the decode layout has one instantiation (the flag is unused there)
#define BCQ_STREAM_GO(QQ, TT, QD, GR)                                                                                  \
    BCQ_LAUNCH((stream_kernel<MODE, 1, QQ, TT, QD, GR, TILED>), grid, block, lds, st, planes, xq, sq, alpha, dy, out, T, \
                       rows, cw, q_used, scale, p.segs_per_wave, p.segs, p.xq_bytes, p.sq_bytes, 127,                  \
                       gsegs > 0 ? gsegs : 1, G, g)
#define BCQ_STREAM_GR(QQ, TT, QD)            \
    if (grouped) {                           \
        BCQ_STREAM_GO(QQ, TT, QD, true);     \
    } else {                                 \
        BCQ_STREAM_GO(QQ, TT, QD, false);    \
    }
#define BCQ_STREAM_QD(QQ, TT)            \
    if (quad) {                          \
        BCQ_STREAM_GR(QQ, TT, true)      \
    } else {                             \
        BCQ_STREAM_GR(QQ, TT, TILED)     \
    }
#define BCQ_STREAM_Q(TT)                              \
    switch (qp) {                                     \
        case 1: BCQ_STREAM_QD(1, TT) break;           \
        case 2: BCQ_STREAM_QD(2, TT) break;           \
        case 3: BCQ_STREAM_QD(3, TT) break;           \
        case 4: BCQ_STREAM_QD(4, TT) break;           \
        default: BCQ_STREAM_QD(8, TT) break;          \
    }
    if (p.halves == 2) {
        BCQ_STREAM_Q(true)
    } else {
        BCQ_STREAM_Q(false)
    }
#undef BCQ_STREAM_Q
#undef BCQ_STREAM_QD
#undef BCQ_STREAM_GR
#undef BCQ_STREAM_GO
    return hipGetLastError();
}

size_t stream_fwd_workspace(int64_t T, int64_t K) { return stream_workspace(T, K, 1); }
size_t stream_bwd_alpha_workspace(int64_t T, int64_t K) { return stream_workspace(T, K, 1); }
size_t stream_bwd_input_workspace(int64_t T, int64_t N, int sets) { return stream_workspace(T, N, sets); }

hipError_t launch_fwd_stream(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                             int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st) {
    return launch_stream<STREAM_FWD>(packed, (const bf16_t*)x, alpha, nullptr, y, T, N, K / 32, q, q, 1.f, workspace, g, K,
                                     st);
}

hipError_t launch_fwd_stream_decode(const uint32_t* tiled, const float* alpha, const void* x, int64_t T, int64_t N,
                                    int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st) {
    return launch_stream<STREAM_FWD, true>(tiled, (const bf16_t*)x, alpha, nullptr, y, T, N, K / 32, q, q, 1.f, workspace,
                                           g, K, st);
}

// canonical packed[q][N][K/32] -> decode layout [N/16 up][K/512 up][q][64 lanes][4 words]; lane = (n % 16) + 16 g holds
// words 16 seg + 4 g .. + 3 of row n; rows and columns beyond the matrix read as 0 bits
__global__ __launch_bounds__(256) void pack_decode_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t cw,
                                                          int q, int64_t segs, int64_t units,
                                                          q_u32x4* __restrict__ tiled) {
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one 16-byte unit of the output
    if (u >= units) return;
    const int lane = (int)(u & 63);
    const int i = (int)((u >> 6) % q);
    const int64_t ts = (u >> 6) / q;
    const int64_t seg = ts % segs, rt = ts / segs;
    const int64_t n = rt * 16 + (lane & 15);
    const int64_t w0 = seg * 16 + 4 * (lane >> 4);
    q_u32x4 v = {0u, 0u, 0u, 0u};
    if (n < N) {
        const uint32_t* src = packed + ((int64_t)i * N + n) * cw;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            if (w0 + jj < cw) v[jj] = src[w0 + jj];
    }
    tiled[u] = v;
}

size_t decode_layout_bytes(int64_t N, int64_t K, int q) {
    return (size_t)((N + 15) / 16) * (size_t)((K + 511) / 512) * (size_t)q * 1024;
}

hipError_t launch_pack_decode(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* tiled, hipStream_t st) {
    const int64_t segs = (K + 511) / 512;
    const int64_t units = (int64_t)(decode_layout_bytes(N, K, q) / 16);
    BCQ_LAUNCH(pack_decode_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, packed, N, K / 32, q, segs,
                       units, reinterpret_cast<q_u32x4*>(tiled));
    return hipGetLastError();
}

hipError_t launch_bwd_alpha_stream(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                   int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                                   void* workspace, hipStream_t st) {
    return launch_stream<STREAM_DALPHA>(packed, (const bf16_t*)x, nullptr, (const bf16_t*)dy, dalpha, T, N, K / 32, q,
                                        q_train, grad_scale, workspace, g, K, st);
}

hipError_t launch_bwd_input_stream(const uint32_t* packed_t, const float* alpha, const void* dy, int64_t T, int64_t N,
                                   int64_t K, int64_t g, int q, void* dx, void* workspace, hipStream_t st) {
    return launch_stream<STREAM_DX>(packed_t, (const bf16_t*)dy, alpha, nullptr, dx, T, K, N / 32, q, q, 1.f, workspace,
                                    g, K, st);
}

}  // namespace bcq
