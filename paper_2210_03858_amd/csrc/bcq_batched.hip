// Batched small-token calls: the forward (Eq. 2), the input gradient (Eq. 3) or the scale gradient (Eq. 4) of MANY
// independent layers in two launches (one activation re-coding pre-kernel + one streaming kernel for the whole batch).
//
// Why: a decoder layer of the paper's models holds 0.2 - 13 MB of sign planes, i.e. 0.03 - 1.6 us of HBM time, while a
// launch plus its first memory round trip costs 4 - 11 us.  Called layer by layer the small-token regime (Section 3:
// small-batch inference is memory-bound; Section 6 "Inference Speed") is therefore bound by launches, not by bytes.
// Here a plan (built once on the host from the layers' shapes and pointers) maps every workgroup of ONE launch to
// (layer, block index inside the layer); the device code of a workgroup is the single-layer kernel body of
// bcq_stream_kernels.h, so results are bit-identical to the layer-by-layer calls on the same kernels.
// The layers of a batch must be independent of each other (the scale gradients of all layers after a backward pass,
// the projections of one block that share an input, a stack of layers for independent requests, ...).
#include "../../include/bcq.h"

#include "bcq_stream_kernels.h"

#include <algorithm>
#include <string.h>
#include <vector>

namespace bcq {

// ---- the plan ("table"): position independent bytes, identical on the host and in device memory -------------------
constexpr uint32_t kBatchMagic = 0x42435142u;  // "BQCB"
constexpr uint32_t kBatchVersion = 1;
// Main-kernel forms.  Up to 8 tokens (one operand half): BATCH_MAIN_TILE, written for batches of small layers (below).
// 9 .. 16 tokens: the single-layer bodies, BATCH_MAIN_LDS (shared activations) / BATCH_MAIN_WAVE (per-wave kernel).
enum { BATCH_MAIN_LDS = 0, BATCH_MAIN_WAVE = 1, BATCH_MAIN_TILE = 2 };

struct BatchHeader {  // 128 bytes
    uint32_t magic, version;
    int32_t op, q, q_used, T, halves, count;
    float scale;
    uint32_t pre_blocks, pre_sets;
    uint32_t main_blocks[2];     // workgroups of the launch of the LDS / WAVE form (0 = none)
    uint32_t tile_blocks;        // workgroups (= pieces) of the TILE form (0 = none)
    // 56 bytes so far
    uint64_t layers_off, pre_map_off, main_map_off[2];
    uint64_t table_bytes, workspace_bytes;
    uint64_t plane_bytes;        // sum of q N K / 8 over the layers (for reporting)
    uint64_t tile_map_off;       // BatchPiece[tile_blocks]
    uint64_t part_off;           // workspace offset of the partial sums of the TILE form
};
static_assert(sizeof(BatchHeader) == 128, "table header layout");

struct BatchLayerDev {  // 128 bytes; what the kernel bodies need of one layer
    const uint32_t* planes;   // canonical planes (forward, scale gradient) or the transposed twin (input gradient)
    const float* alpha;       // forward: epilogue scales; input gradient: folded into the re-coded activations
    const bf16_t* act;        // what the pre-kernel re-codes: x (forward, scale gradient) or dy (input gradient)
    const bf16_t* dy;         // scale gradient: dy for the token reduction
    void* out;
    int64_t rows, cw;         // the plane matrix the kernel streams: rows x 32 cw signs
    uint64_t xq_off, sq_off;  // byte offsets of the re-coded activations and their scales in the workspace
    uint64_t xq_plane, sq_plane;  // bytes of one activation set (input gradient: one set per plane)
    int32_t segs_act;         // 512-index segments of the contraction axis (what the pre-kernel writes per set)
    int32_t segs_main;        // segments the main kernel walks (shared input gradient: q * segs_act virtual segments)
    int32_t spp;              // segments per part (shared form) or per wave (per-wave form)
    uint32_t seg_magic;       // ceil(2^32 / segs_act): virtual segment -> plane (LDS form)
    int32_t nrtg;             // TILE form: row-tile groups of the plane matrix
    int32_t pad32;
    uint64_t seg_magic64;     // TILE form: ceil(2^32 / segs_act), up to 2^32
    uint64_t pad[1];
};

struct BatchPiece {  // TILE form: the work of one workgroup
    uint32_t layer;
    uint32_t rtg0, nrtg;   // row-tile groups [rtg0, rtg0 + nrtg) of the layer
    uint32_t part_kib;     // offset of its partial sums in the partial area, in KiB (layers with more than one chunk)
};
static_assert(sizeof(BatchPiece) == 16, "table piece layout");
static_assert(sizeof(BatchLayerDev) == 128, "table layer layout");

// ---- kernels --------------------------------------------------------------------------------------------------------
// A pointer read from the plan is a generic pointer to the compiler, and loads through it become FLAT loads (which
// also count as LDS operations and serialise with them).  All plan pointers are device-memory pointers: the TILE
// kernel casts them to the global address space explicitly.
#define BCQ_GLOBAL __attribute__((address_space(1)))

template <int MODE>
__global__ __launch_bounds__(256) void quant_act_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                const uint2* __restrict__ map,
                                                                unsigned char* __restrict__ ws, int64_t T, int halves) {
    const uint2 m = map[blockIdx.x];
    const BatchLayerDev& L = layers[m.x];
    // contraction length = 32 cw of the plane matrix (K for the canonical planes, N for the twin)
    quant_act_body<MODE>(L.act, L.alpha, T, L.cw * 32, L.segs_act, halves, 1, ws + L.xq_off, ws + L.sq_off,
                         (size_t)L.xq_plane, (size_t)L.sq_plane, 1, m.y, blockIdx.y);
}

// Shared-activation form (8 row tiles per workgroup, one part of the contraction axis, guarded loop).
template <int MODE, int QP, bool TWO>
__global__ __launch_bounds__(512) void stream_lds_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                  const uint2* __restrict__ map,
                                                                  const unsigned char* __restrict__ ws, int64_t T,
                                                                  int q_used, float scale) {
    const uint2 m = map[blockIdx.x];
    const BatchLayerDev& L = layers[m.x];
    stream_lds_body<MODE, QP, TWO, false, 1, false, false>(L.planes, ws + L.xq_off, ws + L.sq_off, L.alpha, L.dy, L.out, T,
                                                           L.rows, L.cw, q_used, scale, L.spp, L.segs_main, 1, 1,
                                                           (int64_t)L.xq_plane, (int64_t)L.sq_plane, L.seg_magic,
                                                           L.segs_act, m.y, 0);
}

// Per-wave form of the input gradient (twins whose contraction length is no multiple of 512): 4 waves split the
// segments of one 16-row tile.
template <int QP, bool TWO>
__global__ __launch_bounds__(256) void stream_dx_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                 const uint2* __restrict__ map,
                                                                 const unsigned char* __restrict__ ws, int64_t T,
                                                                 int q_used) {
    const uint2 m = map[blockIdx.x];
    const BatchLayerDev& L = layers[m.x];
    stream_body<STREAM_DX, 1, QP, TWO, true, false, false>(L.planes, ws + L.xq_off, ws + L.sq_off, L.alpha, nullptr, L.out, T, L.rows, L.cw, q_used, 1.f, L.spp, L.segs_main,
                                                           (size_t)L.xq_plane, (size_t)L.sq_plane, 127, 1, 1, 0, m.y, 0);
}

constexpr int kWaveFormWaves = 4;

// ---------------------------------------------------------------------------------------------------------------------
// TILE form: the main kernel for batches at up to 8 tokens (both FP8 terms of a token sit in one instruction).
// Written for many small layers rather than one large one:
//   * A workgroup (4 waves) owns a PIECE: a run of row-tile groups of one layer.  It copies the layer's re-coded
//     activations into LDS once per piece (in chunks of 8 segments = 66 KiB; most layers are one chunk), two
//     workgroups fit a compute unit, and between the chunk copies the waves run free of each other: no barrier in
//     the streaming loop, every wave walks its own row-tile groups (wave w takes group w, w + 4, ...).
//   * A wave multiplies PR = QP * RT "plane rows" per segment with one read of the activation operand from LDS:
//     QP planes of RT row tiles (q = 1: four row tiles; q = 2: two; q = 3, 4: one), so the LDS traffic per plane byte
//     does not grow when there are few planes.  The input gradient is one virtual plane over q * segs_act virtual
//     segments of the transposed twin (segment v: plane v / segs_act, its own activation set), i.e. QP = 1, RT = 4.
//   * While a wave multiplies segment s of one row-tile group, the plane words of segment s of its NEXT group are
//     already requested into the register slot that segment just freed: a whole group (up to 8 x PR KiB) in flight.
//   * Sign expansion with ONE operation per operand register: (word << s) | 0x77777777 turns bit b into the FP4 code
//     0x7 | b << 3 = -6 (b = 1, i.e. +1) or +6 (b = 0, i.e. -1); the common factor -1/6 is applied in the epilogue.
//   * Layers with more than 8 segments: the accumulators of a group are carried from chunk to chunk through a
//     wave-private slot of global memory (1 KiB per row tile, written and read back by the same lane).
constexpr int TILE_WAVES = 4;
constexpr int TILE_CSEG = 8;
constexpr int TILE_XB = TILE_CSEG * 4 * QBLK, TILE_SB = TILE_CSEG * QSCL, TILE_LDS = TILE_XB + TILE_SB;

template <int MODE, int QP, int RT>
__global__ __launch_bounds__(256, 2) void stream_tile_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                   const BatchPiece* __restrict__ pieces,
                                                                   const unsigned char* __restrict__ ws,
                                                                   float* partials, int T, float scale) {
    constexpr bool DX = (MODE == STREAM_DX), DA = (MODE == STREAM_DALPHA);
    constexpr int PR = QP * RT;
    static_assert(!DX || QP == 1, "input gradient: one virtual plane");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char* const xb = lds;
    unsigned char* const sb = lds + TILE_XB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, rl = lane & 15, g = lane >> 4;
    const BatchPiece P = pieces[blockIdx.x];
    const BatchLayerDev& L = layers[P.layer];
    const int64_t rows = L.rows;
    const uint32_t cw = (uint32_t)L.cw;
    const int segs = L.segs_main, segs_n = L.segs_act;
    const uint64_t magic = L.seg_magic64;
    const int64_t plane_stride = rows * (int64_t)cw;
    BCQ_GLOBAL const uint32_t* const planes = (BCQ_GLOBAL const uint32_t*)L.planes;
    BCQ_GLOBAL const float* const alpha = (BCQ_GLOBAL const float*)L.alpha;
    BCQ_GLOBAL const bf16_t* const dy = (BCQ_GLOBAL const bf16_t*)L.dy;
    BCQ_GLOBAL void* const outp = (BCQ_GLOBAL void*)L.out;
    const int tcol = rl & 7;  // columns t and t + 8 carry the two terms of token t
    const bool tok_live = tcol < T;
    const int tok = tok_live ? tcol : T - 1;
    const int nchunks = (segs + TILE_CSEG - 1) / TILE_CSEG;
    const int nk = ((int)P.nrtg > wave) ? ((int)P.nrtg - wave + TILE_WAVES - 1) / TILE_WAVES : 0;
    const unsigned char* const xq = ws + L.xq_off;
    const unsigned char* const sq = ws + L.sq_off;
    constexpr float FIX = -1.f / 6.f;
    const uint32_t lane16 = (uint32_t)lane * 16u;

    uint32_t bits[TILE_CSEG][PR][4];
    auto row_offsets = [&](int rtg, uint32_t (&ro)[RT]) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            int64_t row = ((int64_t)rtg * RT + r) * 16 + rl;
            row = row < rows ? row : rows - 1;  // rows beyond the matrix give outputs that are never stored
            ro[r] = (uint32_t)(row * (int64_t)cw);
        }
    };
    auto load_bits = [&](int slot, const uint32_t (&ro)[RT], int vseg) {
        int pl = 0, sg = vseg;
        if (DX) {
            pl = (int)(((uint64_t)(uint32_t)vseg * magic) >> 32);
            sg = vseg - pl * segs_n;
        }
        uint32_t w0 = (uint32_t)sg * 16u + 4u * (uint32_t)g;
        w0 = w0 < cw - 4u ? w0 : cw - 4u;  // a segment that reaches beyond the row is shifted back inside it: the words
                                            // it re-reads meet zero activations
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int i = 0; i < QP; ++i) {
                const q_u32x4 v4 = *(BCQ_GLOBAL const q_u32x4*)(planes + (int64_t)(DX ? pl : i) * plane_stride + (ro[r] + w0));
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) bits[slot][r * QP + i][jj] = v4[jj];
            }
    };

    for (int c = 0; c < nchunks; ++c) {
        const int seg0 = c * TILE_CSEG;
        const int nseg = (segs - seg0) < TILE_CSEG ? (segs - seg0) : TILE_CSEG;
        uint32_t ro_next[RT];
        // plane words of this wave's first group: requested before the chunk copy, in flight during it
        if (nk > 0) {
            row_offsets((int)P.rtg0 + wave, ro_next);
#pragma unroll
            for (int s = 0; s < TILE_CSEG; ++s)
                if (s < nseg) load_bits(s, ro_next, seg0 + s);
        }
        // chunk copy: nseg operand blocks of 8 KiB + nseg x 256 B of scales, global -> registers -> LDS, four segments
        // (eight 4 KiB units of 256 threads x 16 B) at a time
        {
            const q_u32x4* src = reinterpret_cast<const q_u32x4*>(xq + (size_t)seg0 * (4 * QBLK)) + tid;
            q_u32x4* dst = reinterpret_cast<q_u32x4*>(xb) + tid;
            const int nx = nseg * 2;
            q_u32x4 st[8], sts = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int it = 0; it < 8; ++it)
                if (it < nx) st[it] = src[it * 256];
            if (tid < nseg * 16) sts = reinterpret_cast<const q_u32x4*>(sq + (size_t)seg0 * QSCL)[tid];
            __syncthreads();  // every wave is done reading the previous chunk
#pragma unroll
            for (int it = 0; it < 8; ++it)
                if (it < nx) dst[it * 256] = st[it];
            if (tid < nseg * 16) reinterpret_cast<q_u32x4*>(sb)[tid] = sts;
            if (nx > 8) {  // uniform
#pragma unroll
                for (int it = 0; it < 8; ++it)
                    if (8 + it < nx) st[it] = src[(8 + it) * 256];
#pragma unroll
                for (int it = 0; it < 8; ++it)
                    if (8 + it < nx) dst[(8 + it) * 256] = st[it];
            }
            __syncthreads();
        }
        for (int k = 0; k < nk; ++k) {
            const int rtg = (int)P.rtg0 + wave + TILE_WAVES * k;
            const bool more = (k + 1 < nk);
            if (more) row_offsets(rtg + TILE_WAVES, ro_next);
            // epilogue operands of this group, requested before its multiplications
            q_f32x4 ep[RT][DA ? 1 : QP];
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int64_t n0 = ((int64_t)rtg * RT + r) * 16 + 4 * g;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    int64_t n = n0 + v;
                    const bool n_live = n < rows;
                    n = n_live ? n : rows - 1;
                    if (DA) {
                        ep[r][0][v] = (tok_live && n_live)
                                          ? bf16_to_f32(dy[(int64_t)tok * rows + n]) : 0.f;
                    } else if (DX) {
                        ep[r][0][v] = FIX;
                    } else {
#pragma unroll
                        for (int i = 0; i < QP; ++i) ep[r][i][v] = alpha[(int64_t)i * rows + n] * FIX;
                    }
                }
            }
            q_f32x4 acc[RT][QP];
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int i = 0; i < QP; ++i) acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < TILE_CSEG; ++s) {
                if (s < nseg) {  // uniform
                    asm volatile("" ::: "memory");  // keeps the requests of the previous segment above this one
                    const int sv = *reinterpret_cast<const int*>(sb + s * QSCL + lane * 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const unsigned char* bp = xb + (s * 4 + j) * QBLK + lane16;
                        const q_u32x4 lo = *reinterpret_cast<const q_u32x4*>(bp);
                        const q_u32x4 hi = *reinterpret_cast<const q_u32x4*>(bp + QBLK / 2);
                        const q_i32x8 bo = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3],
                                            (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
#pragma unroll
                        for (int r = 0; r < RT; ++r)
#pragma unroll
                            for (int i = 0; i < QP; ++i) {
                                const uint32_t wd = bits[s][r * QP + i][j];
                                q_i32x8 ao;
#pragma unroll
                                for (int sft = 0; sft < 4; ++sft) ao[sft] = (int)((wd << sft) | 0x77777777u);
                                ao[4] = 0;
                                ao[5] = 0;
                                ao[6] = 0;
                                ao[7] = 0;
                                // the instruction picks byte j of the scale register (its op_sel): j must be a constant
                                if (j == 0)
                                    acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo, acc[r][i], 4, 0, 0, 127, 0, sv);
                                else if (j == 1)
                                    acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo, acc[r][i], 4, 0, 0, 127, 1, sv);
                                else if (j == 2)
                                    acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo, acc[r][i], 4, 0, 0, 127, 2, sv);
                                else
                                    acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo, acc[r][i], 4, 0, 0, 127, 3, sv);
                            }
                    }
                    // The matrix instructions are no memory operations: without this pin the optimiser moves them
                    // below the requests that follow, which then need registers of their own and copies afterwards.
#pragma unroll
                    for (int r = 0; r < RT; ++r)
#pragma unroll
                        for (int i = 0; i < QP; ++i) asm volatile("" : "+v"(acc[r][i]));
                    asm volatile("" ::: "memory");
                    if (more) load_bits(s, ro_next, seg0 + s);  // the slot is free: segment s of the next group
                }
            }
            // end of (group, chunk): fold, carry between chunks, store after the last chunk
            const bool last = (c == nchunks - 1);
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int64_t n0 = ((int64_t)rtg * RT + r) * 16 + 4 * g;
                float* const slot = partials + ((size_t)P.part_kib + (size_t)(rtg - (int)P.rtg0) * RT + r) * 256;
                if (DA) {
#pragma unroll
                    for (int o = 0; o < QP; ++o) {
                        q_f32x4 sum;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            // columns t and t + 8 both carry dy of token t: the 16-lane sum adds terms and tokens
                            float x = ep[r][0][v] * acc[r][o][v];
                            x += __shfl_xor(x, 1);
                            x += __shfl_xor(x, 2);
                            x += __shfl_xor(x, 4);
                            x += __shfl_xor(x, 8);
                            sum[v] = x;
                        }
                        if (rl == 0) {
                            q_f32x4* ps = reinterpret_cast<q_f32x4*>(slot + (o * 4 + g) * 4);
                            if (nchunks > 1) {
                                if (c > 0) sum += *ps;
                                if (!last) *ps = sum;
                            }
                            if (last) {
                                BCQ_GLOBAL float* out = (BCQ_GLOBAL float*)outp;
#pragma unroll
                                for (int v = 0; v < 4; ++v)
                                    if (n0 + v < rows) out[(int64_t)o * rows + n0 + v] = sum[v] * (scale * FIX);
                            }
                        }
                    }
                } else {
                    q_f32x4 val = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < QP; ++i)
#pragma unroll
                        for (int v = 0; v < 4; ++v) val[v] += ep[r][i][v] * acc[r][i][v];
#pragma unroll
                    for (int v = 0; v < 4; ++v) val[v] += __shfl_xor(val[v], 8);  // second term's column onto the first's
                    q_f32x4* ps = reinterpret_cast<q_f32x4*>(slot + lane * 4);
                    if (nchunks > 1) {
                        if (c > 0) val += *ps;
                        if (!last) *ps = val;
                    }
                    if (last && tok_live && rl < 8) {
                        BCQ_GLOBAL bf16_t* o = (BCQ_GLOBAL bf16_t*)outp;
                        if (n0 + 3 < rows && (rows & 3) == 0) {
                            q_u32x2 pk;
                            pk[0] = q_pack_bf16x2(val[0], val[1]);
                            pk[1] = q_pack_bf16x2(val[2], val[3]);
                            *(BCQ_GLOBAL q_u32x2*)(o + (int64_t)tok * rows + n0) = pk;
                        } else {
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                if (n0 + v < rows) o[(int64_t)tok * rows + n0 + v] = f32_to_bf16(val[v]);
                        }
                    }
                }
            }
        }
    }
}

// ---- host: sizes and plan ---------------------------------------------------------------------------------------------
struct BatchShape {  // per layer, derived from (op, T, N, K, q, q_used)
    int64_t rows, cw;
    int32_t segs_act, segs_main, spp;
    int form;
    uint32_t main_blocks, sets;
    size_t xq_bytes, sq_bytes;
    // TILE form
    int32_t rt_per_group, nrtg, piece_rtg;  // row tiles per group; groups of the layer; groups per piece
    bool multi_chunk;
};

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// planes a wave multiplies per activation read in the TILE form, and the row tiles it then takes at once
static inline int tile_qp(int op, int q_used) { return op == BCQ_OP_BWD_INPUT ? 1 : q_used; }
static inline int tile_rt(int qp) { return qp == 1 ? 4 : (qp == 2 ? 2 : 1); }

// Work of one TILE-form workgroup, in units of (row-tile group x segment).  Small enough that the launch ends without
// a long tail (the pieces are started longest first), large enough that the chunk copies (one per piece and chunk,
// 8 KiB per segment) stay a small part of the plane bytes; layers with several chunks get longer pieces because every
// chunk of a piece costs a copy with a barrier on either side.
constexpr int kTileUnitsPerPiece = 96;
constexpr int kTileUnitsPerPieceMulti = 320;

static BatchShape batch_shape(int op, int64_t T, int64_t N, int64_t K, int q, int q_used) {
    BatchShape s = {};
    const bool dx = (op == BCQ_OP_BWD_INPUT);
    s.rows = dx ? K : N;
    s.cw = (dx ? N : K) / 32;
    s.segs_act = (int32_t)((s.cw + 15) / 16);
    const int halves = T <= 8 ? 1 : 2;
    s.sets = dx ? (uint32_t)q : 1u;
    s.xq_bytes = (size_t)s.segs_act * 4 * halves * QBLK;
    s.sq_bytes = (size_t)s.segs_act * halves * QSCL;
    const int64_t rt = (s.rows + 15) / 16;
    if (halves == 1) {
        s.form = BATCH_MAIN_TILE;
        s.segs_main = dx ? q * s.segs_act : s.segs_act;
        s.rt_per_group = tile_rt(tile_qp(op, q_used));
        s.nrtg = (int32_t)((rt + s.rt_per_group - 1) / s.rt_per_group);
        s.multi_chunk = s.segs_main > TILE_CSEG;
        const int target = s.multi_chunk ? kTileUnitsPerPieceMulti : kTileUnitsPerPiece;
        int per = (target + s.segs_main - 1) / s.segs_main;
        per = (per + TILE_WAVES - 1) / TILE_WAVES * TILE_WAVES;  // whole rounds of the four waves
        s.piece_rtg = per < TILE_WAVES ? TILE_WAVES : per;
        s.main_blocks = (uint32_t)((s.nrtg + s.piece_rtg - 1) / s.piece_rtg);
        return s;
    }
    // shared-activation form; the input gradient needs whole segments for it, and at least two per plane (the
    // multiply-shift that splits a virtual segment into plane and segment has no 32-bit constant for a divisor of 1)
    if (!dx || (s.cw % 16 == 0 && s.segs_act >= 2)) {
        s.form = BATCH_MAIN_LDS;
        s.segs_main = dx ? q * s.segs_act : s.segs_act;
        s.spp = s.segs_main;
        s.main_blocks = (uint32_t)((rt + 7) / 8);
    } else {
        s.form = BATCH_MAIN_WAVE;
        s.segs_main = s.segs_act;
        s.spp = (s.segs_act + kWaveFormWaves - 1) / kWaveFormWaves;
        s.main_blocks = (uint32_t)rt;
    }
    return s;
}

struct BatchTotals {
    uint64_t pre_blocks = 0, main_blocks[3] = {0, 0, 0};
    uint64_t part_kib = 0;  // partial sums of the TILE form: 1 KiB per row tile of every layer with several chunks
    size_t table_bytes = 0, act_bytes = 0, workspace_bytes = 0;
    uint64_t plane_bytes = 0;
};

static BatchTotals batch_totals(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_used) {
    BatchTotals t;
    for (int64_t l = 0; l < count; ++l) {
        const BatchShape s = batch_shape(op, T, layers[l].N, layers[l].K, q, q_used);
        t.pre_blocks += (uint64_t)s.segs_act;
        t.main_blocks[s.form] += s.main_blocks;
        if (s.form == BATCH_MAIN_TILE && s.multi_chunk) t.part_kib += (uint64_t)s.nrtg * s.rt_per_group;
        t.act_bytes += align_up(s.sets * s.xq_bytes, 256) + align_up(s.sets * s.sq_bytes, 256);
        t.plane_bytes += (uint64_t)q * (uint64_t)layers[l].N * (uint64_t)layers[l].K / 8;
    }
    t.workspace_bytes = t.act_bytes + (size_t)t.part_kib * 1024;
    t.table_bytes = sizeof(BatchHeader) + (size_t)count * sizeof(BatchLayerDev) +
                    (size_t)(t.pre_blocks + t.main_blocks[0] + t.main_blocks[1]) * sizeof(uint2) +
                    (size_t)t.main_blocks[2] * sizeof(BatchPiece);
    t.table_bytes = align_up(t.table_bytes, 256);
    return t;
}

static bool totals_fit(const BatchTotals& t) {
    return t.pre_blocks <= 0x7FFFFFFFull && t.main_blocks[0] <= 0x7FFFFFFFull && t.main_blocks[1] <= 0x7FFFFFFFull &&
           t.main_blocks[2] <= 0x7FFFFFFFull && t.part_kib <= 0x7FFFFFFFull;
}

static bcq_status batch_check(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                              int dtype, bool pointers) {
    using namespace host;
    if (!layers) return BCQ_ERR_NULL;
    if (op != BCQ_OP_FWD && op != BCQ_OP_BWD_INPUT && op != BCQ_OP_BWD_ALPHA) return BCQ_ERR_DTYPE;
    if (count < 1 || count > BCQ_BATCH_MAX_LAYERS || T < 1 || T > BCQ_BATCH_MAX_TOKENS || q < 1 || q > BCQ_BATCH_MAX_Q)
        return BCQ_ERR_SHAPE;
    if (op == BCQ_OP_BWD_ALPHA && (q_train < 1 || q_train > q)) return BCQ_ERR_SHAPE;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        if (!shape_ok(T, b.N, b.K, q)) return BCQ_ERR_SHAPE;
        // 16-byte plane loads: the streamed plane matrix needs a multiple of 4 words per row
        if ((op == BCQ_OP_BWD_INPUT ? b.N : b.K) % 128 != 0) return BCQ_ERR_SHAPE;
    }
    if (dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (!pointers) return BCQ_OK;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        const void* need[4] = {nullptr, nullptr, nullptr, nullptr};
        if (op == BCQ_OP_FWD) { need[0] = b.packed; need[1] = b.alpha; need[2] = b.x; need[3] = b.y; }
        if (op == BCQ_OP_BWD_INPUT) { need[0] = b.packed_t; need[1] = b.alpha; need[2] = b.dy; need[3] = b.dx; }
        if (op == BCQ_OP_BWD_ALPHA) { need[0] = b.packed; need[1] = b.x; need[2] = b.dy; need[3] = b.dalpha; }
        for (const void* p : need)
            if (!p) return BCQ_ERR_NULL;
        for (const void* p : need)
            if (misaligned(p)) return BCQ_ERR_ALIGN;
    }
    return BCQ_OK;
}

template <int MODE>
static hipError_t launch_pre(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    hipLaunchKernelGGL((quant_act_batched_kernel<MODE>), dim3(h.pre_blocks, h.pre_sets), dim3(256), 0, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const uint2*>(dev + h.pre_map_off), ws, (int64_t)h.T, h.halves);
    return hipGetLastError();
}

template <int MODE, int QP, bool TWO>
static hipError_t launch_main_lds_cfg(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws,
                                      int q_used, hipStream_t st) {
    constexpr int H = TWO ? 2 : 1;
    constexpr int LDS_B = 2 * LCS * H * (4 * QBLK + QSCL);
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)stream_lds_batched_kernel<MODE, QP, TWO>, LDS_B);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((stream_lds_batched_kernel<MODE, QP, TWO>), dim3(h.main_blocks[BATCH_MAIN_LDS]), dim3(512), LDS_B, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const uint2*>(dev + h.main_map_off[BATCH_MAIN_LDS]), ws, (int64_t)h.T, q_used,
                       h.scale);
    return hipGetLastError();
}

// the LDS / WAVE forms serve 9 .. 16 tokens only (two operand halves)
template <int MODE>
static hipError_t launch_main_lds(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    if constexpr (MODE == STREAM_DX) {  // one virtual plane
        return launch_main_lds_cfg<MODE, 1, true>(h, dev, ws, 1, st);
    } else {
        switch (h.q_used) {
            case 1: return launch_main_lds_cfg<MODE, 1, true>(h, dev, ws, h.q_used, st);
            case 2: return launch_main_lds_cfg<MODE, 2, true>(h, dev, ws, h.q_used, st);
            case 3: return launch_main_lds_cfg<MODE, 3, true>(h, dev, ws, h.q_used, st);
            default: return launch_main_lds_cfg<MODE, 4, true>(h, dev, ws, h.q_used, st);
        }
    }
}

template <int QP>
static hipError_t launch_main_wave_cfg(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws,
                                       hipStream_t st) {
    hipLaunchKernelGGL((stream_dx_batched_kernel<QP, true>), dim3(h.main_blocks[BATCH_MAIN_WAVE]),
                       dim3(64 * kWaveFormWaves), kWaveFormWaves * 1024, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const uint2*>(dev + h.main_map_off[BATCH_MAIN_WAVE]), ws, (int64_t)h.T, h.q_used);
    return hipGetLastError();
}

static hipError_t launch_main_wave(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    switch (h.q_used) {
        case 1: return launch_main_wave_cfg<1>(h, dev, ws, st);
        case 2: return launch_main_wave_cfg<2>(h, dev, ws, st);
        case 3: return launch_main_wave_cfg<3>(h, dev, ws, st);
        default: return launch_main_wave_cfg<4>(h, dev, ws, st);
    }
}

template <int MODE, int QP, int RT>
static hipError_t launch_main_tile_cfg(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)stream_tile_batched_kernel<MODE, QP, RT>, TILE_LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((stream_tile_batched_kernel<MODE, QP, RT>), dim3(h.tile_blocks), dim3(64 * TILE_WAVES), TILE_LDS, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const BatchPiece*>(dev + h.tile_map_off), ws,
                       reinterpret_cast<float*>(ws + h.part_off), h.T, h.scale);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_main_tile(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    if constexpr (MODE == STREAM_DX) {
        return launch_main_tile_cfg<MODE, 1, 4>(h, dev, ws, st);
    } else {
        switch (h.q_used) {
            case 1: return launch_main_tile_cfg<MODE, 1, 4>(h, dev, ws, st);
            case 2: return launch_main_tile_cfg<MODE, 2, 2>(h, dev, ws, st);
            case 3: return launch_main_tile_cfg<MODE, 3, 1>(h, dev, ws, st);
            default: return launch_main_tile_cfg<MODE, 4, 1>(h, dev, ws, st);
        }
    }
}

template <int MODE>
static hipError_t run_batch(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    hipError_t e = launch_pre<MODE>(h, dev, ws, st);
    if (e == hipSuccess && h.tile_blocks) e = launch_main_tile<MODE>(h, dev, ws, st);
    if (e == hipSuccess && h.main_blocks[BATCH_MAIN_LDS]) e = launch_main_lds<MODE>(h, dev, ws, st);
    if constexpr (MODE == STREAM_DX) {
        if (e == hipSuccess && h.main_blocks[BATCH_MAIN_WAVE]) e = launch_main_wave(h, dev, ws, st);
    }
    return e;
}

}  // namespace bcq

extern "C" {

bcq_status bcq_batch_sizes(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                           int dtype, size_t* table_bytes, size_t* workspace_bytes) {
    if (!table_bytes || !workspace_bytes) return BCQ_ERR_NULL;
    const bcq_status s = bcq::batch_check(op, layers, count, T, q, q_train, dtype, false);
    if (s != BCQ_OK) return s;
    const bcq::BatchTotals t = bcq::batch_totals(op, layers, count, T, q, op == BCQ_OP_BWD_ALPHA ? q_train : q);
    if (!bcq::totals_fit(t)) return BCQ_ERR_SHAPE;
    *table_bytes = t.table_bytes;
    *workspace_bytes = t.workspace_bytes;
    return BCQ_OK;
}

bcq_status bcq_batch_plan(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                          float grad_scale, int dtype, void* table_host, size_t table_bytes) {
    using namespace bcq;
    if (!table_host) return BCQ_ERR_NULL;
    bcq_status s = batch_check(op, layers, count, T, q, q_train, dtype, true);
    if (s != BCQ_OK) return s;
    const int q_used = (op == BCQ_OP_BWD_ALPHA) ? q_train : q;
    const BatchTotals t = batch_totals(op, layers, count, T, q, q_used);
    if (!totals_fit(t)) return BCQ_ERR_SHAPE;
    if (table_bytes < t.table_bytes) return BCQ_ERR_WORKSPACE;

    unsigned char* base = static_cast<unsigned char*>(table_host);
    memset(base, 0, t.table_bytes);
    BatchHeader h = {};
    h.magic = kBatchMagic;
    h.version = kBatchVersion;
    h.op = op;
    h.q = q;
    h.q_used = q_used;
    h.T = (int32_t)T;
    h.halves = T <= 8 ? 1 : 2;
    h.count = (int32_t)count;
    h.scale = (op == BCQ_OP_BWD_ALPHA) ? grad_scale : 1.f;
    h.pre_blocks = (uint32_t)t.pre_blocks;
    h.pre_sets = (op == BCQ_OP_BWD_INPUT) ? (uint32_t)q : 1u;
    h.main_blocks[0] = (uint32_t)t.main_blocks[0];
    h.main_blocks[1] = (uint32_t)t.main_blocks[1];
    h.tile_blocks = (uint32_t)t.main_blocks[2];
    h.layers_off = sizeof(BatchHeader);
    h.pre_map_off = h.layers_off + (uint64_t)count * sizeof(BatchLayerDev);
    h.main_map_off[0] = h.pre_map_off + t.pre_blocks * sizeof(uint2);
    h.main_map_off[1] = h.main_map_off[0] + t.main_blocks[0] * sizeof(uint2);
    h.tile_map_off = h.main_map_off[1] + t.main_blocks[1] * sizeof(uint2);
    h.table_bytes = t.table_bytes;
    h.workspace_bytes = t.workspace_bytes;
    h.plane_bytes = t.plane_bytes;
    h.part_off = t.act_bytes;

    BatchLayerDev* dl = reinterpret_cast<BatchLayerDev*>(base + h.layers_off);
    uint2* pre_map = reinterpret_cast<uint2*>(base + h.pre_map_off);
    struct Item { uint32_t layer, bx; int32_t weight; };
    std::vector<Item> items[2];
    struct PieceItem { BatchPiece p; int64_t weight; };
    std::vector<PieceItem> tiles;
    items[0].reserve(t.main_blocks[0]);
    items[1].reserve(t.main_blocks[1]);
    tiles.reserve(t.main_blocks[2]);
    size_t ws_off = 0;
    uint64_t pb = 0, part_kib = 0;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        const BatchShape sh = batch_shape(op, T, b.N, b.K, q, q_used);
        BatchLayerDev d = {};
        d.planes = (op == BCQ_OP_BWD_INPUT) ? b.packed_t : b.packed;
        d.alpha = b.alpha;
        d.act = reinterpret_cast<const bf16_t*>(op == BCQ_OP_BWD_INPUT ? b.dy : b.x);
        d.dy = reinterpret_cast<const bf16_t*>(b.dy);
        d.out = (op == BCQ_OP_FWD) ? b.y : (op == BCQ_OP_BWD_INPUT ? b.dx : (void*)b.dalpha);
        d.rows = sh.rows;
        d.cw = sh.cw;
        d.xq_off = ws_off;
        ws_off += align_up(sh.sets * sh.xq_bytes, 256);
        d.sq_off = ws_off;
        ws_off += align_up(sh.sets * sh.sq_bytes, 256);
        d.xq_plane = sh.xq_bytes;
        d.sq_plane = sh.sq_bytes;
        d.segs_act = sh.segs_act;
        d.segs_main = sh.segs_main;
        d.spp = sh.spp;
        d.seg_magic64 = (((uint64_t)1 << 32) + (uint64_t)sh.segs_act - 1) / (uint64_t)sh.segs_act;
        d.seg_magic = (uint32_t)d.seg_magic64;  // the LDS form is only chosen with segs_act >= 2, where it fits
        d.nrtg = sh.nrtg;
        dl[l] = d;
        for (int32_t sg = 0; sg < sh.segs_act; ++sg) pre_map[pb++] = make_uint2((uint32_t)l, (uint32_t)sg);
        if (sh.form == BATCH_MAIN_TILE) {
            for (int32_t r0 = 0; r0 < sh.nrtg; r0 += sh.piece_rtg) {
                BatchPiece p;
                p.layer = (uint32_t)l;
                p.rtg0 = (uint32_t)r0;
                p.nrtg = (uint32_t)((sh.nrtg - r0) < sh.piece_rtg ? (sh.nrtg - r0) : sh.piece_rtg);
                p.part_kib = 0;
                if (sh.multi_chunk) {
                    p.part_kib = (uint32_t)part_kib;
                    part_kib += (uint64_t)p.nrtg * sh.rt_per_group;
                }
                tiles.push_back(PieceItem{p, (int64_t)p.nrtg * sh.segs_main});
            }
        } else {
            for (uint32_t bx = 0; bx < sh.main_blocks; ++bx) items[sh.form].push_back(Item{(uint32_t)l, bx, sh.segs_main});
        }
    }
    // The hardware starts workgroups in index order as compute units free up: the longest ones go first, so that the
    // launch does not end with a few long workgroups running alone.
    for (int f = 0; f < 2; ++f) {
        std::stable_sort(items[f].begin(), items[f].end(), [](const Item& a, const Item& b2) { return a.weight > b2.weight; });
        uint2* map = reinterpret_cast<uint2*>(base + h.main_map_off[f]);
        for (size_t i = 0; i < items[f].size(); ++i) map[i] = make_uint2(items[f][i].layer, items[f][i].bx);
    }
    std::stable_sort(tiles.begin(), tiles.end(), [](const PieceItem& a, const PieceItem& b2) { return a.weight > b2.weight; });
    BatchPiece* pm = reinterpret_cast<BatchPiece*>(base + h.tile_map_off);
    for (size_t i = 0; i < tiles.size(); ++i) pm[i] = tiles[i].p;
    memcpy(base, &h, sizeof(h));
    return BCQ_OK;
}

bcq_status bcq_linear_batched(const void* table_host, const void* table_device, size_t table_bytes, void* workspace,
                              size_t workspace_bytes, void* stream) {
    using namespace bcq;
    if (!table_host || !table_device || !workspace) return BCQ_ERR_NULL;
    if (table_bytes < sizeof(BatchHeader)) return BCQ_ERR_WORKSPACE;
    BatchHeader h;
    memcpy(&h, table_host, sizeof(h));
    if (h.magic != kBatchMagic || h.version != kBatchVersion) return BCQ_ERR_DTYPE;  // not a plan of this library
    if (h.table_bytes > table_bytes) return BCQ_ERR_WORKSPACE;
    if (host::misaligned(table_device) || host::misaligned(workspace)) return BCQ_ERR_ALIGN;
    if (workspace_bytes < h.workspace_bytes) return BCQ_ERR_WORKSPACE;
    if (!host::device_ok()) return BCQ_ERR_DEVICE;
    hipStream_t st = (hipStream_t)stream;
    const unsigned char* dev = static_cast<const unsigned char*>(table_device);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    hipError_t e = hipSuccess;
    switch (h.op) {
        case BCQ_OP_FWD: e = run_batch<STREAM_FWD>(h, dev, ws, st); break;
        case BCQ_OP_BWD_ALPHA: e = run_batch<STREAM_DALPHA>(h, dev, ws, st); break;
        case BCQ_OP_BWD_INPUT: e = run_batch<STREAM_DX>(h, dev, ws, st); break;
        default: return BCQ_ERR_DTYPE;
    }
    return e == hipSuccess ? BCQ_OK : BCQ_ERR_DEVICE;
}

}  // extern "C"
