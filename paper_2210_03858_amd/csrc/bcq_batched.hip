// Batched small-token calls: the forward (Eq. 2), the input gradient (Eq. 3) or the scale gradient (Eq. 4) of MANY
// independent layers in two launches (one activation re-coding pre-kernel + one streaming kernel for the whole batch).
//
// Why: a decoder layer of the paper's models holds 0.2 - 13 MB of sign planes, i.e. 0.03 - 1.6 us of HBM time, while a
// launch plus its first memory round trip costs 4 - 11 us.  Called layer by layer the small-token regime (Section 3:
// small-batch inference is memory-bound; Section 6 "Inference Speed") is therefore bound by launches, not by bytes.
// Here a plan (built once on the host from the layers' shapes and pointers) cuts all layers into PIECES, one per
// workgroup of ONE launch.  The layers of a batch must be independent of each other (the scale gradients of all
// layers after a backward pass, the projections of one block that share an input, a stack of layers for independent
// requests, ...).
//
// The planes are read in the DECODE layout (bcq_pack_decode): [row tile][segment][plane][64 lanes][4 words], so that
// everything a wave needs for one (row tile, segment) is one contiguous run of q KiB and a wave walks through memory
// in address order.  Measured on this part with load-only kernels over 550 MB: such a stream reaches 5.9 TB/s at any
// number of requests in flight, while the canonical layout (16 rows x 64 B per request, one region per plane) gives
// 4.3 - 4.7 TB/s with four planes and falls with every further request in flight.
#include "../../include/bcq.h"

#include "bcq_stream_kernels.h"

#include <algorithm>
#include <functional>
#include <string.h>
#include <vector>

namespace bcq {

// ---- the plan ("table"): position independent bytes, identical on the host and in device memory -------------------
constexpr uint32_t kBatchMagic = 0x42435142u;  // "BQCB"
constexpr uint32_t kBatchVersion = 2;

struct BatchHeader {  // 128 bytes
    uint32_t magic, version;
    int32_t op, q, q_used, T, halves, count;
    float scale;
    uint32_t pre_blocks, pre_sets;   // grid of the pre-kernel: (segments of all layers, activation sets per layer)
    uint32_t tile_blocks;            // workgroups (= pieces) of the main kernel
    uint32_t pad0[2];
    uint64_t layers_off, pre_map_off, tile_map_off;
    uint64_t table_bytes, workspace_bytes;
    uint64_t plane_bytes;            // sum of q N K / 8 over the layers (for reporting)
    uint64_t pad1[3];
};
static_assert(sizeof(BatchHeader) == 128, "table header layout");

struct BatchLayerDev {  // 128 bytes; what the kernels need of one layer
    const uint32_t* planes;   // decode layout of the canonical planes (forward, scale gradient) or of the twin (input gradient)
    const float* alpha;       // forward: epilogue scales; input gradient: folded into the re-coded activations
    const bf16_t* act;        // what the pre-kernel re-codes: x (forward, scale gradient) or dy (input gradient)
    const bf16_t* dy;         // scale gradient: dy for the token reduction
    void* out;
    int64_t rows, cw;         // the plane matrix the kernel streams: rows x 32 cw signs (cw: real words per row)
    uint64_t xq_off, sq_off;  // byte offsets of the re-coded activations and their scales in the workspace
    uint64_t xq_plane, sq_plane;  // byte offset from one activation set to the next
    int32_t segs_act;         // 512-index segments of the contraction axis
    int32_t segs_main;        // segments the main kernel walks (input gradient: q * segs_act virtual segments)
    int32_t chunk_segs;       // segments per chunk of activations in LDS
    int32_t q_mem;            // planes per (row tile, segment) in memory (input gradient: 1, the planes are virtual segments)
    int32_t seg_mul;          // pre-kernel: block of (segment, set) at index segment * seg_mul + set
    int32_t nrt;              // row tiles of the plane matrix
    uint64_t pad[2];
};
static_assert(sizeof(BatchLayerDev) == 128, "table layer layout");

struct BatchPiece {  // the work of one workgroup of the main kernel
    uint32_t layer;
    uint32_t rtg0, nrtg;   // row-tile groups [rtg0, rtg0 + nrtg) of the layer
    uint32_t pad;
};
static_assert(sizeof(BatchPiece) == 16, "table piece layout");

// ---- kernels --------------------------------------------------------------------------------------------------------
// A pointer read from the plan is a generic pointer to the compiler, and loads through it become FLAT loads (which
// also count as LDS operations and serialise with them).  All plan pointers are device-memory pointers: the main
// kernel casts them to the global address space explicitly.
#define BCQ_GLOBAL __attribute__((address_space(1)))

// blockIdx.x -> (layer, segment) through `map`; the loads of the map and of the layer record are uniform (scalar).
template <int MODE>
__global__ __launch_bounds__(256) void quant_act_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                const uint2* __restrict__ map,
                                                                unsigned char* __restrict__ ws, int64_t T, int halves) {
    const uint2 m = map[blockIdx.x];
    const BatchLayerDev& L = layers[m.x];
    // contraction length = 32 cw of the plane matrix (K for the canonical planes, N for the twin)
    quant_act_body<MODE>(L.act, L.alpha, T, L.cw * 32, L.segs_act, halves, 1, ws + L.xq_off, ws + L.sq_off,
                         (size_t)L.xq_plane, (size_t)L.sq_plane, 1, L.seg_mul, m.y, blockIdx.y);
}

// ---------------------------------------------------------------------------------------------------------------------
// The main kernel.  Written for many small layers rather than one large one:
//   * A workgroup (8 waves, one per compute unit, 256 registers per lane) owns a PIECE: a run of row-tile groups of
//     one layer.  It copies the layer's re-coded activations into LDS once per piece (in chunks of 132 KiB: 16 segments
//     at up to 8 tokens, where both FP8 terms of a token sit in one instruction, 8 segments at 9 .. 16 tokens; most
//     layers are one chunk), and between the chunk copies the waves run free of each other: no barrier in the
//     streaming loop, every wave walks its own row-tile groups (wave w takes group w, w + 8, ...).  (Two workgroups
//     of 4 waves with chunks of 8 segments were measured 1 - 8 % slower: every piece reads its layer's activation
//     sets, the input gradient's q sets per segment above all, and twice the rows per piece halve that traffic.)
//   * A wave multiplies PR = QP * RT "plane rows" per segment with one read of the activation operand from LDS:
//     QP planes of RT row tiles (q = 1: four row tiles; q = 2: two; q = 3, 4: one), so the LDS traffic per plane byte
//     does not grow when there are few planes.  The input gradient is one virtual plane over q * segs_act virtual
//     segments of the transposed twin (virtual segment v = segment * q + plane, each with its own activation set
//     dy * alpha_plane; in the decode layout of the twin these ARE consecutive KiB), i.e. QP = 1, RT = 4.
//   * A wave's work inside a chunk is a flat sequence of UNITS (group k, segment s).  The plane words of a unit are
//     requested TILE_RING units ahead into a ring of register sets addressed by the unrolled position (three units =
//     12 KiB per wave; two measured equal at up to 8 tokens and slower at 16, four slower at 8).  Every ring step
//     issues exactly one unit's requests, also where there is nothing left to multiply (the sequence is padded to a
//     multiple of the ring length; the padding steps request the first units of the next chunk), so the number of requests between
//     a request and its use is a compile-time constant and the compiler's wait counts are exact: a step waits for
//     its own unit only, never for the younger requests behind it.
//   * For the same reason nothing in the loop reads global memory but the planes: the epilogue operands of the whole
//     piece (alpha, or dy for the scale gradient) and the sums carried from chunk to chunk sit in LDS.
//   * Sign expansion with ONE operation per operand register: (word << s) | 0x77777777 turns bit b into the FP4 code
//     0x7 | b << 3 = -6 (b = 1, i.e. +1) or +6 (b = 0, i.e. -1); the common factor -1/6 is applied in the epilogue.
#ifndef TILE_WAVES_N
#define TILE_WAVES_N 8  // 4 is supported too (then two workgroups per compute unit, chunks of half the size), and 12 with TILE_SETS_N 14
                        // (170 registers per lane: 12 % slower at up to 8 tokens on the 2560-wide stack, 8 % faster on the input gradient at 16)
#endif
constexpr int TILE_WAVES = TILE_WAVES_N;
constexpr int TILE_THREADS = 64 * TILE_WAVES;
#ifndef TILE_RING_N
#define TILE_RING_N 3
#endif
constexpr int TILE_RING = TILE_RING_N;   // units in flight per wave
#ifndef TILE_SETS_N
#define TILE_SETS_N (2 * TILE_WAVES_N)
#endif
constexpr int TILE_SETS = TILE_SETS_N;  // operand-block sets of 8 KiB (+ 256 B of scales) in one chunk
constexpr int TILE_XB = TILE_SETS * 4 * QBLK, TILE_SB = TILE_SETS * QSCL;
constexpr int TILE_AUX = 3072 * TILE_WAVES;  // epilogue operands of the piece + sums carried between chunks
constexpr int TILE_LDS = TILE_XB + TILE_SB + TILE_AUX;
__host__ __device__ constexpr int tile_cseg(int halves) { return TILE_SETS / halves; }  // segments per chunk, at most
// carried sums of one row tile: the live lanes x 16 B (the scale gradient needs QP x 64 B, which is less)
__host__ __device__ constexpr int tile_part_slot(int halves) { return halves == 2 ? 1024 : 512; }

// LDS bytes of the epilogue operands of a piece of `nrtg` groups, and of its carried sums (several chunks only)
__host__ __device__ constexpr int tile_ep_bytes(int mode, int qp, int rt, int nrtg, int halves) {
    return mode == STREAM_DX ? 0 : (mode == STREAM_FWD ? nrtg * rt * 16 * qp * 4 : nrtg * rt * 16 * (8 * halves) * 2);
}
__host__ __device__ constexpr int tile_part_bytes(int rt, int nrtg, int halves) {
    return ((nrtg + TILE_WAVES - 1) / TILE_WAVES) * TILE_WAVES * rt * tile_part_slot(halves);
}

// Moves inside a row of 16 lanes with the data-parallel primitives of the vector ALU (a few cycles; a shuffle through
// the LDS crossbar costs an LDS instruction and its latency).  All patterns used are permutations of the row.
template <int CTRL>
__device__ __forceinline__ float row16_move(float v) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a row, in every lane: neighbours, pairs, mirrored halves of 8, mirrored row
__device__ __forceinline__ float row16_sum(float x) {
    x += row16_move<0xB1>(x);   // quad_perm [1, 0, 3, 2]
    x += row16_move<0x4E>(x);   // quad_perm [2, 3, 0, 1]
    x += row16_move<0x141>(x);  // lane i of each 8 takes lane 7 - i
    x += row16_move<0x140>(x);  // lane i takes lane 15 - i
    return x;
}

template <int MODE, int QP, int RT, bool TWO>
__global__ __launch_bounds__(TILE_THREADS, (TILE_WAVES <= 4 ? 2 : 1)) void stream_tile_batched_kernel(const BatchLayerDev* __restrict__ layers,
                                                                      const BatchPiece* __restrict__ pieces,
                                                                      const unsigned char* __restrict__ ws, int T,
                                                                      float scale) {
    constexpr bool DX = (MODE == STREAM_DX), DA = (MODE == STREAM_DALPHA);
    constexpr int PR = QP * RT, H = TWO ? 2 : 1, TT = 8 * H;
    constexpr int PART_SLOT = tile_part_slot(H);
    static_assert(!DX || QP == 1, "input gradient: one virtual plane");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char* const xb = lds;
    unsigned char* const sb = lds + TILE_XB;
    unsigned char* const aux = lds + TILE_XB + TILE_SB;
    const int tid = threadIdx.x, lane = tid & 63, rl = lane & 15, g = lane >> 4;
    // the wave index as a scalar: everything derived from it (group counts, cursors, loop bounds) then stays in scalar
    // registers and the branches on it are scalar branches instead of execution-mask updates
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const BatchPiece P = pieces[blockIdx.x];
    const BatchLayerDev& L = layers[P.layer];
    const int64_t rows = L.rows;
    const int segs = L.segs_main, cseg = L.chunk_segs, q_mem = L.q_mem, nrt = L.nrt;
    BCQ_GLOBAL const uint32_t* const planes = (BCQ_GLOBAL const uint32_t*)L.planes;
    const int tcol = TWO ? rl : (rl & 7);  // one half: columns t and t + 8 carry the two terms of token t
    const bool tok_live = tcol < T;
    const int tok = tok_live ? tcol : T - 1;
    const int nchunks = (segs + cseg - 1) / cseg;
    const int nk = ((int)P.nrtg > wave) ? ((int)P.nrtg - wave + TILE_WAVES - 1) / TILE_WAVES : 0;
    const int rtg_first = (int)P.rtg0 + wave;
    const unsigned char* const xq = ws + L.xq_off;
    const unsigned char* const sq = ws + L.sq_off;
    constexpr float FIX = -1.f / 6.f;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const int piece_rows = (int)P.nrtg * RT * 16;
    const int64_t piece_row0 = (int64_t)P.rtg0 * RT * 16;
    unsigned char* const part = aux + tile_ep_bytes(MODE, QP, RT, (int)P.nrtg, H);  // this piece's carried sums

    // Epilogue operands of the piece: requested here into registers (up to three 16-byte vectors per thread), written to
    // LDS together with the first chunk of activations, so that all start-up requests of the workgroup are in flight
    // at once (one memory round trip instead of one per loop iteration).
    //   forward: alpha[i][row] * (-1/6) as fp32, [QP][piece_rows]
    //   scale gradient: dy[t][row] as bf16, [TT][piece_rows]; tokens beyond T and rows beyond the matrix as zeros
    constexpr int EPV = 3;
    q_u32x4 epv[EPV];
    const int ep_per = MODE == STREAM_FWD ? piece_rows / 4 : piece_rows / 8;  // vectors per plane / per token
    const int ep_total = DX ? 0 : (MODE == STREAM_FWD ? QP : TT) * ep_per;
    const bool ep_vec = DX || (MODE == STREAM_FWD ? (rows & 3) == 0 : (rows & 7) == 0);  // rows start 16-byte aligned
    if (!DX && ep_vec) {
#pragma unroll
        for (int it = 0; it < EPV; ++it) {
            const int e = tid + it * 64 * TILE_WAVES;
            epv[it] = q_u32x4{0u, 0u, 0u, 0u};
            if (e < ep_total) {
                const int a = e / ep_per, lv = e - a * ep_per;  // plane or token, vector inside its row of the table
                if (MODE == STREAM_FWD) {
                    const int64_t n = piece_row0 + 4 * lv;
                    if (n < rows) epv[it] = *(BCQ_GLOBAL const q_u32x4*)((BCQ_GLOBAL const float*)L.alpha + (int64_t)a * rows + n);
                } else {
                    const int64_t n = piece_row0 + 8 * lv;
                    if (a < T && n < rows) epv[it] = *(BCQ_GLOBAL const q_u32x4*)((BCQ_GLOBAL const bf16_t*)L.dy + (int64_t)a * rows + n);
                }
            }
        }
    }
    auto store_ep = [&]() {
        if (DX) return;
        if (ep_vec) {
#pragma unroll
            for (int it = 0; it < EPV; ++it) {
                const int e = tid + it * 64 * TILE_WAVES;
                if (e < ep_total) {
                    q_u32x4 v = epv[it];
                    if (MODE == STREAM_FWD) {
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = __float_as_uint(__uint_as_float(v[x]) * FIX);
                    }
                    reinterpret_cast<q_u32x4*>(aux)[e] = v;
                }
            }
        } else if (MODE == STREAM_FWD) {  // rows not a multiple of 4: element by element
            BCQ_GLOBAL const float* const alpha = (BCQ_GLOBAL const float*)L.alpha;
            float* dst = reinterpret_cast<float*>(aux);
            for (int e = tid; e < QP * piece_rows; e += 64 * TILE_WAVES) {
                const int i = e / piece_rows, lr = e - i * piece_rows;
                const int64_t n = piece_row0 + lr;
                dst[e] = n < rows ? alpha[(int64_t)i * rows + n] * FIX : 0.f;
            }
        } else {  // rows not a multiple of 8
            BCQ_GLOBAL const bf16_t* const dy = (BCQ_GLOBAL const bf16_t*)L.dy;
            bf16_t* dst = reinterpret_cast<bf16_t*>(aux);
            for (int e = tid; e < TT * piece_rows; e += 64 * TILE_WAVES) {
                const int t = e / piece_rows, lr = e - t * piece_rows;
                const int64_t n = piece_row0 + lr;
                dst[e] = (t < T && n < rows) ? dy[(int64_t)t * rows + n] : (bf16_t)0;
            }
        }
    };

    // ---- the ring of plane words
    uint32_t bits[TILE_RING][PR][4];
    // decode layout: row tile rt, segment vseg, plane i -> 1 KiB at ((rt * segs + vseg) * q_mem + i) KiB, 16 B per lane
    const uint32_t lane4 = (uint32_t)lane * 4u;
    auto load_unit = [&](int slot, int rtg, int vseg) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            int rt = rtg * RT + r;
            rt = rt < nrt ? rt : nrt - 1;  // row tiles beyond the matrix give outputs that are never stored
            BCQ_GLOBAL const uint32_t* const tb = planes + ((int64_t)rt * segs + vseg) * ((int64_t)q_mem * 256);
#pragma unroll
            for (int i = 0; i < QP; ++i) {
                const q_u32x4 v4 = *(BCQ_GLOBAL const q_u32x4*)(tb + i * 256 + lane4);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) bits[slot][r * QP + i][jj] = v4[jj];
            }
        }
    };
    // request cursor: unit (lk, ls) of chunk lc, the next one to be requested; it runs TILE_RING units ahead of the
    // multiplications and crosses into the next chunk on its own
    int lc = 0, lk = 0, ls = 0, lpad = 0;  // lpad: padding steps still to spend at the end of chunk lc
    auto chunk_nseg = [&](int c) { return (segs - c * cseg) < cseg ? (segs - c * cseg) : cseg; };
    auto request_next = [&](int slot) {
        // address of the unit under the cursor; beyond the piece's last unit: that last unit again (unused)
        const int nsg = chunk_nseg(lc);
        load_unit(slot, rtg_first + TILE_WAVES * lk, lc * cseg + ls);
        if (lpad > 0) {  // a padding step of chunk lc: the cursor already points at the next chunk's first unit
            --lpad;
            return;
        }
        // advance
        if (ls + 1 < nsg) {
            ++ls;
        } else if (lk + 1 < nk) {
            ls = 0;
            ++lk;
        } else if (lc + 1 < nchunks) {  // chunk lc is exhausted: spend its padding steps, then go on with chunk lc + 1
            const int n = nk * nsg;
            lpad = ((n + TILE_RING - 1) / TILE_RING) * TILE_RING - n;
            ++lc;
            lk = 0;
            ls = 0;
        }  // else: stay on the piece's last unit
    };
    if (nk > 0) {
#pragma unroll
        for (int d = 0; d < TILE_RING; ++d) request_next(d);
    }

    q_f32x4 acc[RT][QP];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int i = 0; i < QP; ++i) acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};

    for (int c = 0; c < nchunks; ++c) {
        const int seg0 = c * cseg;
        const int nseg = chunk_nseg(c);
        // chunk copy: nseg x H operand-block sets of 8 KiB + nseg x H x 256 B of scales, global -> registers -> LDS; all
        // (up to sixteen) steps of all threads x 16 B are requested before the first is written
        {
            const q_u32x4* src = reinterpret_cast<const q_u32x4*>(xq + (size_t)seg0 * (4 * H * QBLK)) + tid;
            q_u32x4* dst = reinterpret_cast<q_u32x4*>(xb) + tid;
            const int nx = nseg * H * 2;
            constexpr int CPY = (TILE_XB / 16 + TILE_THREADS - 1) / TILE_THREADS;  // copy steps of all threads x 16 B for a full chunk
            q_u32x4 st[CPY], sts = {0u, 0u, 0u, 0u};
            const int nvec = nx * 256;  // 16-byte vectors of this chunk
#pragma unroll
            for (int it = 0; it < CPY; ++it)
                if (tid + it * TILE_THREADS < nvec) st[it] = src[it * TILE_THREADS];
            if (tid < nseg * H * 16) sts = reinterpret_cast<const q_u32x4*>(sq + (size_t)seg0 * (H * QSCL))[tid];
            __syncthreads();  // every wave is done reading the previous chunk
            if (c == 0) store_ep();
#pragma unroll
            for (int it = 0; it < CPY; ++it)
                if (tid + it * TILE_THREADS < nvec) dst[it * TILE_THREADS] = st[it];
            if (tid < nseg * H * 16) reinterpret_cast<q_u32x4*>(sb)[tid] = sts;
            __syncthreads();
        }
        if (nk == 0) continue;  // a wave without groups only helps with the copies
        const int n_units = nk * nseg;
        const bool last = (c == nchunks - 1);
        int ck = 0, cs = 0;  // unit being multiplied
        for (int base = 0; base < n_units; base += TILE_RING) {
#pragma unroll
            for (int d = 0; d < TILE_RING; ++d) {
                asm volatile("" ::: "memory");  // keeps the requests of the previous step above this one
                if (base + d < n_units) {  // uniform; no global memory access inside
                    const uint32_t xo = (uint32_t)cs * (4u * H * QBLK) + lane16;
                    int sv[H];
#pragma unroll
                    for (int h = 0; h < H; ++h) sv[h] = *reinterpret_cast<const int*>(sb + (cs * H + h) * QSCL + lane * 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        q_i32x8 bo[H];
#pragma unroll
                        for (int h = 0; h < H; ++h) {
                            const unsigned char* bp = xb + xo + (j * H + h) * QBLK;
                            const q_u32x4 lo = *reinterpret_cast<const q_u32x4*>(bp);
                            const q_u32x4 hi = *reinterpret_cast<const q_u32x4*>(bp + QBLK / 2);
                            bo[h] = q_i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3],
                                            (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
                        }
#pragma unroll
                        for (int r = 0; r < RT; ++r)
#pragma unroll
                            for (int i = 0; i < QP; ++i) {
                                const uint32_t wd = bits[d][r * QP + i][j];
                                q_i32x8 ao;
#pragma unroll
                                for (int sft = 0; sft < 4; ++sft) ao[sft] = (int)((wd << sft) | 0x77777777u);
                                ao[4] = 0;
                                ao[5] = 0;
                                ao[6] = 0;
                                ao[7] = 0;
#pragma unroll
                                for (int h = 0; h < H; ++h) {
                                    // the instruction picks byte j of the scale register (its op_sel): j must be a constant
                                    if (j == 0)
                                        acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo[h], acc[r][i], 4, 0, 0, 127, 0, sv[h]);
                                    else if (j == 1)
                                        acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo[h], acc[r][i], 4, 0, 0, 127, 1, sv[h]);
                                    else if (j == 2)
                                        acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo[h], acc[r][i], 4, 0, 0, 127, 2, sv[h]);
                                    else
                                        acc[r][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao, bo[h], acc[r][i], 4, 0, 0, 127, 3, sv[h]);
                                }
                            }
                    }
                    if (cs == nseg - 1) {  // uniform: the group's last segment of this chunk
                        const int kl = ck * TILE_WAVES + wave;  // group inside the piece
#pragma unroll
                        for (int r = 0; r < RT; ++r) {
                            const int lr0 = (kl * RT + r) * 16 + 4 * g;  // first of this lane's 4 rows, inside the piece
                            const int64_t n0 = piece_row0 + lr0;
                            unsigned char* const slot = part + (size_t)((ck * TILE_WAVES + wave) * RT + r) * PART_SLOT;
                            if (DA) {
                                const q_u32x2 dyp = *reinterpret_cast<const q_u32x2*>(aux + ((size_t)tcol * piece_rows + lr0) * 2);
                                const float dyv[4] = {__uint_as_float(dyp[0] << 16), __uint_as_float(dyp[0] & 0xFFFF0000u),
                                                      __uint_as_float(dyp[1] << 16), __uint_as_float(dyp[1] & 0xFFFF0000u)};
#pragma unroll
                                for (int o = 0; o < QP; ++o) {
                                    q_f32x4 sum;
#pragma unroll
                                    for (int v = 0; v < 4; ++v) {
                                        // one half: columns t and t + 8 both carry dy of token t; the 16-lane sum adds the
                                        // terms and the tokens
                                        float x = dyv[v] * acc[r][o][v];
                                        x = row16_sum(x);
                                        sum[v] = x;
                                    }
                                    if (rl == 0) {
                                        q_f32x4* ps = reinterpret_cast<q_f32x4*>(slot + (o * 4 + g) * 16);
                                        if (nchunks > 1) {
                                            if (c > 0) sum += *ps;
                                            if (!last) *ps = sum;
                                        }
                                        if (last) {
                                            BCQ_GLOBAL float* out = (BCQ_GLOBAL float*)L.out;
#pragma unroll
                                            for (int v = 0; v < 4; ++v)
                                                if (n0 + v < rows) out[(int64_t)o * rows + n0 + v] = sum[v] * (scale * FIX);
                                        }
                                    }
                                }
                            } else {
                                q_f32x4 val = {0.f, 0.f, 0.f, 0.f};
                                if (DX) {
#pragma unroll
                                    for (int v = 0; v < 4; ++v) val[v] = acc[r][0][v] * FIX;
                                } else {
#pragma unroll
                                    for (int i = 0; i < QP; ++i) {
                                        const q_f32x4 al = *reinterpret_cast<const q_f32x4*>(aux + ((size_t)i * piece_rows + lr0) * 4);
#pragma unroll
                                        for (int v = 0; v < 4; ++v) val[v] += al[v] * acc[r][i][v];
                                    }
                                }
                                if (!TWO) {  // second term's column onto the first's
#pragma unroll
                                    for (int v = 0; v < 4; ++v) val[v] += row16_move<0x128>(val[v]);  // from lane ^ 8
                                }
                                if (TWO || rl < 8) {
                                    q_f32x4* ps = reinterpret_cast<q_f32x4*>(slot + (TWO ? lane : g * 8 + rl) * 16);
                                    if (nchunks > 1) {
                                        if (c > 0) val += *ps;
                                        if (!last) *ps = val;
                                    }
                                    if (last && tok_live) {
                                        BCQ_GLOBAL bf16_t* o = (BCQ_GLOBAL bf16_t*)L.out;
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
#pragma unroll
                        for (int r = 0; r < RT; ++r)
#pragma unroll
                            for (int i = 0; i < QP; ++i) acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
                        cs = 0;
                        ++ck;
                    } else {
                        ++cs;
                    }
                }
                // The matrix instructions are no memory operations: without this pin the optimiser moves them below
                // the requests that follow, which then need registers of their own and copies afterwards.
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int i = 0; i < QP; ++i) asm volatile("" : "+v"(acc[r][i]));
                asm volatile("" ::: "memory");
                request_next(d);  // always: the number of requests between a request and its use is a constant
            }
        }
    }
}

// ---- host: sizes and plan ---------------------------------------------------------------------------------------------
struct BatchShape {  // per layer, derived from (op, T, N, K, q, q_used)
    int64_t rows, cw;
    int32_t segs_act, segs_main, chunk_segs, q_mem, seg_mul, nrt;
    uint32_t sets;
    size_t xq_bytes, sq_bytes;          // all sets
    size_t xq_plane, sq_plane;          // from one set to the next
    int32_t rt_per_group, nrtg, piece_rtg;  // row tiles per group; groups of the layer / per piece
    uint32_t pieces;
};

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// planes a wave multiplies per activation read, and the row tiles it then takes at once
static inline int tile_qp(int op, int q_used) { return op == BCQ_OP_BWD_INPUT ? 1 : q_used; }
// (at 9 .. 16 tokens at most two: the carried sums of a row tile take 1 KiB there, and one round of four groups must
// fit the LDS area)
static inline int tile_rt(int qp, int halves) { return qp == 1 ? (halves == 2 ? 2 : 4) : (qp == 2 ? 2 : 1); }

// Work of one workgroup (a piece), in units of (row-tile group x segment).  The hardware starts the pieces in
// index order as slots free up (one workgroup per compute unit of the 256), the longest first.  The size is chosen
// per batch (choose_piece_units): small enough that the last round of pieces is not half empty, large enough that
// the start-up of a piece (plan look-up, first memory round trip, one activation copy with two barriers per chunk)
// stays a small part of its streaming time.  Layers with several chunks get pieces of three times the size.
constexpr int kTileSlots = 256 * (TILE_WAVES <= 4 ? 2 : 1);
constexpr int kTileStartupUnits = 12;       // start-up of a piece, in units of streaming time (about 4 us)
constexpr int kTileChunkStartupUnits = 7;   // every further chunk: a copy between two barriers
constexpr int kTileMultiFactor = 3;

static BatchShape batch_shape(int op, int64_t T, int64_t N, int64_t K, int q, int q_used, int piece_units) {
    BatchShape s = {};
    const bool dx = (op == BCQ_OP_BWD_INPUT);
    const int halves = T <= 8 ? 1 : 2;
    s.rows = dx ? K : N;
    s.cw = (dx ? N : K) / 32;
    s.segs_act = (int32_t)((s.cw + 15) / 16);
    s.nrt = (int32_t)((s.rows + 15) / 16);
    s.sets = dx ? (uint32_t)q : 1u;
    s.xq_bytes = (size_t)s.sets * s.segs_act * 4 * halves * QBLK;
    s.sq_bytes = (size_t)s.sets * s.segs_act * halves * QSCL;
    if (dx) {  // sets interleaved by segment: virtual segment v = segment * q + plane is block v
        s.xq_plane = (size_t)4 * halves * QBLK;
        s.sq_plane = (size_t)halves * QSCL;
        s.seg_mul = q;
        s.q_mem = 1;
        s.segs_main = q * s.segs_act;
    } else {
        s.xq_plane = s.xq_bytes;
        s.sq_plane = s.sq_bytes;
        s.seg_mul = 1;
        s.q_mem = q;
        s.segs_main = s.segs_act;
    }
    const int qp = tile_qp(op, q_used);
    s.rt_per_group = tile_rt(qp, halves);
    s.nrtg = (s.nrt + s.rt_per_group - 1) / s.rt_per_group;
    const int cseg = tile_cseg(halves);
    const int nch = (s.segs_main + cseg - 1) / cseg;
    s.chunk_segs = (s.segs_main + nch - 1) / nch;  // chunks of about equal length
    const bool multi = nch > 1;
    const int mode = dx ? STREAM_DX : (op == BCQ_OP_FWD ? STREAM_FWD : STREAM_DALPHA);
    const int target = multi ? kTileMultiFactor * piece_units : piece_units;
    int per = (target + s.segs_main - 1) / s.segs_main;
    per = (per + TILE_WAVES - 1) / TILE_WAVES * TILE_WAVES;  // whole rounds of the waves
    if (per < TILE_WAVES) per = TILE_WAVES;
    // the epilogue operands of the piece and, with several chunks, its carried sums must fit their LDS area
    while (per > TILE_WAVES && tile_ep_bytes(mode, qp, s.rt_per_group, per, halves) +
                                       (multi ? tile_part_bytes(s.rt_per_group, per, halves) : 0) > TILE_AUX)
        per -= TILE_WAVES;
    s.piece_rtg = per;
    s.pieces = (uint32_t)((s.nrtg + s.piece_rtg - 1) / s.piece_rtg);
    return s;
}
// one round of four groups always fits (the scale gradient's dy table is the largest epilogue operand)
static_assert(tile_ep_bytes(STREAM_DALPHA, 1, 4, TILE_WAVES, 1) + tile_part_bytes(4, TILE_WAVES, 1) <= TILE_AUX, "");
static_assert(tile_ep_bytes(STREAM_DALPHA, 1, 2, TILE_WAVES, 2) + tile_part_bytes(2, TILE_WAVES, 2) <= TILE_AUX, "");
static_assert(tile_ep_bytes(STREAM_FWD, 4, 1, TILE_WAVES, 2) + tile_part_bytes(1, TILE_WAVES, 2) <= TILE_AUX, "");

// Picks the piece size for a batch: list scheduling (longest piece first, one slot per compute unit) of the pieces every candidate size
// gives, with the start-up costs above; the candidate with the shortest schedule wins.  Pure host arithmetic.
static int choose_piece_units(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_used) {
    int best = 96;
    double best_span = -1.0;
    std::vector<int64_t> costs;
    std::vector<int64_t> slots;
    for (int cand = 48; cand <= 60 * TILE_WAVES; cand += 8) {
        costs.clear();
        for (int64_t l = 0; l < count; ++l) {
            const BatchShape s = batch_shape(op, T, layers[l].N, layers[l].K, q, q_used, cand);
            const int nch = (s.segs_main + s.chunk_segs - 1) / s.chunk_segs;
            const int64_t fixed = kTileStartupUnits + (int64_t)(nch - 1) * kTileChunkStartupUnits;
            for (int32_t r0 = 0; r0 < s.nrtg; r0 += s.piece_rtg) {
                const int32_t n = (s.nrtg - r0) < s.piece_rtg ? (s.nrtg - r0) : s.piece_rtg;
                // the waves take the groups in rounds: a piece lasts as long as its busiest wave
                const int64_t rounds = (n + TILE_WAVES - 1) / TILE_WAVES;
                costs.push_back(rounds * TILE_WAVES * (int64_t)s.segs_main + fixed);
            }
        }
        std::sort(costs.begin(), costs.end(), [](int64_t a, int64_t b) { return a > b; });
        slots.assign(kTileSlots, 0);
        std::make_heap(slots.begin(), slots.end(), std::greater<int64_t>());
        int64_t span = 0;
        for (int64_t c : costs) {
            std::pop_heap(slots.begin(), slots.end(), std::greater<int64_t>());
            slots.back() += c;
            span = slots.back() > span ? slots.back() : span;
            std::push_heap(slots.begin(), slots.end(), std::greater<int64_t>());
        }
        if (best_span < 0 || (double)span < best_span * 0.995) {  // ties go to the smaller size
            best_span = (double)span;
            best = cand;
        }
    }
    return best;
}

struct BatchTotals {
    int piece_units = 96;
    uint64_t pre_blocks = 0, pieces = 0;
    size_t table_bytes = 0, workspace_bytes = 0;
    uint64_t plane_bytes = 0;
};

static BatchTotals batch_totals(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_used) {
    BatchTotals t;
    t.piece_units = choose_piece_units(op, layers, count, T, q, q_used);
    for (int64_t l = 0; l < count; ++l) {
        const BatchShape s = batch_shape(op, T, layers[l].N, layers[l].K, q, q_used, t.piece_units);
        t.pre_blocks += (uint64_t)s.segs_act;
        t.pieces += s.pieces;
        t.workspace_bytes += align_up(s.xq_bytes, 256) + align_up(s.sq_bytes, 256);
        t.plane_bytes += (uint64_t)q * (uint64_t)layers[l].N * (uint64_t)layers[l].K / 8;
    }
    t.table_bytes = sizeof(BatchHeader) + (size_t)count * sizeof(BatchLayerDev) + (size_t)t.pre_blocks * sizeof(uint2) +
                    (size_t)t.pieces * sizeof(BatchPiece);
    t.table_bytes = align_up(t.table_bytes, 256);
    return t;
}

static bool totals_fit(const BatchTotals& t) { return t.pre_blocks <= 0x7FFFFFFFull && t.pieces <= 0x7FFFFFFFull; }

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
        if (op == BCQ_OP_BWD_INPUT && b.N % 32 != 0) return BCQ_ERR_SHAPE;  // the twin packs 32 rows of W per word
    }
    if (dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (!pointers) return BCQ_OK;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        const void* need[4] = {nullptr, nullptr, nullptr, nullptr};
        if (op == BCQ_OP_FWD) { need[0] = b.tiled; need[1] = b.alpha; need[2] = b.x; need[3] = b.y; }
        if (op == BCQ_OP_BWD_INPUT) { need[0] = b.tiled_t; need[1] = b.alpha; need[2] = b.dy; need[3] = b.dx; }
        if (op == BCQ_OP_BWD_ALPHA) { need[0] = b.tiled; need[1] = b.x; need[2] = b.dy; need[3] = b.dalpha; }
        for (const void* p : need)
            if (!p) return BCQ_ERR_NULL;
        for (const void* p : need)
            if (misaligned(p)) return BCQ_ERR_ALIGN;
    }
    return BCQ_OK;
}

template <int MODE>
static hipError_t launch_pre(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    BCQ_LAUNCH((quant_act_batched_kernel<MODE>), dim3(h.pre_blocks, h.pre_sets), dim3(256), 0, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const uint2*>(dev + h.pre_map_off), ws, (int64_t)h.T, h.halves);
    return hipGetLastError();
}

template <int MODE, int QP, int RT, bool TWO>
static hipError_t launch_main_cfg(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)stream_tile_batched_kernel<MODE, QP, RT, TWO>, TILE_LDS);
    if (e != hipSuccess) return e;
    BCQ_LAUNCH((stream_tile_batched_kernel<MODE, QP, RT, TWO>), dim3(h.tile_blocks), dim3(64 * TILE_WAVES), TILE_LDS,
                       st, reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const BatchPiece*>(dev + h.tile_map_off), ws, h.T, h.scale);
    return hipGetLastError();
}

template <int MODE, bool TWO>
static hipError_t launch_main(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    constexpr int RT1 = TWO ? 2 : 4;  // row tiles per group with one plane: as tile_rt
    if constexpr (MODE == STREAM_DX) {
        return launch_main_cfg<MODE, 1, RT1, TWO>(h, dev, ws, st);
    } else {
        switch (h.q_used) {
            case 1: return launch_main_cfg<MODE, 1, RT1, TWO>(h, dev, ws, st);
            case 2: return launch_main_cfg<MODE, 2, 2, TWO>(h, dev, ws, st);
            case 3: return launch_main_cfg<MODE, 3, 1, TWO>(h, dev, ws, st);
            default: return launch_main_cfg<MODE, 4, 1, TWO>(h, dev, ws, st);
        }
    }
}

template <int MODE>
static hipError_t run_batch(const BatchHeader& h, const unsigned char* dev, unsigned char* ws, hipStream_t st) {
    hipError_t e = launch_pre<MODE>(h, dev, ws, st);
    if (e != hipSuccess) return e;
    return h.halves == 2 ? launch_main<MODE, true>(h, dev, ws, st) : launch_main<MODE, false>(h, dev, ws, st);
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
    h.tile_blocks = (uint32_t)t.pieces;
    h.layers_off = sizeof(BatchHeader);
    h.pre_map_off = h.layers_off + (uint64_t)count * sizeof(BatchLayerDev);
    h.tile_map_off = h.pre_map_off + t.pre_blocks * sizeof(uint2);
    h.table_bytes = t.table_bytes;
    h.workspace_bytes = t.workspace_bytes;
    h.plane_bytes = t.plane_bytes;

    BatchLayerDev* dl = reinterpret_cast<BatchLayerDev*>(base + h.layers_off);
    uint2* pre_map = reinterpret_cast<uint2*>(base + h.pre_map_off);
    struct PieceItem { BatchPiece p; int64_t weight; };
    std::vector<PieceItem> tiles;
    tiles.reserve(t.pieces);
    size_t ws_off = 0;
    uint64_t pb = 0;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        const BatchShape sh = batch_shape(op, T, b.N, b.K, q, q_used, t.piece_units);
        BatchLayerDev d = {};
        d.planes = (op == BCQ_OP_BWD_INPUT) ? b.tiled_t : b.tiled;
        d.alpha = b.alpha;
        d.act = reinterpret_cast<const bf16_t*>(op == BCQ_OP_BWD_INPUT ? b.dy : b.x);
        d.dy = reinterpret_cast<const bf16_t*>(b.dy);
        d.out = (op == BCQ_OP_FWD) ? b.y : (op == BCQ_OP_BWD_INPUT ? b.dx : (void*)b.dalpha);
        d.rows = sh.rows;
        d.cw = sh.cw;
        d.xq_off = ws_off;
        ws_off += align_up(sh.xq_bytes, 256);
        d.sq_off = ws_off;
        ws_off += align_up(sh.sq_bytes, 256);
        d.xq_plane = sh.xq_plane;
        d.sq_plane = sh.sq_plane;
        d.segs_act = sh.segs_act;
        d.segs_main = sh.segs_main;
        d.chunk_segs = sh.chunk_segs;
        d.q_mem = sh.q_mem;
        d.seg_mul = sh.seg_mul;
        d.nrt = sh.nrt;
        dl[l] = d;
        for (int32_t sg = 0; sg < sh.segs_act; ++sg) pre_map[pb++] = make_uint2((uint32_t)l, (uint32_t)sg);
        for (int32_t r0 = 0; r0 < sh.nrtg; r0 += sh.piece_rtg) {
            BatchPiece p;
            p.layer = (uint32_t)l;
            p.rtg0 = (uint32_t)r0;
            p.nrtg = (uint32_t)((sh.nrtg - r0) < sh.piece_rtg ? (sh.nrtg - r0) : sh.piece_rtg);
            p.pad = 0;
            tiles.push_back(PieceItem{p, (int64_t)p.nrtg * sh.segs_main});
        }
    }
    // The hardware starts workgroups in index order as compute units free up: the longest ones go first, so that the
    // launch does not end with a few long workgroups running alone.
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

bcq_status bcq_batch_prepare(const void* table_host, size_t table_bytes) {
    // a dry run of bcq_linear_batched: stand-in pointers, no launch
    void* const p = reinterpret_cast<void*>((uintptr_t)1 << 20);
    bcq::tl_dry_run = true;
    const bcq_status s = bcq_linear_batched(table_host, p, table_bytes, p, ~(size_t)0, nullptr);
    bcq::tl_dry_run = false;
    return s;
}

}  // extern "C"
