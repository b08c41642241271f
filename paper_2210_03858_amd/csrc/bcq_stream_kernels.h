// Small-token path on the block-scaled FP4 x FP8 matrix instruction of gfx950 (up to 16 tokens per tile, bf16 I/O,
// row-wise scales).  It evaluates AlphaTuning Eq. 2 / Eq. 4 / Eq. 3 plane by plane, as they are written,
//     y[t][n]     = sum_i alpha_i[n] * C_i[n][t]          C_i[n][t] = sum_k B_i[n][k] x[t][k]          (Eq. 2)
//     dalpha_i[n] = s * sum_t dy[t][n] * C_i[n][t]                                                      (Eq. 4)
//     dx[t][k]    = sum_i sum_n B_i[n][k] * (alpha_i[n] dy[t][n])                                       (Eq. 3)
// streaming the packed sign planes from HBM exactly once.  What matters here is the work per weight BIT:
//   * v_mfma_scale_f32_16x16x128_f8f6f4 takes the signs as FP4 (e2m1) codes: +1 = 0x2, -1 = 0xA.  One packed word
//     (32 signs) becomes the 4 operand registers of a lane with one shift and one three-input bit operation each:
//         reg_s = ((word << s) & 0x88888888) ^ 0xAAAAAAAA,  s = 0..3
//     (nibble jj of reg_s carries bit 4 jj + 3 - s of the word) - 8 vector-ALU operations per 32 weights.
//   * The activations are the other operand as FP8 (e4m3) with a power-of-two scale per 32 contraction indices
//     (hardware block scaling).  A bf16 value has 8 significant bits = two e4m3 terms of 4 bits each, so
//     x = s (f1 + f2 / 16) EXACTLY for every bf16 element within 2^-13 of its block's maximum (smaller elements keep
//     an absolute error below 2^-21 of that maximum).  That holds for the forward and the scale gradient, whose
//     re-coded operand is a bf16 activation.  The input gradient re-codes the fp32 product dy * alpha_i: two FP8 terms
//     keep 8 of its 24 significant bits, i.e. every term of Eq. 3 carries a relative error of up to 2^-9, the same
//     size as rounding alpha_i * dy to bf16 (and as the bf16 weight sums of the matrix-core path).  A block that holds
//     an Inf or a NaN is given the NaN scale byte, so a non-finite activation turns exactly its own token's outputs
//     into NaN.  A short pre-kernel writes the two terms, already in the
//     register order of the instruction and with the contraction index permuted to match the sign expansion
//     above.  With at most 8 tokens both terms sit side by side in the 16 columns of ONE instruction
//     (column t and t + 8), else they take two instructions.
// Measured on this part: 15.3 ns per instruction per SIMD for 16 x 16 x 128, i.e. 4.4x the contraction length per
// nanosecond of the bf16 16x16x32 form the other small-token kernel uses.
//
// Operand layout of the instruction (found by register-only probes and used below): hardware contraction index
// kappa in [0, 128), chunk c = kappa / 16.  FP4 operand: lane (row, g) holds kappa = 32 g .. 32 g + 31 as nibbles
// 0 .. 31 of its four registers.  FP8 operand: lane (col, g) holds chunks g and g + 4 in bytes 0 .. 15 and
// 16 .. 31 of its eight registers.  The scale byte of lane (col, g) multiplies kappa = 32 g .. 32 g + 31.
// Result register v of lane l: row 4 (l / 16) + v, column l % 16.
//
// Work split as in the other small-token kernel: a workgroup owns 16 R rows of the plane matrix and one 16-token
// tile; its waves split the 512-column segments and add their tiles through LDS in wave order (deterministic).
#pragma once
#include "bcq_internal.h"

namespace bcq {

typedef __attribute__((ext_vector_type(8))) int q_i32x8;
typedef __attribute__((ext_vector_type(4))) float q_f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t q_u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t q_u32x2;
typedef __attribute__((ext_vector_type(2))) float q_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 q_bf16x2;

enum { STREAM_FWD = 0, STREAM_DALPHA = 1, STREAM_DX = 2 };

constexpr int QBLK = 2048;   // bytes of one FP8 operand: 2 register halves x 64 lanes x 16 B
constexpr int QSCL = 256;    // bytes of the scales of one segment and half: 64 lanes x 4 instructions

struct StreamPlan {
    int R, W, segs_per_wave, halves, tiles;
    int64_t segs;
    unsigned grid_x;
    size_t xq_bytes, sq_bytes;  // per plane set (DX has q of them)
};

__device__ __forceinline__ uint32_t q_pack_bf16x2(float lo, float hi) {
    q_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, q_bf16x2));
}

// ---------------------------------------------------------------------------------------------------------
// Pre-kernel: activations -> two block-scaled FP8 terms in operand order.
// One thread per (token tile, segment, instruction j, token, 32-index block G): it owns packed-word position
// 16 seg + 4 G + j of the contraction axis (32 columns), finds the block's power-of-two scale, and writes
// 2 x 16 bytes per term plus the scale bytes.  DX: the activation is dy[t][n] * alpha_i[n][grp] for set
// blockIdx.y = i NG + grp (NG scale groups along the columns of W; row-wise scales: NG = 1).
// One unit of the re-coding: the 32 values v of one token (column tl of its 16-token tile) and one packed-word
// position (block G of instruction j) -> two FP8 terms and their scale bytes, stored into the operand blocks of
// instruction j (xb: [half][2 KiB]) and the scales of the segment (sb: [half][256 B]); global memory or LDS.
__device__ __forceinline__ void recode_unit(const float (&v)[32], int tl, int G, int j, bool one_half, unsigned char* xb,
                                            unsigned char* sb) {
    float amax = 0.f;
    bool finite = true;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        amax = fmaxf(amax, fabsf(v[e]));
        finite = finite && (fabsf(v[e]) <= 3.0e38f);  // false for Inf and NaN
    }
    // smallest power of two 2^E with amax / 2^E <= 448 (largest e4m3 value = 1.75 * 2^8); scale byte = E + 127
    int sb1 = 127;
    if (amax > 0.f && finite) {
        const uint32_t u = __float_as_uint(amax);
        const int e = (int)(u >> 23) - 127;
        const int E = ((u & 0x7FFFFFu) <= 0x600000u) ? e - 8 : e - 7;
        sb1 = E + 127;
        sb1 = sb1 < 0 ? 0 : sb1;
    }
    int sb2 = sb1 >= 4 ? sb1 - 4 : 0;                             // second term: 1/16 of the first scale
    const float inv1 = __uint_as_float((uint32_t)(254 - sb1) << 23); // 2^-(sb1 - 127); sb1 <= 247, so it is normal
    const float up2 = __uint_as_float((uint32_t)(127 + sb1 - sb2) << 23);
    // A block that holds an Inf or a NaN gets the NaN scale byte (0xFF) for both terms: every product of the block, and
    // with it every output of this token that contracts over the block, becomes NaN.  A non-finite activation so shows
    // in its own token's outputs and in no other token's (tokens are separate columns of the instruction, each with
    // scale bytes of its own).
    const int sbw1 = finite ? sb1 : 255, sbw2 = finite ? sb2 : 255;
    // element kappa' = 8 s + jj of the block is bit (column) 4 jj + 3 - s of the word
    uint32_t t1[8], t2[8];
#pragma unroll
    for (int pr = 0; pr < 16; ++pr) {
        const int k0 = 2 * pr, k1 = 2 * pr + 1;
        const float x0 = v[4 * (k0 & 7) + 3 - (k0 >> 3)] * inv1, x1 = v[4 * (k1 & 7) + 3 - (k1 >> 3)] * inv1;
        const int p1 = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
        const q_f32x2 d = __builtin_amdgcn_cvt_pk_f32_fp8(p1, false);
        const int p2 = __builtin_amdgcn_cvt_pk_fp8_f32((x0 - d[0]) * up2, (x1 - d[1]) * up2, 0, false);
        if ((pr & 1) == 0) {
            t1[pr >> 1] = (uint32_t)p1 & 0xFFFFu;
            t2[pr >> 1] = (uint32_t)p2 & 0xFFFFu;
        } else {
            t1[pr >> 1] |= (uint32_t)p1 << 16;
            t2[pr >> 1] |= (uint32_t)p2 << 16;
        }
    }
    // chunk 2 G + cc (cc = 0, 1) lives in lane group (2 G + cc) % 4, register half (2 G + cc) / 4; an operand block is
    // stored as [register half][lane][16 B], so that a 16-byte read per lane is contiguous over the wave.
    // One half (at most 8 tokens): the second term of token tl sits in column tl + 8 of the same block.
    const int col1 = tl, col2 = one_half ? tl + 8 : tl;
    const int half2 = one_half ? 0 : 1;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
        const int c = 2 * G + cc, gB = c & 3, hh = c >> 2;
        const q_u32x4 o1 = {t1[4 * cc], t1[4 * cc + 1], t1[4 * cc + 2], t1[4 * cc + 3]};
        const q_u32x4 o2 = {t2[4 * cc], t2[4 * cc + 1], t2[4 * cc + 2], t2[4 * cc + 3]};
        *reinterpret_cast<q_u32x4*>(xb + hh * (QBLK / 2) + (gB * 16 + col1) * 16) = o1;
        *reinterpret_cast<q_u32x4*>(xb + half2 * QBLK + hh * (QBLK / 2) + (gB * 16 + col2) * 16) = o2;
    }
    sb[(col1 + 16 * G) * 4 + j] = (unsigned char)sbw1;
    sb[half2 * QSCL + (col2 + 16 * G) * 4 + j] = (unsigned char)sbw2;
}

// 32 bf16 values -> fp32
__device__ __forceinline__ void load_unit(const bf16_t* src, float (&v)[32]) {
    const q_u32x4* s4 = reinterpret_cast<const q_u32x4*>(src);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const q_u32x4 r = s4[b];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[8 * b + 2 * e] = __uint_as_float(r[e] << 16);
            v[8 * b + 2 * e + 1] = __uint_as_float(r[e] & 0xFFFF0000u);
        }
    }
}

// bx, by: the block indices the launch geometry of the single-layer kernel gives (a batched launch looks them up)
template <int MODE>
__device__ __forceinline__ void quant_act_body(const bf16_t* __restrict__ act, const float* __restrict__ alpha,
                                               int64_t T, int64_t C, int64_t segs, int halves, int tiles,
                                               unsigned char* __restrict__ xq, unsigned char* __restrict__ sq,
                                               size_t xq_plane, size_t sq_plane, int NG, int seg_mul, uint32_t bx,
                                               uint32_t by) {
    const int64_t idx = (int64_t)bx * 256 + threadIdx.x;
    const bool one_half_map = (halves == 1);
    // two halves: 4 blocks x 16 tokens x 4 instructions = 256 units per (tile, segment).  One half: only tokens 0 .. 7
    // have units; they are mapped onto the first 128 threads so that two waves work with all lanes instead of four
    // waves with half of them.
    if (one_half_map && (threadIdx.x & 255) >= 128) return;
    // the token index runs fastest over the lanes: the 16-byte stores of neighbouring lanes are then neighbours in the
    // operand block (column = token), 128 or 256 bytes in a row instead of one piece per lane
    const int tl = one_half_map ? (int)(idx & 7) : (int)(idx & 15);
    const int G = one_half_map ? (int)((idx >> 3) & 3) : (int)((idx >> 4) & 3);
    const int j = one_half_map ? (int)((idx >> 5) & 3) : (int)((idx >> 6) & 3);
    const int64_t seg = (idx >> 8) % segs, tile = (idx >> 8) / segs;
    if (tile >= tiles) return;
    const int plane = (int)by;
    xq += (size_t)plane * xq_plane;
    sq += (size_t)plane * sq_plane;
    const int64_t t = tile * 16 + tl;
    const bool one_half = (halves == 1);
    if (one_half && tl >= 8) return;  // columns 8 .. 15 of the single half belong to the second term of tokens 0 .. 7
    const int64_t word = seg * 16 + 4 * G + j;  // 32 columns of the contraction axis
    const bool live = (t < T) && (word * 32 < C);
    float v[32];
    if (live) {
        load_unit(act + t * C + word * 32, v);
        if (MODE == STREAM_DX) {
            const int pl_i = plane / NG, grp = plane % NG;
            const float* a = alpha + ((int64_t)pl_i * C + word * 32) * NG + grp;  // alpha[i][n][grp], n = 32 word + e
            if (NG == 1) {  // row-wise scales: 32 consecutive floats, 128-byte aligned (C is a multiple of 32)
                const q_f32x4* a4 = reinterpret_cast<const q_f32x4*>(a);
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const q_f32x4 av = a4[b];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[4 * b + e] *= av[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 32; ++e) v[e] *= a[(int64_t)e * NG];
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 32; ++e) v[e] = 0.f;
    }
    // seg_mul > 1 interleaves the sets: block (segment, set) at index segment * seg_mul + set (xq_plane, sq_plane = one block)
    recode_unit(v, tl, G, j, one_half, xq + ((size_t)(tile * segs + seg) * seg_mul * 4 + j) * halves * QBLK,
                sq + (size_t)(tile * segs + seg) * seg_mul * halves * QSCL);
}

template <int MODE>
__global__ __launch_bounds__(256) void quant_act_kernel(const bf16_t* __restrict__ act, const float* __restrict__ alpha,
                                                        int64_t T, int64_t C, int64_t segs, int halves, int tiles,
                                                        unsigned char* __restrict__ xq, unsigned char* __restrict__ sq,
                                                        size_t xq_plane, size_t sq_plane, int NG) {
    quant_act_body<MODE>(act, alpha, T, C, segs, halves, tiles, xq, sq, xq_plane, sq_plane, NG, 1, blockIdx.x, blockIdx.y);
}

// ---------------------------------------------------------------------------------------------------------
// planes: [q][rows][cw] words (canonical for FWD / DALPHA, twin for DX); xq / sq: output of quant_act_kernel
// (DX: one set per plane).  rows x 32 cw is the plane matrix seen by this kernel.
// QUAD: the plane rows are read 16 bytes per lane (needs cw % 4 == 0); a segment that reaches beyond the row is
// shifted back inside it - the words it then re-reads meet zero activations.
// GROUPED: group-wise scales alpha[q][N][G].  Forward: the plane sums are folded into y with the group's scales at
// every group boundary (gsegs segments).  Scale gradient: every group's sums are reduced over the tokens and stored
// at its end; the host gives every wave whole groups, so no cross-wave sum is needed.  Input gradient: the set of
// re-coded activations is chosen by the group of the workgroup's rows (dxg rows of the twin per group).
// TILED (forward only): `planes` is the decode layout [row tile][segment][plane][64 lanes][4 words] (padded to whole
// row tiles and segments), so the 1 KiB a wave reads per plane and segment is one contiguous run.
template <int MODE, int R, int QP, bool TWO, bool QUAD, bool GROUPED, bool TILED>
__device__ __forceinline__ void stream_body(const uint32_t* __restrict__ planes, const unsigned char* __restrict__ xq,
                                            const unsigned char* __restrict__ sq, const float* __restrict__ alpha,
                                            const bf16_t* __restrict__ dy, void* __restrict__ out, int64_t T, int64_t rows,
                                            int64_t cw, int q_used, float scale, int segs_per_wave, int64_t segs,
                                            size_t xq_plane, size_t sq_plane, int scale_a, int gsegs, int G, int64_t dxg,
                                            uint32_t bx, uint32_t by) {
    extern __shared__ __attribute__((aligned(16))) float red[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int rl = lane & 15, g = lane >> 4;
    const int64_t row0 = (int64_t)bx * 16 * R;
    const int64_t tile = by;
    const int64_t t0 = tile * 16;
    constexpr int H = TWO ? 2 : 1;
    constexpr int NACC = (MODE == STREAM_DX) ? 1 : QP;
    constexpr int PPP = QP;  // planes handled per segment (DX: q_used real planes, the rest repeat the last)

    q_f32x4 acc[R][NACC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < NACC; ++i) acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};

    // Addresses are a uniform 64-bit base (scalar registers) plus a 32-bit lane offset: rows * cw <= 2^29 words.
    const uint32_t cw32 = (uint32_t)cw;
    uint32_t roff[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t rr = row0 + 16 * r + rl;
        rr = rr < rows ? rr : rows - 1;  // rows beyond the matrix give outputs that are never stored
        roff[r] = (uint32_t)(rr * cw);
    }
    const int64_t plane_stride = rows * cw;
    const uint32_t* pl[PPP];
#pragma unroll
    for (int i = 0; i < PPP; ++i) pl[i] = planes + (int64_t)(i < q_used ? i : q_used - 1) * plane_stride;

    // result column of this lane -> token: with one half, columns t and t + 8 both belong to token t
    const int tcol = TWO ? rl : (rl & 7);
    const bool tok_live = (t0 + tcol) < T;
    const int64_t tok = tok_live ? t0 + tcol : T - 1;

    float ep[R][QP][4];  // FWD: alpha_i of this lane's 4 rows; DALPHA: dy of this lane's token and 4 rows (slot 0)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int64_t n = row0 + 16 * r + 4 * g + v;
            const bool n_live = n < rows;
            n = n_live ? n : rows - 1;
            if (MODE == STREAM_FWD) {
#pragma unroll
                for (int i = 0; i < QP; ++i)
                    ep[r][i][v] = (!GROUPED && i < q_used) ? alpha[(int64_t)i * rows + n] : 0.f;
            } else if (MODE == STREAM_DALPHA) {
                ep[r][0][v] = (tok_live && n_live) ? bf16_to_f32(dy[tok * rows + n]) : 0.f;
            }
        }

    const int seg_begin = wave * segs_per_wave;
    constexpr int NSET = (MODE == STREAM_DX) ? PPP : 1;  // DX: every plane has its own scaled activations
    const unsigned char* xqp[NSET];
    const unsigned char* sqp[NSET];
#pragma unroll
    for (int ps = 0; ps < NSET; ++ps) {
        int pc = ps < q_used ? ps : q_used - 1;
        if (GROUPED && MODE == STREAM_DX) pc = pc * G + (int)(row0 / dxg);  // the 16 R rows lie in one group (g % 32 == 0)
        xqp[ps] = xq + (size_t)pc * xq_plane + (size_t)tile * segs * 4 * H * QBLK;
        sqp[ps] = sq + (size_t)pc * sq_plane + (size_t)tile * segs * H * QSCL;
    }
    const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u;

    // Software pipeline: the plane words of the NEXT segment and the activation operand of the NEXT instruction
    // group are requested before the matrix instructions of the current one are issued.
    uint32_t bits[2][R][PPP][4];
    q_i32x8 bop[2][NSET][H];
    int sc[2][NSET][H];
    auto load_bits = [&](int seg, int buf) {
        uint32_t w0 = (uint32_t)seg * 16u + 4u * (uint32_t)g;
        if (TILED) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t* tb = planes + (((row0 >> 4) + r) * segs + seg) * (int64_t)(q_used * 256) + lane * 4;
#pragma unroll
                for (int i = 0; i < PPP; ++i) {
                    const q_u32x4 v4 = *reinterpret_cast<const q_u32x4*>(tb + (i < q_used ? i : q_used - 1) * 256);
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) bits[buf][r][i][jj] = v4[jj];
                }
            }
        } else if (QUAD) {
            w0 = w0 < cw32 - 4u ? w0 : cw32 - 4u;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < PPP; ++i) {
                    const q_u32x4 v4 = *reinterpret_cast<const q_u32x4*>(pl[i] + (roff[r] + w0));
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) bits[buf][r][i][jj] = v4[jj];
                }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < PPP; ++i)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        uint32_t wj = w0 + (uint32_t)jj;
                        wj = wj < cw32 ? wj : cw32 - 1u;  // columns beyond C meet zero activations
                        bits[buf][r][i][jj] = pl[i][roff[r] + wj];
                    }
        }
#pragma unroll
        for (int ps = 0; ps < NSET; ++ps)
#pragma unroll
            for (int h = 0; h < H; ++h)
                sc[buf][ps][h] = *reinterpret_cast<const int*>(sqp[ps] + (uint32_t)((seg * H + h) * QSCL) + lane4);
    };
    auto load_bop = [&](int seg, int jj, int buf) {
#pragma unroll
        for (int ps = 0; ps < NSET; ++ps)
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const unsigned char* bp = xqp[ps] + (uint32_t)(((seg * 4 + jj) * H + h) * QBLK);
                const q_u32x4 lo = *reinterpret_cast<const q_u32x4*>(bp + lane16);
                const q_u32x4 hi = *reinterpret_cast<const q_u32x4*>(bp + lane16 + (uint32_t)(QBLK / 2));
                bop[buf][ps][h] = q_i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3],
                                          (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
    };
    int seg_end = seg_begin + segs_per_wave;
    seg_end = seg_end < (int)segs ? seg_end : (int)segs;
    // group-wise scales (forward / scale gradient): y accumulated over the groups, scales of the current group
    q_f32x4 yv[R];
    float ga[R][QP][4];
#pragma unroll
    for (int r = 0; r < R; ++r) yv[r] = q_f32x4{0.f, 0.f, 0.f, 0.f};
    auto load_group_alpha = [&](int grp) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int64_t n = row0 + 16 * r + 4 * g + v;
                n = n < rows ? n : rows - 1;
#pragma unroll
                for (int i = 0; i < QP; ++i) ga[r][i][v] = (i < q_used) ? alpha[((int64_t)i * rows + n) * G + grp] : 0.f;
            }
    };
    if (seg_begin < seg_end) {  // uniform per wave
        load_bits(seg_begin, 0);
        load_bop(seg_begin, 0, 0);
    }
    for (int seg = seg_begin; seg < seg_end; ++seg) {
        const int nseg = (seg + 1 < seg_end) ? seg + 1 : seg;  // the last segment re-requests itself (unused)
        if (GROUPED && MODE == STREAM_FWD && (seg == seg_begin || seg % gsegs == 0)) load_group_alpha(seg / gsegs);
        load_bits(nseg, 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < 3)
                load_bop(seg, j + 1, (j + 1) & 1);
            else
                load_bop(nseg, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < PPP; ++i) {
                    const uint32_t wd = bits[0][r][i][j];
                    q_i32x8 aop;
#pragma unroll
                    for (int sft = 0; sft < 4; ++sft) aop[sft] = (int)(((wd << sft) & 0x88888888u) ^ 0xAAAAAAAAu);
                    aop[4] = 0;
                    aop[5] = 0;
                    aop[6] = 0;
                    aop[7] = 0;
                    constexpr int DXI = (MODE == STREAM_DX) ? 1 : 0;
                    const int ai = DXI ? 0 : i;
                    const int ps = DXI ? i : 0;
                    if (MODE == STREAM_DX && i >= q_used) continue;  // uniform: planes beyond q do not exist
#pragma unroll
                    for (int h = 0; h < H; ++h) {
                        // the instruction picks byte j of the scale register (its op_sel), so j must be a constant
                        const q_i32x8 bo = bop[j & 1][ps][h];
                        const int sv = sc[0][ps][h];
                        if (j == 0)
                            acc[r][ai] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo, acc[r][ai], 4, 0, 0, scale_a, 0, sv);
                        else if (j == 1)
                            acc[r][ai] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo, acc[r][ai], 4, 0, 0, scale_a, 1, sv);
                        else if (j == 2)
                            acc[r][ai] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo, acc[r][ai], 4, 0, 0, scale_a, 2, sv);
                        else
                            acc[r][ai] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo, acc[r][ai], 4, 0, 0, scale_a, 3, sv);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (GROUPED && MODE != STREAM_DX && ((seg + 1) % gsegs == 0 || seg + 1 == seg_end)) {  // uniform: a group ends
            const int grp = seg / gsegs;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (MODE == STREAM_FWD) {
#pragma unroll
                    for (int i = 0; i < QP; ++i)
#pragma unroll
                        for (int v = 0; v < 4; ++v) yv[r][v] += ga[r][i][v] * acc[r][i][v];
                } else {
                    // both columns of a token (t and t + 8 with one half) carry dy of that token: the 16-lane sum
                    // adds the two terms and the tokens at once
                    const int64_t n = row0 + 16 * r + 4 * g;
#pragma unroll
                    for (int o = 0; o < QP; ++o)
                        if (o < q_used) {
                            q_f32x4 sum;
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                float x = ep[r][0][v] * acc[r][o][v];
                                x += __shfl_xor(x, 1);
                                x += __shfl_xor(x, 2);
                                x += __shfl_xor(x, 4);
                                x += __shfl_xor(x, 8);
                                sum[v] = x * scale;
                            }
                            if (rl == 0)
#pragma unroll
                                for (int v = 0; v < 4; ++v)
                                    if (n + v < rows)
                                        reinterpret_cast<float*>(out)[(((int64_t)o * rows + n + v) * G) + grp] = sum[v];
                        }
                }
#pragma unroll
                for (int i = 0; i < NACC; ++i) acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        // hand the prefetched segment over (register moves; the next iteration's requests go to buffer 1 again)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < PPP; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) bits[0][r][i][jj] = bits[1][r][i][jj];
#pragma unroll
        for (int ps = 0; ps < NSET; ++ps)
#pragma unroll
            for (int h = 0; h < H; ++h) sc[0][ps][h] = sc[1][ps][h];
    }

    if (GROUPED && MODE == STREAM_DALPHA) return;  // every group was stored at its end
    if (GROUPED && MODE == STREAM_FWD) {            // continue below with y in place of the plane sums
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r][0] = yv[r];
#pragma unroll
            for (int v = 0; v < 4; ++v) ep[r][0][v] = 1.f;
#pragma unroll
            for (int i = 1; i < QP; ++i) {
                acc[r][i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int v = 0; v < 4; ++v) ep[r][i][v] = 0.f;
            }
        }
    }
    // one half: add the second term's columns (t + 8) onto the first term's (t); lanes l and l ^ 8 swap
    if (!TWO) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[r][i][v] += __shfl_xor(acc[r][i][v], 8);
    }

    // From here on as in the bf16 small-token kernel.  Result register v of lane l: row 4 (l / 16) + v, token column.
    constexpr int NOUT = (MODE == STREAM_DALPHA) ? QP : 1;
    const int nout = (MODE == STREAM_DALPHA) ? q_used : 1;
    q_f32x4 part[R][NOUT];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (MODE == STREAM_FWD) {
            q_f32x4 y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < QP; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) y[v] += ep[r][i][v] * acc[r][i][v];  // alpha of unused planes is 0
            part[r][0] = y;
        } else if (MODE == STREAM_DX) {
            part[r][0] = acc[r][0];
        } else {
#pragma unroll
            for (int i = 0; i < NOUT; ++i) part[r][i] = acc[r][i < NACC ? i : 0];
        }
    }
    if (W > 1) {  // cross-wave sum in wave order: red[w][r][o][lane][4]
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) *reinterpret_cast<q_f32x4*>(&red[(((wave * R + r) * nout + o) * 64 + lane) * 4]) = part[r][o];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) {
                    q_f32x4 sum = part[r][o];
                    for (int w = 1; w < W; ++w) sum += *reinterpret_cast<const q_f32x4*>(&red[(((w * R + r) * nout + o) * 64 + lane) * 4]);
                    part[r][o] = sum;
                }
    }
    const bool col_live = tok_live && (TWO || rl < 8);  // with one half, columns 8 .. 15 duplicate columns 0 .. 7
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t n = row0 + 16 * r + 4 * g;  // first of this lane's 4 rows
        if (MODE == STREAM_DALPHA) {
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
                if (o < nout) {
                    q_f32x4 sum;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float x = col_live ? ep[r][0][v] * part[r][o][v] : 0.f;
                        x += __shfl_xor(x, 1);
                        x += __shfl_xor(x, 2);
                        x += __shfl_xor(x, 4);
                        x += __shfl_xor(x, 8);
                        sum[v] = x * scale;
                    }
                    if (rl == 0)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (n + v < rows) reinterpret_cast<float*>(out)[(int64_t)o * rows + n + v] = sum[v];
                }
        } else {
            bf16_t* o = reinterpret_cast<bf16_t*>(out);
            if (col_live) {
                if (n + 3 < rows && (rows & 3) == 0) {
                    q_u32x2 pk;
                    pk[0] = q_pack_bf16x2(part[r][0][0], part[r][0][1]);
                    pk[1] = q_pack_bf16x2(part[r][0][2], part[r][0][3]);
                    *reinterpret_cast<q_u32x2*>(o + tok * rows + n) = pk;
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (n + v < rows) o[tok * rows + n + v] = f32_to_bf16(part[r][0][v]);
                }
            }
        }
    }
}

template <int MODE, int R, int QP, bool TWO, bool QUAD, bool GROUPED, bool TILED>
__global__ __launch_bounds__(512) void stream_kernel(const uint32_t* __restrict__ planes,
                                                      const unsigned char* __restrict__ xq,
                                                      const unsigned char* __restrict__ sq,
                                                      const float* __restrict__ alpha, const bf16_t* __restrict__ dy,
                                                      void* __restrict__ out, int64_t T, int64_t rows, int64_t cw,
                                                      int q_used, float scale, int segs_per_wave, int64_t segs,
                                                      size_t xq_plane, size_t sq_plane, int scale_a, int gsegs, int G,
                                                      int64_t dxg) {
    stream_body<MODE, R, QP, TWO, QUAD, GROUPED, TILED>(planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale,
                                                        segs_per_wave, segs, xq_plane, sq_plane, scale_a, gsegs, G, dxg,
                                                        blockIdx.x, blockIdx.y);
}

// Common end of the one-row-tile kernels.  acc: plane sums (or y in slot 0 with ep = 1, 0, ..) of this wave's part of
// the contraction; ep: FWD alpha_i of the lane's 4 rows, DALPHA dy of the lane's token (slot 0).  The nparts parts of a
// row tile are added in part order through `red` (slot of part p of row tile `sub`: p * pstride + sub); every wave
// of the workgroup must call this (it contains a barrier), and `red` must be free for reuse when it does.
template <int MODE, int QP, bool TWO>
__device__ __forceinline__ void stream_finish(q_f32x4 (&acc)[QP], float (&ep)[QP][4], float* red, int nparts, int part_id,
                                              int pstride, int sub, int lane, int64_t row0, int64_t rows, int64_t tok,
                                              bool tok_live, int q_used, float scale, void* out) {
    const int rl = lane & 15, g = lane >> 4;
    if (!TWO) {  // one half: add the second term's columns (t + 8) onto the first term's (t)
#pragma unroll
        for (int i = 0; i < QP; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][v] += __shfl_xor(acc[i][v], 8);
    }
    constexpr int NOUT = (MODE == STREAM_DALPHA) ? QP : 1;
    const int nout = (MODE == STREAM_DALPHA) ? q_used : 1;
    q_f32x4 part[NOUT];
    if (MODE == STREAM_FWD) {
        q_f32x4 y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < QP; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) y[v] += ep[i][v] * acc[i][v];  // alpha of unused planes is 0
        part[0] = y;
    } else {
#pragma unroll
        for (int i = 0; i < NOUT; ++i) part[i] = acc[i];
    }
    if (nparts > 1) {
#pragma unroll
        for (int o = 0; o < NOUT; ++o)
            if (o < nout && part_id > 0)
                *reinterpret_cast<q_f32x4*>(&red[(((part_id * pstride + sub) * nout + o) * 64 + lane) * 4]) = part[o];
        __syncthreads();
        if (part_id != 0) return;
#pragma unroll
        for (int o = 0; o < NOUT; ++o)
            if (o < nout) {
                q_f32x4 sum = part[o];
                for (int w = 1; w < nparts; ++w)
                    sum += *reinterpret_cast<const q_f32x4*>(&red[(((w * pstride + sub) * nout + o) * 64 + lane) * 4]);
                part[o] = sum;
            }
    }
    const bool col_live = tok_live && (TWO || rl < 8);  // with one half, columns 8 .. 15 duplicate columns 0 .. 7
    const int64_t n = row0 + 4 * g;                     // first of this lane's 4 rows
    if (MODE == STREAM_DALPHA) {
#pragma unroll
        for (int o = 0; o < NOUT; ++o)
            if (o < nout) {
                q_f32x4 sum;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float x = col_live ? ep[0][v] * part[o][v] : 0.f;
                    x += __shfl_xor(x, 1);
                    x += __shfl_xor(x, 2);
                    x += __shfl_xor(x, 4);
                    x += __shfl_xor(x, 8);
                    sum[v] = x * scale;
                }
                if (rl == 0)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (n + v < rows) reinterpret_cast<float*>(out)[(int64_t)o * rows + n + v] = sum[v];
            }
    } else {
        bf16_t* o = reinterpret_cast<bf16_t*>(out);
        if (col_live) {
            if (n + 3 < rows && (rows & 3) == 0) {
                q_u32x2 pk;
                pk[0] = q_pack_bf16x2(part[0][0], part[0][1]);
                pk[1] = q_pack_bf16x2(part[0][2], part[0][3]);
                *reinterpret_cast<q_u32x2*>(o + tok * rows + n) = pk;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n + v < rows) o[tok * rows + n + v] = f32_to_bf16(part[0][v]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Forward / scale gradient for plane matrices with many rows: the activation operand goes through LDS.
// A compute unit keeps a limited number of cache misses in flight, and in stream_kernel most of them fetch the
// re-coded activations (the same bytes for every row tile) instead of sign planes.  Here a workgroup of 8 waves
// covers RW = 8 / KW row tiles x KW parts of the contraction axis; the activations of LCS segments per part are
// copied global -> registers -> LDS once per workgroup (double buffered, one barrier per LCS segments) and every
// wave reads its operand from there, so the misses in flight are almost all sign planes.  The plane words sit in a
// ring of LCS register sets addressed by the unrolled position, LCS - 1 segments ahead of the multiplication (a
// register move would have to wait for the load it copies).  Needs cw % 4 == 0.
// EXACT: every part has spp segments and spp % LCS == 0 - no guards in the loop.
// Input gradient (STREAM_DX): every plane (and, with group-wise scales, every scale group of the workgroup's rows) has
// its own scaled activations, so nothing of the operand is shared between planes and the call is a one-plane forward
// over q * segs_n VIRTUAL segments of the transposed twin: virtual segment v = plane v / segs_n, segment v % segs_n
// (the division is a multiplication by seg_magic).
constexpr int LCS = 4;

// 32 signs of a packed word -> the four FP4 operand registers of a lane (+1 = 0x2, -1 = 0xA; registers 4 .. 7 of the
// builtin's operand type are not part of an FP4 operand)
__device__ __forceinline__ void expand_one(uint32_t wd, q_i32x8& aop) {
#pragma unroll
    for (int sft = 0; sft < 4; ++sft) aop[sft] = (int)(((wd << sft) & 0x88888888u) ^ 0xAAAAAAAAu);
    aop[4] = 0;
    aop[5] = 0;
    aop[6] = 0;
    aop[7] = 0;
}

template <int MODE, int QP, bool TWO, bool GROUPED, int KW, bool EXACT, bool TILED>
__device__ __forceinline__ void stream_lds_body(const uint32_t* __restrict__ planes, const unsigned char* __restrict__ xq,
                                                const unsigned char* __restrict__ sq, const float* __restrict__ alpha,
                                                const bf16_t* __restrict__ dy, void* __restrict__ out, int64_t T,
                                                int64_t rows, int64_t cw, int q_used, float scale, int spp, int64_t segs,
                                                int gsegs, int G, int64_t xq_plane, int64_t sq_plane, uint32_t seg_magic,
                                                int segs_n, uint32_t bx, uint32_t by) {
    constexpr bool DX = (MODE == STREAM_DX);
    static_assert(!DX || (QP == 1 && !GROUPED && !TILED), "input gradient: one virtual plane, twin layout (scale groups are handled at run time)");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int H = TWO ? 2 : 1, RW = 8 / KW, PF = LCS - 1;
    constexpr int XPART = LCS * 4 * H * QBLK, XBUF = KW * XPART;  // operand blocks of one part / of one buffer
    constexpr int SPART = LCS * H * QSCL, SBUF = KW * SPART;      // scales
    constexpr int BUFB = XBUF + SBUF;
    constexpr int NIT = XBUF / (512 * 16);  // 16-byte units per thread and chunk (= KW LCS H)
    constexpr int NSU = SBUF / 16;          // threads that copy one 16-byte unit of scales
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kp = wave / RW, rtile = wave % RW;
    const int rl = lane & 15, g = lane >> 4;
    const int64_t row0 = ((int64_t)bx * RW + rtile) * 16;
    const int64_t tile = by;
    const int64_t t0 = tile * 16;

    q_f32x4 acc[QP];
#pragma unroll
    for (int i = 0; i < QP; ++i) acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};

    const uint32_t cw32 = (uint32_t)cw;
    uint32_t roff;
    {
        int64_t rr = row0 + rl;
        rr = rr < rows ? rr : rows - 1;  // rows beyond the matrix give outputs that are never stored
        roff = (uint32_t)(rr * cw);
    }
    const int64_t plane_stride = rows * cw;
    const uint32_t* pl[QP];
#pragma unroll
    for (int i = 0; i < QP; ++i) pl[i] = planes + (int64_t)(i < q_used ? i : q_used - 1) * plane_stride;

    const int tcol = TWO ? rl : (rl & 7);
    const bool tok_live = (t0 + tcol) < T;
    const int64_t tok = tok_live ? t0 + tcol : T - 1;
    float ep[QP][4];  // FWD: alpha_i of this lane's 4 rows; DALPHA: dy of this lane's token and 4 rows (slot 0)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int64_t n = row0 + 4 * g + v;
        const bool n_live = n < rows;
        n = n_live ? n : rows - 1;
        if (MODE == STREAM_FWD) {
#pragma unroll
            for (int i = 0; i < QP; ++i) ep[i][v] = (!GROUPED && i < q_used) ? alpha[(int64_t)i * rows + n] : 0.f;
        } else if (DX) {
            ep[0][v] = 0.f;  // unused: the scales are part of the activations
        } else {
            ep[0][v] = (tok_live && n_live) ? bf16_to_f32(dy[tok * rows + n]) : 0.f;
        }
    }

    // DX: a set of activations per plane, [plane][token tile][segment]
    const int64_t segs_tile = DX ? segs_n : segs;
    const unsigned char* xqt = xq + (size_t)tile * segs_tile * 4 * H * QBLK;
    const unsigned char* sqt = sq + (size_t)tile * segs_tile * H * QSCL;
    auto split = [&](int vseg, int& pl_i, int& sg) {  // virtual segment -> plane, segment
        pl_i = (int)(((uint64_t)(uint32_t)vseg * seg_magic) >> 32);
        sg = vseg - pl_i * segs_n;
    };
    // DX with group-wise scales: G activation sets per plane; the host takes this kernel only when the rows of a
    // workgroup (16 RW of them) lie in one scale group
    const int dx_grp = (DX && G > 1) ? (int)(((int64_t)bx * RW * 16) / (rows / G)) : 0;
    const int part_begin = kp * spp;
    int part_end = part_begin + spp;
    part_end = part_end < (int)segs ? part_end : (int)segs;
    const bool part_live = EXACT || part_begin < part_end;
    const int nchunks = (spp + LCS - 1) / LCS;
    const int last_seg = (int)segs - 1;

    // staging: chunk c of every part, global -> registers -> LDS buffer
    q_u32x4 stg[NIT], stgs;
    auto stage_load = [&](int c) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int p = it / (LCS * H), r = it % (LCS * H);  // part, 8 KiB slab of its chunk
            int seg = p * spp + c * LCS + r / H;
            if (!EXACT) seg = seg < last_seg ? seg : last_seg;  // in bounds; segments beyond a part are never multiplied
            const unsigned char* src = xqt;
            if (DX) {
                int pl_i, sg;
                split(seg, pl_i, sg);
                src += (size_t)(pl_i * G + dx_grp) * xq_plane;
                seg = sg;
            }
            stg[it] = *reinterpret_cast<const q_u32x4*>(src + (size_t)seg * (4 * H * QBLK) + (r % H) * 8192 + tid * 16);
        }
        if (tid < NSU) {
            const int p = tid / (LCS * H * 16), r2 = tid % (LCS * H * 16);
            int seg = p * spp + c * LCS + r2 / (H * 16);
            if (!EXACT) seg = seg < last_seg ? seg : last_seg;
            const unsigned char* src = sqt;
            if (DX) {
                int pl_i, sg;
                split(seg, pl_i, sg);
                src += (size_t)(pl_i * G + dx_grp) * sq_plane;
                seg = sg;
            }
            stgs = *reinterpret_cast<const q_u32x4*>(src + (size_t)seg * (H * QSCL) + (r2 % (H * 16)) * 16);
        }
    };
    auto stage_store = [&](int buf) {
        unsigned char* b = lds + buf * BUFB;
#pragma unroll
        for (int it = 0; it < NIT; ++it) *reinterpret_cast<q_u32x4*>(b + it * 8192 + tid * 16) = stg[it];
        if (tid < NSU) *reinterpret_cast<q_u32x4*>(b + XBUF + tid * 16) = stgs;
    };

    uint32_t bits[LCS][QP][4];
    // decode layout: row tiles beyond the padded matrix (last workgroup) re-read the last one; nothing of them is stored
    const int64_t rt_pad = (rows + 15) >> 4;
    const int64_t rt_mine = (row0 >> 4) < rt_pad ? (row0 >> 4) : rt_pad - 1;
    auto load_bits = [&](int seg, int slot) {
        if (TILED) {
            const uint32_t* tb = planes + (rt_mine * segs + seg) * (int64_t)(q_used * 256) + lane * 4;
#pragma unroll
            for (int i = 0; i < QP; ++i) {
                const q_u32x4 v4 = *reinterpret_cast<const q_u32x4*>(tb + (i < q_used ? i : q_used - 1) * 256);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) bits[slot][i][jj] = v4[jj];
            }
            return;
        }
        if (DX) {  // plane and segment of the virtual segment (cw % 16 == 0: whole segments)
            int pl_i, sg;
            split(seg, pl_i, sg);
            const q_u32x4 v4 = *reinterpret_cast<const q_u32x4*>(planes + (int64_t)pl_i * plane_stride +
                                                                  (roff + (uint32_t)sg * 16u + 4u * (uint32_t)g));
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) bits[slot][0][jj] = v4[jj];
            return;
        }
        uint32_t w0 = (uint32_t)seg * 16u + 4u * (uint32_t)g;
        w0 = w0 < cw32 - 4u ? w0 : cw32 - 4u;  // a segment that reaches beyond the row is shifted back inside it
#pragma unroll
        for (int i = 0; i < QP; ++i) {
            const q_u32x4 v4 = *reinterpret_cast<const q_u32x4*>(pl[i] + (roff + w0));
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) bits[slot][i][jj] = v4[jj];
        }
    };

    q_f32x4 yv = {0.f, 0.f, 0.f, 0.f};
    float ga[QP][4];
    auto load_group_alpha = [&](int grp) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int64_t n = row0 + 4 * g + v;
            n = n < rows ? n : rows - 1;
#pragma unroll
            for (int i = 0; i < QP; ++i) ga[i][v] = (i < q_used) ? alpha[((int64_t)i * rows + n) * G + grp] : 0.f;
        }
    };

    stage_load(0);
    if (part_live) {
#pragma unroll
        for (int d = 0; d < PF; ++d) {
            const int sg = part_begin + d;
            load_bits(EXACT ? sg : (sg < part_end ? sg : part_end - 1), d);
        }
    }
    stage_store(0);
    __syncthreads();

#pragma unroll 1
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        stage_load(c + 1 < nchunks ? c + 1 : c);  // after the last chunk: re-requests it (unused)
        const unsigned char* xb = lds + buf * BUFB + kp * XPART;
        const unsigned char* sb = lds + buf * BUFB + XBUF + kp * SPART;
        // operand of instruction group (s, j) and scales of segment s, LDS -> registers one group ahead of their use
        q_i32x8 bo[2][H];
        int sv[2][H];
        auto read_b = [&](int s, int j, int slot) {
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const unsigned char* bp = xb + ((s * 4 + j) * H + h) * QBLK + lane * 16;
                const q_u32x4 lo = *reinterpret_cast<const q_u32x4*>(bp);
                const q_u32x4 hi = *reinterpret_cast<const q_u32x4*>(bp + QBLK / 2);
                bo[slot][h] = q_i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3],
                                      (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
        };
        auto read_s = [&](int s, int slot) {
#pragma unroll
            for (int h = 0; h < H; ++h) sv[slot][h] = *reinterpret_cast<const int*>(sb + (s * H + h) * QSCL + lane * 4);
        };
        read_s(0, 0);
        read_b(0, 0, 0);
#pragma unroll
        for (int s = 0; s < LCS; ++s) {
            const int seg = part_begin + c * LCS + s;  // its planes sit in ring set s
            asm volatile("" ::: "memory");  // keeps the loads of the four unrolled segments where they are written
            if (part_live) {
                const int pseg = seg + PF;
                load_bits(pseg < part_end ? pseg : part_end - 1, (s + PF) % LCS);  // beyond the part: unused
            }
            __builtin_amdgcn_sched_barrier(0);
            if (EXACT || seg < part_end) {  // uniform per wave
                if (GROUPED && MODE == STREAM_FWD && (seg == part_begin || seg % gsegs == 0)) load_group_alpha(seg / gsegs);
                // The FP4 operands of instruction group j + 1 are expanded while the matrix instructions of group j
                // run: each expansion is written right behind one matrix instruction, into registers no instruction
                // in flight reads (two sets), so the vector ALU works in the shadow of the matrix pipe.
                q_i32x8 ao[2][QP];
                auto expand = [&](int j, int set) {
#pragma unroll
                    for (int i = 0; i < QP; ++i) expand_one(bits[s][i][j], ao[set][i]);
                };
                expand(0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // group (s, j) sits in slot (4 s + j) % 2 = j % 2; request the next group of this chunk
                    if (j < 3) {
                        read_b(s, j + 1, (j + 1) & 1);
                    } else if (s + 1 < LCS) {
                        read_b(s + 1, 0, 0);
                        read_s(s + 1, (s + 1) & 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < QP; ++i) {
#pragma unroll
                        for (int h = 0; h < H; ++h) {
                            // the instruction picks byte j of the scale register (its op_sel): j must be a constant
                            if (j == 0)
                                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao[j & 1][i], bo[j & 1][h], acc[i], 4, 0, 0, 127, 0, sv[s & 1][h]);
                            else if (j == 1)
                                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao[j & 1][i], bo[j & 1][h], acc[i], 4, 0, 0, 127, 1, sv[s & 1][h]);
                            else if (j == 2)
                                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao[j & 1][i], bo[j & 1][h], acc[i], 4, 0, 0, 127, 2, sv[s & 1][h]);
                            else
                                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ao[j & 1][i], bo[j & 1][h], acc[i], 4, 0, 0, 127, 3, sv[s & 1][h]);
                        }
                        if (j < 3) expand_one(bits[s][i][j + 1], ao[(j + 1) & 1][i]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // pins the matrix instructions of this segment before the loads of the next (they are no memory
                // operations, so the barrier above alone lets the optimiser sink them to the end of the chunk)
#pragma unroll
                for (int i = 0; i < QP; ++i) asm volatile("" : "+v"(acc[i]));
                if (GROUPED && ((seg + 1) % gsegs == 0 || seg + 1 == part_end)) {  // uniform: a scale group ends
                    const int grp = seg / gsegs;
                    if (MODE == STREAM_FWD) {
#pragma unroll
                        for (int i = 0; i < QP; ++i)
#pragma unroll
                            for (int v = 0; v < 4; ++v) yv[v] += ga[i][v] * acc[i][v];
                    } else {
                        // both columns of a token (t and t + 8 with one half) carry dy of that token: the 16-lane sum
                        // adds the two terms and the tokens at once
                        const int64_t n = row0 + 4 * g;
#pragma unroll
                        for (int o = 0; o < QP; ++o)
                            if (o < q_used) {
                                q_f32x4 sum;
#pragma unroll
                                for (int v = 0; v < 4; ++v) {
                                    float x = ep[0][v] * acc[o][v];
                                    x += __shfl_xor(x, 1);
                                    x += __shfl_xor(x, 2);
                                    x += __shfl_xor(x, 4);
                                    x += __shfl_xor(x, 8);
                                    sum[v] = x * scale;
                                }
                                if (rl == 0)
#pragma unroll
                                    for (int v = 0; v < 4; ++v)
                                        if (n + v < rows)
                                            reinterpret_cast<float*>(out)[(((int64_t)o * rows + n + v) * G) + grp] = sum[v];
                            }
                    }
#pragma unroll
                    for (int i = 0; i < QP; ++i) acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        stage_store(buf ^ 1);
        __syncthreads();  // chunk c + 1 is visible; everyone is done reading chunk c
    }

    if (GROUPED && MODE == STREAM_DALPHA) return;  // every group was stored at its end
    if (GROUPED && MODE == STREAM_FWD) {            // continue below with y in place of the plane sums
        acc[0] = yv;
#pragma unroll
        for (int v = 0; v < 4; ++v) ep[0][v] = 1.f;
#pragma unroll
        for (int i = 1; i < QP; ++i) {
            acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v) ep[i][v] = 0.f;
        }
    }
    stream_finish<MODE, QP, TWO>(acc, ep, reinterpret_cast<float*>(lds), KW, kp, RW, rtile, lane, row0, rows, tok, tok_live,
                                 q_used, scale, out);
}

template <int MODE, int QP, bool TWO, bool GROUPED, int KW, bool EXACT, bool TILED>
__global__ __launch_bounds__(512) void stream_lds_kernel(const uint32_t* __restrict__ planes,
                                                          const unsigned char* __restrict__ xq,
                                                          const unsigned char* __restrict__ sq,
                                                          const float* __restrict__ alpha,
                                                          const bf16_t* __restrict__ dy, void* __restrict__ out,
                                                          int64_t T, int64_t rows, int64_t cw, int q_used, float scale,
                                                          int spp, int64_t segs, int gsegs, int G, int64_t xq_plane,
                                                          int64_t sq_plane, uint32_t seg_magic, int segs_n) {
    stream_lds_body<MODE, QP, TWO, GROUPED, KW, EXACT, TILED>(planes, xq, sq, alpha, dy, out, T, rows, cw, q_used, scale, spp,
                                                              segs, gsegs, G, xq_plane, sq_plane, seg_magic, segs_n,
                                                              blockIdx.x, blockIdx.y);
}

// ---------------------------------------------------------------------------------------------------------
// Forward / scale gradient when a wave has only one or two segments (small layers: the call is bound by launch and
// memory latency, not by bandwidth): the wave re-codes the activations of its own segment into LDS itself, so the
// call is ONE kernel and needs no workspace.  The re-coding costs about 480 vector-ALU operations per lane and
// segment (it is repeated by every row tile), which is why larger layers keep the separate pre-kernel.
// One workgroup = one row tile; its W waves split the segments.  LDS: W wave-private staging areas
// ([4 instructions][halves][2 KiB] + [halves][256 B] scales), reused for the cross-wave sum at the end.
// gsegs == 0: row-wise scales; else groups of gsegs segments (every wave owns whole groups).
template <int MODE, int QP, bool TWO>
__global__ __launch_bounds__(512) void stream_fused_kernel(const uint32_t* __restrict__ planes,
                                                            const bf16_t* __restrict__ act,
                                                            const float* __restrict__ alpha,
                                                            const bf16_t* __restrict__ dy, void* __restrict__ out,
                                                            int64_t T, int64_t rows, int64_t cw, int q_used, float scale,
                                                            int segs_per_wave, int64_t segs, int gsegs, int G) {
    static_assert(MODE != STREAM_DX, "forward and scale gradient only");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int H = TWO ? 2 : 1;
    constexpr int WST = 4 * H * QBLK + H * QSCL;  // staging bytes of one wave
    constexpr int NU = 2 * H;                     // re-coding units per lane and segment (128 H live units)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int rl = lane & 15, g = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * 16;
    const int64_t t0 = (int64_t)blockIdx.y * 16;
    const int64_t C = cw * 32;
    const bool grouped = gsegs > 0;
    unsigned char* wst = lds + wave * WST;

    q_f32x4 acc[QP];
#pragma unroll
    for (int i = 0; i < QP; ++i) acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
    const uint32_t cw32 = (uint32_t)cw;
    uint32_t roff;
    {
        int64_t rr = row0 + rl;
        rr = rr < rows ? rr : rows - 1;  // rows beyond the matrix give outputs that are never stored
        roff = (uint32_t)(rr * cw);
    }
    const int64_t plane_stride = rows * cw;
    const int tcol = TWO ? rl : (rl & 7);
    const bool tok_live = (t0 + tcol) < T;
    const int64_t tok = tok_live ? t0 + tcol : T - 1;
    float ep[QP][4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        int64_t n = row0 + 4 * g + v;
        const bool n_live = n < rows;
        n = n_live ? n : rows - 1;
        if (MODE == STREAM_FWD) {
#pragma unroll
            for (int i = 0; i < QP; ++i) ep[i][v] = (!grouped && i < q_used) ? alpha[(int64_t)i * rows + n] : 0.f;
        } else {
            ep[0][v] = (tok_live && n_live) ? bf16_to_f32(dy[tok * rows + n]) : 0.f;
        }
    }
    q_f32x4 yv = {0.f, 0.f, 0.f, 0.f};
    float ga[QP][4];  // group-wise forward: scales of the current group

    const int seg_begin = wave * segs_per_wave;
    int seg_end = seg_begin + segs_per_wave;
    seg_end = seg_end < (int)segs ? seg_end : (int)segs;
    for (int seg = seg_begin; seg < seg_end; ++seg) {
        // activations of this segment first (loads return in issue order and these are needed first), then the planes
        q_u32x4 raw[NU][4];
        bool live[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int uu = lane + 64 * u;
            const int Gb = uu & 3, tl = (uu >> 2) & (8 * H - 1), j = uu >> (TWO ? 6 : 5);
            const int64_t t = t0 + tl, word = (int64_t)seg * 16 + 4 * Gb + j;
            live[u] = (t < T) && (word * 32 < C);
            const q_u32x4* src = reinterpret_cast<const q_u32x4*>(act + (live[u] ? t * C + word * 32 : 0));
#pragma unroll
            for (int b = 0; b < 4; ++b) raw[u][b] = src[b];  // a dead unit reads the first 64 bytes of act (in bounds)
        }
        uint32_t bits[QP][4];
        {
            uint32_t w0 = (uint32_t)seg * 16u + 4u * (uint32_t)g;
#pragma unroll
            for (int i = 0; i < QP; ++i) {
                const uint32_t* pl = planes + (int64_t)(i < q_used ? i : q_used - 1) * plane_stride;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    uint32_t wj = w0 + (uint32_t)jj;
                    wj = wj < cw32 ? wj : cw32 - 1u;  // columns beyond C meet zero activations
                    bits[i][jj] = pl[roff + wj];
                }
            }
        }
        if (grouped && MODE == STREAM_FWD && (seg == seg_begin || seg % gsegs == 0)) {
            const int grp = seg / gsegs;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int64_t n = row0 + 4 * g + v;
                n = n < rows ? n : rows - 1;
#pragma unroll
                for (int i = 0; i < QP; ++i) ga[i][v] = (i < q_used) ? alpha[((int64_t)i * rows + n) * G + grp] : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int uu = lane + 64 * u;
            const int Gb = uu & 3, tl = (uu >> 2) & (8 * H - 1), j = uu >> (TWO ? 6 : 5);
            float v[32];
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[8 * b + 2 * e] = live[u] ? __uint_as_float(raw[u][b][e] << 16) : 0.f;
                    v[8 * b + 2 * e + 1] = live[u] ? __uint_as_float(raw[u][b][e] & 0xFFFF0000u) : 0.f;
                }
            recode_unit(v, tl, Gb, j, !TWO, wst + j * H * QBLK, wst + 4 * H * QBLK);
        }
        // the staging area is private to the wave: LDS operations of one wave complete in issue order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int sv[H];
#pragma unroll
        for (int h = 0; h < H; ++h) sv[h] = *reinterpret_cast<const int*>(wst + 4 * H * QBLK + h * QSCL + lane * 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q_i32x8 bo[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const unsigned char* bp = wst + (j * H + h) * QBLK + lane * 16;
                const q_u32x4 lo = *reinterpret_cast<const q_u32x4*>(bp);
                const q_u32x4 hi = *reinterpret_cast<const q_u32x4*>(bp + QBLK / 2);
                bo[h] = q_i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            }
#pragma unroll
            for (int i = 0; i < QP; ++i) {
                q_i32x8 aop;
                expand_one(bits[i][j], aop);
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    // the instruction picks byte j of the scale register (its op_sel): j must be a constant
                    if (j == 0)
                        acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo[h], acc[i], 4, 0, 0, 127, 0, sv[h]);
                    else if (j == 1)
                        acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo[h], acc[i], 4, 0, 0, 127, 1, sv[h]);
                    else if (j == 2)
                        acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo[h], acc[i], 4, 0, 0, 127, 2, sv[h]);
                    else
                        acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aop, bo[h], acc[i], 4, 0, 0, 127, 3, sv[h]);
                }
            }
        }
        if (grouped && ((seg + 1) % gsegs == 0 || seg + 1 == seg_end)) {  // uniform: a scale group ends
            const int grp = seg / gsegs;
            if (MODE == STREAM_FWD) {
#pragma unroll
                for (int i = 0; i < QP; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) yv[v] += ga[i][v] * acc[i][v];
            } else {
                const int64_t n = row0 + 4 * g;
#pragma unroll
                for (int o = 0; o < QP; ++o)
                    if (o < q_used) {
                        q_f32x4 sum;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            float x = ep[0][v] * acc[o][v];
                            x += __shfl_xor(x, 1);
                            x += __shfl_xor(x, 2);
                            x += __shfl_xor(x, 4);
                            x += __shfl_xor(x, 8);
                            sum[v] = x * scale;
                        }
                        if (rl == 0)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                if (n + v < rows) reinterpret_cast<float*>(out)[(((int64_t)o * rows + n + v) * G) + grp] = sum[v];
                    }
            }
#pragma unroll
            for (int i = 0; i < QP; ++i) acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
        }
        // the next segment overwrites the staging area: its reads above are done (same wave, issue order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (grouped && MODE == STREAM_DALPHA) return;  // every group was stored at its end
    if (grouped && MODE == STREAM_FWD) {            // continue with y in place of the plane sums
        acc[0] = yv;
#pragma unroll
        for (int v = 0; v < 4; ++v) ep[0][v] = 1.f;
#pragma unroll
        for (int i = 1; i < QP; ++i) {
            acc[i] = q_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v) ep[i][v] = 0.f;
        }
    }
    if (W > 1) __syncthreads();  // the cross-wave sum reuses the staging areas
    stream_finish<MODE, QP, TWO>(acc, ep, reinterpret_cast<float*>(lds), W, wave, 1, 0, lane, row0, rows, tok, tok_live,
                                 q_used, scale, out);
}

}  // namespace bcq
