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
//      4 x 4 MFMA tiles of v_mfma_f32_32x32x16_bf16.  The activation tile goes global -> LDS directly
//      (buffer_load ... lds, three stages in flight, 16-byte chunks XOR-swizzled by row so that the fragment
//      reads are bank-conflict free); the weight fragments are loaded straight from the workspace into
//      registers (1 KiB coalesced per wave load), so LDS carries only the activations.
#include "bcq_internal.h"
#include <type_traits>

namespace bcq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;


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
// Workgroup -> tile mapping.  Consecutive workgroup ids go round-robin over the 8 XCDs, each with its own L2.
// The tile grid is cut into super-blocks of a x b tiles; all workgroups that run on one XCD at the same time
// belong to one super-block, so that XCD's L2 fetches only a/tiles_m of the first operand and b/tiles_n of the
// second instead of a whole operand.
struct TileMap {
    int tiles_m, tiles_n, a, b, sbm, sbn;
};

__device__ __forceinline__ bool map_tile(const TileMap& tm, int copies, int bid, int& copy, int& tile_m, int& tile_n) {
    const int xcd = bid & 7, slot = bid >> 3;
    const int per = tm.a * tm.b;
    const int sbg = (slot / per) * 8 + xcd;  // super-block index over all copies of the tile grid
    const int within = slot % per;
    const int nsb = tm.sbm * tm.sbn;
    if (sbg >= nsb * copies) return false;
    copy = sbg / nsb;
    const int sb = sbg % nsb;
    tile_m = (sb % tm.sbm) * tm.a + within % tm.a;
    tile_n = (sb / tm.sbm) * tm.b + within / tm.a;
    return tile_m < tm.tiles_m && tile_n < tm.tiles_n;
}

// Super-block shape: about `cap` tiles (what one XCD runs concurrently), minimising the bytes both operands bring
// in, a * cost_m + b * cost_n.  Returns the number of workgroups to launch.
static inline unsigned make_tile_map(int tiles_m, int tiles_n, int copies, int cap, double cost_m, double cost_n,
                                     TileMap* out) {
    // never make a super-block larger than one XCD's share of all tiles (copies = independent tile grids, e.g.
    // token slices), or some XCDs would get no work
    const long share = ((long)tiles_m * tiles_n * copies + 7) / 8;
    if (cap > share) cap = (int)(share < 1 ? 1 : share);
    int best_a = 1, best_b = 1;
    double best = 1e300;
    for (int a = 1; a <= tiles_m && a <= cap; ++a) {
        for (int b = 1; b <= tiles_n && a * b <= cap; ++b) {
            const int sbm = (tiles_m + a - 1) / a, sbn = (tiles_n + b - 1) / b;
            const long nsb = (long)sbm * sbn * copies;
            // work really done per XCD round, including empty slots of ragged super-blocks and idle XCDs
            const double slots = (double)((nsb + 7) / 8) * 8 * a * b;
            const double waste = slots / ((double)tiles_m * tiles_n * copies);
            const double per_tile = (a * cost_m + b * cost_n) / ((double)a * b);
            const double score = per_tile * waste * waste * waste;  // balance first, then operand traffic
            if (score < best) {
                best = score;
                best_a = a;
                best_b = b;
            }
        }
    }
    out->tiles_m = tiles_m;
    out->tiles_n = tiles_n;
    out->a = best_a;
    out->b = best_b;
    out->sbm = (tiles_m + best_a - 1) / best_a;
    out->sbn = (tiles_n + best_b - 1) / best_b;
    const int nsb = out->sbm * out->sbn * copies;
    return (unsigned)(((nsb + 7) / 8) * 8 * best_a * best_b);
}

// ---------------------------------------------------------------------------------------------------------
// 32 fp32 sums -> 16 bf16 pairs -> four 16-byte fragment slots of 8 contraction indices each
__device__ __forceinline__ void store_word_frags(const float (&s)[32], u32x4* __restrict__ frag, int64_t block0, int c) {
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) {
        u32x4 v;
#pragma unroll
        for (int p = 0; p < 4; ++p) v[p] = pack_bf16x2(s[8 * gg + 2 * p], s[8 * gg + 2 * p + 1]);
        frag[(block0 + (gg >> 1)) * 64 + c + 32 * (gg & 1)] = v;
    }
}

// expand for the forward: columns of the GEMM = rows n of W, contraction = k.
// thread = (c = n % 32, one packed word = 32 columns k) -> four 16-byte fragment slots.
__global__ __launch_bounds__(256) void expand_fwd_kernel(const uint32_t* __restrict__ packed,
                                                         const float* __restrict__ alpha, int64_t N, int64_t K,
                                                         int64_t g, int q, int64_t R16 /* padded K / 16 */,
                                                         u32x4* __restrict__ frag) {
    const int c = threadIdx.x & 31;
    const int64_t ct = blockIdx.x;
    const int64_t n = ct * 32 + c;
    const int64_t Kw = K / 32;
    const int64_t w = (int64_t)blockIdx.y * 8 + (threadIdx.x >> 5);
    if (w * 2 >= R16) return;
    const bool live = (n < N) && (w < Kw);
    const int64_t G = K / g, grp = live ? (w * 32) / g : 0;  // a packed word lies in one scale group (g % 32 == 0)
    float s[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) s[e] = 0.f;
    for (int i = 0; i < q; ++i) {
        const float a = live ? alpha[((int64_t)i * N + n) * G + grp] : 0.f;
        const uint32_t bits = live ? packed[((int64_t)i * N + n) * Kw + w] : 0u;
#pragma unroll
        for (int e = 0; e < 32; ++e) s[e] += ((bits >> e) & 1u) ? a : -a;
    }
    store_word_frags(s, frag, ct * R16 + 2 * w, c);
}

// expand for the input gradient: columns of the GEMM = columns k of W, contraction = n.  Reads the transposed
// twin when the caller has one (one word = 32 consecutive n of this thread's column), else the canonical words
// (the 32 lanes of a column tile share a word and each takes its own bit).  The scales of the block's 256 rows
// pass through LDS.
template <bool TWIN>
__global__ __launch_bounds__(256) void expand_bwd_kernel(const uint32_t* __restrict__ planes,
                                                         const float* __restrict__ alpha, int64_t N, int64_t K,
                                                         int64_t g, int q, int64_t R16 /* padded N / 16 */,
                                                         u32x4* __restrict__ frag) {
    __shared__ float sa[8][256];
    const int c = threadIdx.x & 31, vl = threadIdx.x >> 5;
    const int64_t ct = blockIdx.x;  // K / 32 column tiles, exactly one packed word wide
    const int64_t Kw = K / 32, Nw = N / 32;
    const int64_t n_blk = (int64_t)blockIdx.y * 256;
    const int64_t G = K / g, grp = (ct * 32) / g;  // the 32 columns of this block share one scale group
    for (int i = 0; i < q; ++i) {
        const int64_t n = n_blk + threadIdx.x;
        sa[i][threadIdx.x] = (n < N) ? alpha[((int64_t)i * N + n) * G + grp] : 0.f;  // rows beyond N expand to zero
    }
    __syncthreads();
    const int64_t v = (int64_t)blockIdx.y * 8 + vl;  // word index along n
    if (v * 2 >= R16) return;
    const int64_t k = ct * 32 + c;
    float s[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) s[e] = 0.f;
    for (int i = 0; i < q; ++i) {
        uint32_t bits = 0u;
        if (TWIN) {
            bits = (v < Nw) ? planes[((int64_t)i * K + k) * Nw + v] : 0u;
        } else {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const int64_t n = v * 32 + e;
                const uint32_t wv = (n < N) ? planes[((int64_t)i * N + n) * Kw + ct] : 0u;
                bits |= ((wv >> c) & 1u) << e;
            }
        }
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const float a = sa[i][vl * 32 + e];
            s[e] += ((bits >> e) & 1u) ? a : -a;
        }
    }
    store_word_frags(s, frag, ct * R16 + 2 * v, c);
}

// ---------------------------------------------------------------------------------------------------------
// C[M][NC] = A[M][R] * Bfrag, A row-major bf16 with leading dimension lda, Bfrag in fragment order with R16
// slices per column tile (R16 * 16 >= R, a multiple of 128), C row-major bf16 with leading dimension ldc.
// Workgroup tile (64 TM) x (64 TN), 4 waves in a 2 x 2 grid, each wave TM x TN MFMA tiles.
// The weight fragment is the first MFMA operand, so one lane ends up with 4 consecutive output columns of
// one token.  Nothing branches on the ragged edges: activation rows beyond M and bytes beyond the end of A come
// back as zeros from the buffer range check, contraction indices beyond R meet zero weights, and column tiles
// beyond NC are clamped to the last valid tile (their products are never stored).
template <int TM, int TN>
struct GemmCfg {
    static constexpr int BMT = 64 * TM, BNT = 64 * TN;
    static constexpr int BKC = (TM * TN <= 2) ? 128 : 64;      // contraction per K-step: 64-token tiles take longer steps
    static constexpr int KS = BKC / 16;                        // 16-slices per K-step
    static constexpr int ROWB = BKC * 2;                       // LDS row of the activation tile (8 or 16 swizzled chunks of 16 B)
    static constexpr int STAGE_B = BMT * ROWB;                 // one activation stage
    static constexpr int NST = 3;                              // stages in flight
    static constexpr int EPI_ROWB = 64 * TN + 8;               // epilogue row: 32 TN columns of bf16 + pad
    static constexpr int EPI_B = 4 * 64 * EPI_ROWB;            // 4 waves x 64 tokens
    static constexpr int LDS_B = (NST * STAGE_B > EPI_B) ? NST * STAGE_B : EPI_B;
    static constexpr int OCC = (TM * TN >= 16) ? 1 : 2;
};

template <int TM, int TN>
__global__ __launch_bounds__(256, (TM * TN >= 16 ? 1 : 2)) void gemm_kernel(
    const bf16_t* __restrict__ A, int64_t lda, const u32x4* __restrict__ Bfrag, bf16_t* __restrict__ C, int64_t ldc,
    int64_t M, int64_t NC, int64_t R, int64_t R16, TileMap tmap) {
#if defined(__HIP_DEVICE_COMPILE__)  // the buffer-resource builtins exist in the device pass only
    using Cfg = GemmCfg<TM, TN>;
    constexpr int STAGE_B = Cfg::STAGE_B, ROWB = Cfg::ROWB, KS = Cfg::KS, BKC = Cfg::BKC, NST = Cfg::NST;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps descriptors and LDS bases scalar
    const int wm = wave >> 1, wn = wave & 1;

    int tile_m, tile_n, copy_unused;
    if (!map_tile(tmap, 1, blockIdx.x, copy_unused, tile_m, tile_n)) return;  // padding workgroup of the last round
    const int64_t m0 = (int64_t)tile_m * Cfg::BMT, n0 = (int64_t)tile_n * Cfg::BNT;
    const int64_t ct_count = (NC + 31) / 32;

    f32x16 acc[TN][TM];  // [weight tile][token tile]
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Activation tile: global -> LDS without passing registers (buffer_load ... lds, 16 B per lane).  One wave
    // instruction fills 1 KiB of LDS = RPB tile rows of CPR chunks; lane l lands in row l / CPR, slot l % CPR and
    // fetches the chunk that the swizzle assigns to that slot, so the fragment reads (16 lanes: one chunk index of
    // 16 consecutive rows) are bank-conflict free without padding:
    //   128-byte rows: slot = chunk ^ (r & 7) ^ ((r >> 3) & 1)   (rows r and r + 8 lie four passes over the 64
    //                                                              banks apart and would meet in the same banks)
    //   256-byte rows: slot = chunk ^ (r & 15)                    (every row starts at bank 0)
    // Each wave has one buffer descriptor, based at the first of its 16 TM rows and ending at the end of A, so
    // rows beyond M read zeros; the per-lane offset is loop invariant up to the swizzle term of the row group
    // (NV variants), the row group and the K-step advance through the scalar offset (below 2^31 because
    // lda < 2^24, checked by the host).
    constexpr int CPR = ROWB / 16;             // chunks per row
    constexpr int RPB = 64 / CPR;              // rows per wave instruction
    constexpr int NDMA = Cfg::BMT / RPB / 4;   // wave instructions per wave and stage
    constexpr int NV = (CPR == 8) ? 2 : 4;     // distinct swizzle terms of a row group: (j & 1) or (j & 3) << 2
    static_assert(CPR == 8 || CPR == 16, "128- or 256-byte rows");
    static_assert(NDMA % NV == 0, "the row-group term depends on the instruction index only");
    const int64_t steps = R16 * 16 / BKC;
    const int64_t last = steps - 1;
    const int64_t wrow0 = m0 + wave * NDMA * RPB;
    const int64_t left = (M - wrow0) * lda * 2;  // bytes from this wave's first row to the end of A (lda >= R)
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(A + (left > 0 ? wrow0 * lda : 0)), 0, (int)(left > 0 ? (left < 0x7fffffffll ? left : 0x7fffffffll) : 0),
        0x00020000);
    const int drow = lane / CPR, dslot = lane % CPR;
    uint32_t voff[NV], voff_tail[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int achunk = dslot ^ drow ^ ((CPR == 8) ? v : (v << 2));
        voff[v] = (uint32_t)(drow * lda * 2 + achunk * 16);
        // the last K-step may reach beyond R: its chunks are clamped into the row (they meet zero weights)
        int64_t k_tail = last * BKC + achunk * 8;
        k_tail = k_tail < R - 8 ? k_tail : R - 8;
        voff_tail[v] = (uint32_t)(drow * lda * 2 + k_tail * 2);
    }
    const int group_b = (int)(RPB * lda * 2);   // bytes between two row groups
    auto dma_a = [&](int64_t step, int stage) {
        const bool tail = step >= last;
        uint32_t vo[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) vo[v] = tail ? voff_tail[v] : voff[v];
        const int so = tail ? 0 : (int)(step * BKC * 2);
#pragma unroll
        for (int j = 0; j < NDMA; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc, (void __attribute__((address_space(3)))*)(smem + stage * STAGE_B + (wave * NDMA + j) * 1024), 16,
                vo[j % NV], so + j * group_b, 0, 0);
    };

    // weight fragments of this wave: column tiles ct0 .. ct0+TN-1, straight from global memory into registers
    const int64_t ct0 = (n0 + wn * 32 * TN) / 32;
    const u32x4* bptr[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int64_t ct = ct0 + j;
        ct = ct < ct_count ? ct : ct_count - 1;
        bptr[j] = Bfrag + ct * R16 * 64 + lane;
    }
    u32x4 b[KS][TN];  // [kk][j]; slot kk is refilled for the next K-step right after its MFMAs are issued
    auto load_b = [&](int kk, int64_t step) {
#pragma unroll
        for (int j = 0; j < TN; ++j) b[kk][j] = bptr[j][(step * KS + kk) * 64];
    };

    // Fragment reads are inline assembly: the compiler guards every LDS read it sees that may alias a direct-to-LDS
    // load with a wait for ALL outstanding loads.  wait_x / wait_stage tie the fragment registers to an explicit
    // s_waitcnt, so no consumer can be scheduled above the wait.
    u32x4 xf[2][TM];  // activation fragments of two consecutive 16-slices
    // lane (r = lane % 32, h = lane / 32) takes chunk 2 kk + h of row wm * 32 TM + 32 i + r
    const int xrow = wm * 32 * TM + (lane & 31);
    const int xswz = (CPR == 8) ? ((xrow & 7) ^ ((xrow >> 3) & 1)) : (xrow & 15);  // the same for rows 32 i further on
    uint32_t xoff[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
        xoff[kk] = (uint32_t)(xrow * ROWB + (((2 * kk + (lane >> 5)) ^ xswz) * 16));
    auto read_x = [&](int stage, int kk) {
        const uint32_t addr = xoff[kk] + (uint32_t)(stage * STAGE_B);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(xf[kk & 1][i]) : "v"(addr), "n"(i * 32 * ROWB));
    };
    // gfx9 s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
    auto wait_regs = [&](int kk, auto imm) {
        constexpr int IMM = decltype(imm)::value;
        u32x4* f = xf[kk & 1];
        if constexpr (TM == 4)
            asm volatile("s_waitcnt %4" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(IMM) : "memory");
        else if constexpr (TM == 2)
            asm volatile("s_waitcnt %2" : "+v"(f[0]), "+v"(f[1]) : "n"(IMM) : "memory");
        else
            asm volatile("s_waitcnt %1" : "+v"(f[0]) : "n"(IMM) : "memory");
    };
    // the fragments of slice kk are usable once only the TM reads of the following slice are outstanding
    auto wait_x = [&](int kk) { wait_regs(kk, std::integral_constant<int, 63 | (3 << 14) | (7 << 4) | (TM << 8)>()); };
    // Before the barrier of a K-step: every LDS read of this wave has returned (the stage may be refilled after
    // the barrier) and this wave's part of the next stage has landed.  That stage was requested a whole K-step
    // ago and loads complete in order, so it is enough that at most the loads issued during this K-step (the
    // fill and KS - 1 slices of weights) remain in flight - which the coming MFMAs need anyway.
    auto wait_stage = [&](int kk) {
        constexpr int MAXV = NDMA + (KS - 1) * TN;
        wait_regs(kk, std::integral_constant<int, (MAXV & 15) | ((MAXV >> 4) << 14) | (7 << 4) | (0 << 8)>());
    };
    auto mfma_slice = [&](int kk) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(b[kk][j]), as_bf16x8(xf[kk & 1][i]),
                                                                    acc[j][i], 0, 0, 0);
    };

    // Prologue: stages 0 .. NST-2 requested, then the weights of step 0.  These first weight loads are inline
    // assembly as well, so that they are issued HERE, in flight together with the activation stages (the
    // compiler would sink them below the barrier); tie_b makes them usable.
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) dma_a(p, p);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(b[kk][j]) : "v"(bptr[j] + kk * 64));
    {
        constexpr int MAXV = (NST - 2) * NDMA + KS * TN;  // stage 0 has landed (this wave's part)
        asm volatile("s_waitcnt %0" ::"n"((MAXV & 15) | ((MAXV >> 4) << 14) | (7 << 4) | (15 << 8)) : "memory");
    }
    __builtin_amdgcn_s_barrier();
    read_x(0, 0);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {  // all prologue loads have returned
        u32x4* f = b[kk];
        if constexpr (TN == 4)
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3])::"memory");
        else if constexpr (TN == 2)
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(f[0]), "+v"(f[1])::"memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(f[0])::"memory");
    }

    // One K-step = KS 16-slices.  At its start the stage NST - 1 steps ahead is requested into the buffer that was
    // read during the previous step.  Per slice: issue the LDS reads of the next slice, the MFMAs of this one,
    // then refill this slice's weight registers for the next K-step (a full step of latency cover).  The
    // hand-over to the next stage (wait, barrier, first fragment read) sits BEFORE the MFMAs of the last slice,
    // whose operands are already in registers, so the matrix pipe stays busy across the barrier.
    int st = 0;  // stage of step s
    for (int64_t s = 0; s < steps; ++s) {
        const int64_t nx = s < last ? s + 1 : last;
        const int st_next = (st + 1 == NST) ? 0 : st + 1;
        const int st_fill = (st == 0) ? NST - 1 : st - 1;
        dma_a(s + NST - 1, st_fill);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KS - 1; ++kk) {
            read_x(st, kk + 1);
            wait_x(kk);
            mfma_slice(kk);
            load_b(kk, nx);
            __builtin_amdgcn_sched_barrier(0);
        }
        wait_stage(KS - 1);
        __builtin_amdgcn_s_barrier();
        read_x(st_next, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_slice(KS - 1);
        load_b(KS - 1, nx);
        __builtin_amdgcn_sched_barrier(0);
        st = st_next;
    }
    // the clamped requests of the last steps are still writing LDS, and the last fragment read is in flight
    wait_regs(0, std::integral_constant<int, 0 | (7 << 4)>());

    // epilogue: acc register 4g+e of lane l is weight column 8g + 4*(l/32) + e, token l%32 of its 32 x 32 tile.
    // Pass the tile through LDS (64 tokens per wave at a time) so that global stores are 16 B per lane and
    // whole rows of 64 TN bytes are contiguous.
    constexpr int EROW = Cfg::EPI_ROWB;
    const bool vec_ok = (ldc % 8 == 0);
    if (vec_ok) {
        unsigned char* ew = smem + wave * 64 * EROW;
        constexpr int CH = 4 * TN;        // 16-byte chunks per row
        constexpr int RPI = 64 / CH;      // rows per store instruction
        __syncthreads();  // every wave is done with the activation stages; from here on a wave touches only its own region
#pragma unroll
        for (int pass = 0; pass < (TM + 1) / 2; ++pass) {
            // LDS executes one wave's instructions in order: between its own writes and reads of its region only the
            // compiler has to keep the order
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
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
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
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
#endif
}

static inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

constexpr int RPAD = 128;  // contraction padding of the expanded operand: the longest K-step of any tile configuration
size_t mfma_fwd_workspace(int64_t N, int64_t K) { return (size_t)(round_up(N, 32) * round_up(K, RPAD) * 2); }
size_t mfma_bwd_input_workspace(int64_t N, int64_t K) { return (size_t)(round_up(K, 32) * round_up(N, RPAD) * 2); }

template <int TM, int TN>
static hipError_t launch_gemm_cfg(const bf16_t* A, int64_t lda, const u32x4* frag, bf16_t* C, int64_t ldc, int64_t M,
                                  int64_t NC, int64_t R, int64_t R16, hipStream_t st) {
    using Cfg = GemmCfg<TM, TN>;
    static LdsLimit limit;
    hipError_t e = limit.ensure((const void*)gemm_kernel<TM, TN>, Cfg::LDS_B);
    if (e != hipSuccess) return e;
    const int tiles_m = (int)((M + Cfg::BMT - 1) / Cfg::BMT), tiles_n = (int)((NC + Cfg::BNT - 1) / Cfg::BNT);
    TileMap tmap;
    const unsigned wgs = make_tile_map(tiles_m, tiles_n, 1, 32 * Cfg::OCC, (double)Cfg::BMT, (double)Cfg::BNT, &tmap);
    BCQ_LAUNCH((gemm_kernel<TM, TN>), dim3(wgs), dim3(256), Cfg::LDS_B, st, A, lda, frag, C, ldc, M, NC, R, R16,
                       tmap);
    return hipGetLastError();
}

// Tile choice from measurements on the workloads' shapes: 256 x 256 tiles (one workgroup per compute unit, the best
// MFMA rate) when they fill at least 80 % of their last round on the 256 compute units, else 128 x 128 tiles
// (two or three resident per compute unit, so ragged tile counts level out).  256 x 128 never won by more than 6 %.
static hipError_t launch_gemm(const bf16_t* A, int64_t lda, const u32x4* frag, bf16_t* C, int64_t ldc, int64_t M,
                              int64_t NC, int64_t R, int64_t R16, hipStream_t st) {
    const int64_t tiles = ((M + 255) / 256) * ((NC + 255) / 256);
    const int64_t rounds = (tiles + 255) / 256;
    if (tiles * 10 >= rounds * 256 * 8) return launch_gemm_cfg<4, 4>(A, lda, frag, C, ldc, M, NC, R, R16, st);
    // few tokens (a few hundred): 128 x 128 tiles would leave compute units without work; 64-token tiles fill them
    const int64_t tiles128 = ((M + 127) / 128) * ((NC + 127) / 128);
    if (tiles128 < 192) {
        const int64_t tiles_64x128 = ((M + 63) / 64) * ((NC + 127) / 128);
        if (tiles_64x128 >= 192) return launch_gemm_cfg<1, 2>(A, lda, frag, C, ldc, M, NC, R, R16, st);
        return launch_gemm_cfg<1, 1>(A, lda, frag, C, ldc, M, NC, R, R16, st);
    }
    return launch_gemm_cfg<2, 2>(A, lda, frag, C, ldc, M, NC, R, R16, st);
}

hipError_t launch_fwd_mfma(const uint32_t* packed, const float* alpha, const void* x, int64_t T, int64_t N,
                           int64_t K, int64_t g, int q, void* y, void* workspace, hipStream_t st) {
    const int64_t R16 = round_up(K, RPAD) / 16;
    const int64_t ct = (N + 31) / 32;
    dim3 grid((unsigned)ct, (unsigned)((R16 / 2 + 7) / 8));
    BCQ_LAUNCH(expand_fwd_kernel, grid, dim3(256), 0, st, packed, alpha, N, K, g, q, R16, (u32x4*)workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_gemm((const bf16_t*)x, K, (const u32x4*)workspace, (bf16_t*)y, N, T, N, K, R16, st);
}

hipError_t launch_bwd_input_mfma(const uint32_t* packed, const uint32_t* packed_t, const float* alpha, const void* dy,
                                 int64_t T, int64_t N, int64_t K, int64_t g, int q, void* dx, void* workspace,
                                 hipStream_t st) {
    const int64_t R16 = round_up(N, RPAD) / 16;
    dim3 grid((unsigned)(K / 32), (unsigned)((R16 / 2 + 7) / 8));
    if (packed_t && N % 32 == 0)
        BCQ_LAUNCH(expand_bwd_kernel<true>, grid, dim3(256), 0, st, packed_t, alpha, N, K, g, q, R16,
                           (u32x4*)workspace);
    else
        BCQ_LAUNCH(expand_bwd_kernel<false>, grid, dim3(256), 0, st, packed, alpha, N, K, g, q, R16,
                           (u32x4*)workspace);
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
// Both MFMA operands need the token index innermost, which neither activation has in memory.  LDS fragment
// reads are the scarce resource of a compute unit (a 16-byte-per-lane read instruction takes ~16 clocks), so
// only ONE operand may pass through LDS:
//   1. transpose_frag_kernel rewrites the smaller activation (x if K <= N, else dy) into MFMA fragment order
//      with the token index innermost (8 x 8 register transposes); its fragments are then loaded straight
//      from global memory, 1 KiB coalesced per wave load, exactly like the expanded weights of the forward.
//   2. dalpha_kernel: 256 (k) x 256 (n) tile of G^T for one slice of the tokens; 4 waves in a 2 x 2 grid, each
//      128 x 128 = 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 with X^T as first and dY^T as second operand, so a
//      lane holds one n and 16 k of every tile.  The other activation goes global -> registers -> 8 x 8
//      transpose (32 v_perm) -> XOR-swizzled LDS tile [column][64 tokens]; writes and fragment reads are
//      bank-conflict free.  The epilogue forms the signed sums over k for every trained plane.
//   3. dalpha_reduce_kernel adds the partial sums of all (token slice, k tile) pairs in a fixed order (no
//      floating-point atomics, bit-reproducible).
constexpr int DA_TILE = 256;               // k and n extent of a workgroup tile
constexpr int DA_STAGE = DA_TILE * 128;    // bytes per LDS stage: 256 columns x 64 tokens x 2 B

__device__ __forceinline__ int da_swz(int col, int chunk) { return col * 128 + ((chunk ^ (col & 7) ^ ((col >> 3) & 7)) << 4); }

// 8 x 8 transpose of 16-bit elements: in[r] holds row r (8 elements), out[c] holds column c.
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int w = 0; w < 4; ++w)
            out[c][w] = __builtin_amdgcn_perm(in[2 * w + 1][c >> 1], in[2 * w][c >> 1], (c & 1) ? 0x07060302u : 0x05040100u);
}

// act[T][C] (row-major bf16) -> fragments with the token index innermost: for column tile ct (32 columns) and
// token slice ks (16 tokens) one 1 KiB block; lane (c % 32) + 32 g holds tokens 16 ks + 8 g .. + 7 of column c.
// Tokens >= T (up to T16 * 16) and columns >= C are written as zeros.
__global__ __launch_bounds__(256) void transpose_frag_kernel(const bf16_t* __restrict__ act, int64_t T, int64_t C,
                                                             int64_t T16, u32x4* __restrict__ frag) {
    const int cb = threadIdx.x & 15, tbl = threadIdx.x >> 4;       // 16 column blocks x 16 token blocks per group
    const int64_t c0 = ((int64_t)blockIdx.x * 16 + cb) * 8;       // first of 8 columns
    const int64_t tb = (int64_t)blockIdx.y * 16 + tbl;            // block of 8 tokens
    if (tb * 8 >= T16 * 16) return;
    u32x4 in[8], out[8];
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t t = tb * 8 + r;
        in[r] = (t < T && c0 < C) ? *reinterpret_cast<const u32x4*>(act + t * C + c0) : zero;
    }
    transpose8x8(in, out);
    const int64_t ct = c0 / 32, ks = tb >> 1;
    const int g = (int)(tb & 1);
    if (ct * 32 >= ((C + 31) / 32) * 32) return;
#pragma unroll
    for (int c = 0; c < 8; ++c) frag[(ct * T16 + ks) * 64 + (c0 % 32) + c + 32 * g] = out[c];
}

// XG: x comes as fragments from global memory and dy through LDS; otherwise the reverse.
// QT: planes summed in the epilogue (q_train rounded up to 1, 2, 3, 4 or 8; extra planes are computed, not stored).
// FINE: partial sums are kept per 32 columns k (for scale groups that are not whole 256-column tiles) instead of
//       per tile; they go to part[split][plane][n][8 tiles_k] and dalpha_reduce_fine_kernel adds each group's run.
template <bool XG, int QT, bool FINE>
__global__ __launch_bounds__(256, 1) void dalpha_kernel(const bf16_t* __restrict__ L /* activation through LDS */,
                                                        int64_t ldl, int64_t lcols,
                                                        const u32x4* __restrict__ Gfrag, int64_t T16,
                                                        const uint32_t* __restrict__ packed,
                                                        float* __restrict__ part, int64_t T, int64_t N, int64_t K,
                                                        int q_train, TileMap tmap, int splits,
                                                        int64_t tokens_per_split) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;  // wm: k half, wn: n half
    const int tiles_k = tmap.tiles_m;
    int split, tile_k, tile_n;
    if (!map_tile(tmap, splits, blockIdx.x, split, tile_k, tile_n)) return;
    const int64_t k0 = (int64_t)tile_k * DA_TILE, n0 = (int64_t)tile_n * DA_TILE;
    const int64_t t_begin = (int64_t)split * tokens_per_split;  // a multiple of 64
    const int64_t t_end = (t_begin + tokens_per_split < T) ? t_begin + tokens_per_split : T;
    const int64_t steps = (t_end - t_begin + 63) / 64;
    const int64_t step0 = t_begin / 64;

    f32x16 acc[4][4];  // [k tile][n tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // LDS-side activation: thread = (cb = column block of 8, tb = token block of 8)
    const int cb = tid & 31, tb = tid >> 5;
    int64_t lcol = (XG ? n0 : k0) + cb * 8;
    lcol = lcol < lcols - 8 ? lcol : lcols - 8;  // clamped columns only feed outputs that are never stored
    u32x4 lr[8];
    // rows of one step: uniform base (advances by 64 rows per step) + 32-bit lane offset + r rows
    const uint32_t row_b = (uint32_t)(ldl * 2);
    const uint32_t voff0 = (uint32_t)(tb * 8) * row_b + (uint32_t)(lcol * 2);
    auto load_blocks = [&](int64_t step) {
        const int64_t t0 = (step0 + step) * 64;
        const unsigned char* base = reinterpret_cast<const unsigned char*>(L + t0 * ldl);
        if (t0 + 64 <= T) {
#pragma unroll
            for (int r = 0; r < 8; ++r) lr[r] = *reinterpret_cast<const u32x4*>(base + (voff0 + (uint32_t)r * row_b));
        } else {  // last, ragged step: rows beyond T are clamped (they meet zero fragments of the other operand)
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                int64_t t = t0 + tb * 8 + r;
                t = t < T ? t : T - 1;
                lr[r] = *reinterpret_cast<const u32x4*>(L + t * ldl + lcol);
            }
        }
    };
    // column c of this thread's 8 x 8 block: 8 tokens of one column = one 16-byte LDS chunk (4 v_perm + 1 write)
    auto store_col = [&](int buf, int c) {
        u32x4 o;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            o[w] = __builtin_amdgcn_perm(lr[2 * w + 1][c >> 1], lr[2 * w][c >> 1], (c & 1) ? 0x07060302u : 0x05040100u);
        *reinterpret_cast<u32x4*>(smem + buf * DA_STAGE + da_swz(cb * 8 + c, tb)) = o;
    };
    auto store_blocks = [&](int buf) {
#pragma unroll
        for (int c = 0; c < 8; ++c) store_col(buf, c);
    };
    bf16x8 lf[2][4];
    const int lbase = (XG ? wn : wm) * 128 + (lane & 31);
    auto read_frags = [&](int buf, int kk) {
        const unsigned char* sl = smem + buf * DA_STAGE;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            lf[kk & 1][i] = *reinterpret_cast<const bf16x8*>(sl + da_swz(lbase + i * 32, kk * 2 + (lane >> 5)));
    };
    // global-side fragments of this wave: 4 column tiles
    const int64_t gct_count = ((XG ? K : N) + 31) / 32;
    const int64_t gct0 = ((XG ? k0 + wm * 128 : n0 + wn * 128)) / 32;
    const u32x4* gptr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int64_t ct = gct0 + j;
        ct = ct < gct_count ? ct : gct_count - 1;
        gptr[j] = Gfrag + (ct * T16 + step0 * 4) * 64 + lane;
    }
    u32x4 g[4][4];  // [kk][tile]
    auto load_g = [&](int kk, int64_t step) {
#pragma unroll
        for (int j = 0; j < 4; ++j) g[kk][j] = gptr[j][(step * 4 + kk) * 64];
    };
    auto mfma_one = [&](int kk, int i, int j) {
        if (XG)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(g[kk][i]), lf[kk & 1][j], acc[i][j], 0, 0, 0);
        else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lf[kk & 1][i], as_bf16x8(g[kk][j]), acc[i][j], 0, 0, 0);
    };
    auto mfma_slice = [&](int kk) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) mfma_one(kk, i, j);
    };

    // Three LDS stages.  The blocks of step s + 1 are requested during step s - 1, transposed and written into
    // their stage during the FIRST slice of step s, interleaved with its MFMAs (a stage is free from the barrier
    // that ends the step after its last read), and read from the barrier that ends step s: the global latency
    // has a whole step of cover and neither the transposes nor the LDS writes wait in front of a barrier.
    const int64_t last = steps - 1;
    load_blocks(0);
    load_g(0, 0);
    store_blocks(0);
    load_blocks(last < 1 ? last : 1);  // followed by three slices of fragment loads, as in every step of the loop
#pragma unroll
    for (int kk = 1; kk < 4; ++kk) load_g(kk, 0);
    __syncthreads();
    read_frags(0, 0);
    int stg = 0;  // stage of step s
    for (int64_t s = 0; s < steps; ++s) {
        const int64_t nx = s < last ? s + 1 : last;
        const int64_t nx2 = s + 2 < steps ? s + 2 : last;
        const int stg_next = (stg == 2) ? 0 : stg + 1;
        read_frags(stg, 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {  // two MFMAs (64 clocks of the matrix pipe) cover one column's perms and write
            mfma_one(0, c >> 1, 2 * (c & 1));
            mfma_one(0, c >> 1, 2 * (c & 1) + 1);
            store_col(stg_next, c);
            __builtin_amdgcn_sched_barrier(0);
        }
        load_g(0, nx);
        load_blocks(nx2);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 1; kk < 3; ++kk) {
            read_frags(stg, kk + 1);
            mfma_slice(kk);
            load_g(kk, nx);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 4, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        read_frags(stg_next, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_slice(3);
        load_g(3, nx);
        __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 4, 0);
        __builtin_amdgcn_sched_barrier(0);
        stg = stg_next;
    }
    __syncthreads();

    // epilogue: signed sums over this wave's 128 k for each plane; lane owns n = n_base + j*32 + lane%32.
    // All packed words of all trained planes are requested first (one memory latency instead of one per plane);
    // a sign is applied as a factor +-1.0 built from the (inverted) plane bit: shift, and-or, fused multiply-add
    // per value (the product with +-1.0 is exact, so this equals adding the signed value).
    float* red = reinterpret_cast<float*>(smem);  // [plane][wm][256 n]
    const int64_t Kw = K / 32;
    uint32_t words[QT][4][4];  // [plane][k tile][n tile], already inverted and shifted to this lane's rows
    const int64_t kt0 = (k0 + wm * 128) / 32;                      // first of this wave's four k tiles
    const bool quad = (kt0 + 3 < Kw) && ((Kw & 3) == 0);           // one aligned 16-byte load per row and plane
#pragma unroll
    for (int p = 0; p < QT; ++p) {
        const int pc = p < q_train ? p : q_train - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
            const int64_t nc = n < N ? n : N - 1;
            const uint32_t* prow = packed + ((int64_t)pc * N + nc) * Kw;
            u32x4 w4;
            if (quad) {
                w4 = *reinterpret_cast<const u32x4*>(prow + kt0);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t kt = kt0 + i < Kw ? kt0 + i : Kw - 1;  // tiles beyond K hold zero accumulators
                    w4[i] = prow[kt];
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) words[p][i][j] = ~(w4[i] >> (4 * (lane >> 5)));
        }
    }
    if (FINE) {
        // one signed sum per (plane, 32-column k tile, n): red[plane][chunk = 4 wm + i][256 n]
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float fs[QT][4];
#pragma unroll
            for (int p = 0; p < QT; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) fs[p][j] = 0.f;
            if ((k0 + wm * 128 + i * 32) < K) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int bit = 8 * (v >> 2) + (v & 3);
                        const float a = acc[i][j][v];
#pragma unroll
                        for (int p = 0; p < QT; ++p)
                            fs[p][j] = __builtin_fmaf(a, __uint_as_float(((words[p][i][j] << (31 - bit)) & 0x80000000u) | 0x3f800000u), fs[p][j]);
                    }
            }
#pragma unroll
            for (int p = 0; p < QT; ++p)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float s = fs[p][j];
                    s += __shfl_xor(s, 32);
                    if (lane < 32) red[(p * 8 + wm * 4 + i) * 256 + wn * 128 + j * 32 + lane] = s;
                }
        }
        __syncthreads();
        const int64_t n = n0 + tid;
        const int64_t Kc = (int64_t)tiles_k * 8;
        if (n < N) {
            for (int p = 0; p < q_train; ++p) {
                float* dst = part + (((int64_t)split * q_train + p) * N + n) * Kc + (int64_t)tile_k * 8;
                u32x4 lo, hi;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    lo[c] = __float_as_uint(red[(p * 8 + c) * 256 + tid]);
                    hi[c] = __float_as_uint(red[(p * 8 + 4 + c) * 256 + tid]);
                }
                *reinterpret_cast<u32x4*>(dst) = lo;
                *reinterpret_cast<u32x4*>(dst + 4) = hi;
            }
        }
        return;
    }
    // every accumulator is read once and added, with its sign, into the sums of all planes
    float sums[QT][4];  // [plane][n tile]
#pragma unroll
    for (int p = 0; p < QT; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j) sums[p][j] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if ((k0 + wm * 128 + i * 32) < K) {  // uniform: tiles beyond K hold nothing
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int bit = 8 * (v >> 2) + (v & 3);
                    const float a = acc[i][j][v];
#pragma unroll
                    for (int p = 0; p < QT; ++p)  // sign bit set where the plane bit is 0 (-1): words are inverted
                        sums[p][j] = __builtin_fmaf(a, __uint_as_float(((words[p][i][j] << (31 - bit)) & 0x80000000u) | 0x3f800000u), sums[p][j]);
                }
        }
    }
#pragma unroll
    for (int p = 0; p < QT; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float s = sums[p][j];
            s += __shfl_xor(s, 32);
            if (lane < 32) red[(p * 2 + wm) * 256 + wn * 128 + j * 32 + lane] = s;
        }
    __syncthreads();
    const int64_t part_id = (int64_t)split * tiles_k + tile_k;
    for (int p = 0; p < q_train; ++p) {
        const int64_t n = n0 + tid;
        if (n < N) part[(part_id * q_train + p) * N + n] = red[(p * 2 + 0) * 256 + tid] + red[(p * 2 + 1) * 256 + tid];
    }
}

// dalpha[pn][grp] = scale * sum over token slices and over the k tiles of group grp of part[slice][tile][pn],
// pn = plane * N + n; `tpg` consecutive k tiles form one scale group (row-wise: all of them, G = 1).
// A workgroup owns 64 consecutive outputs; its four waves each add a quarter of the partial sums (every fourth one,
// eight loads in flight) and wave 0 adds the four quarters in wave order: a fixed order, bit-reproducible.
__global__ __launch_bounds__(256) void dalpha_reduce_kernel(const float* __restrict__ part, float* __restrict__ dalpha,
                                                            int64_t rows /* q_train * N */, int64_t G, int splits,
                                                            int tiles_k, int tpg, float scale, AdamWArgs opt) {
    __shared__ float quarter[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t idx = (int64_t)blockIdx.x * 64 + lane;
    const bool live = idx < rows * G;
    const int64_t pn = live ? idx / G : 0, grp = live ? idx % G : 0;
    const int items = splits * tpg;  // item it = (slice it / tpg, tile it % tpg of the group)
    float s = 0.f;
    int it = wave;
    for (; it + 28 < items; it += 32) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int iu = it + 4 * u;
            v[u] = part[((int64_t)(iu / tpg) * tiles_k + grp * tpg + iu % tpg) * rows + pn];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; it < items; it += 4) s += part[((int64_t)(it / tpg) * tiles_k + grp * tpg + it % tpg) * rows + pn];
    quarter[wave][lane] = s;
    __syncthreads();
    if (wave != 0 || !live) return;
    const float total = scale * ((quarter[0][lane] + quarter[1][lane]) + (quarter[2][lane] + quarter[3][lane]));
    dalpha[idx] = total;
    if (opt.alpha) adamw_apply(opt, idx, total);
}

// Fine partials part[slice][pn][Kc] (one value per 32 columns): a group is a run of cpg consecutive values.
// Same split of the work as above: item it = (slice it / cpg, value it % cpg of the run).
__global__ __launch_bounds__(256) void dalpha_reduce_fine_kernel(const float* __restrict__ part,
                                                                 float* __restrict__ dalpha, int64_t rows, int64_t G,
                                                                 int splits, int64_t Kc, int cpg, float scale,
                                                                 AdamWArgs opt) {
    __shared__ float quarter[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t idx = (int64_t)blockIdx.x * 64 + lane;
    const bool live = idx < rows * G;
    const int64_t pn = live ? idx / G : 0, grp = live ? idx % G : 0;
    const int items = splits * cpg;
    float s = 0.f;
    for (int it = wave; it < items; it += 4)
        s += part[((int64_t)(it / cpg) * rows + pn) * Kc + grp * cpg + it % cpg];
    quarter[wave][lane] = s;
    __syncthreads();
    if (wave != 0 || !live) return;
    const float total = scale * ((quarter[0][lane] + quarter[1][lane]) + (quarter[2][lane] + quarter[3][lane]));
    dalpha[idx] = total;
    if (opt.alpha) adamw_apply(opt, idx, total);
}

struct DalphaPlan {
    int tiles_k, tiles_n, splits;
    int64_t per_split, T16;
    bool xg, fine;
    size_t frag_bytes, part_bytes;
};

static DalphaPlan dalpha_plan(int64_t T, int64_t N, int64_t K, int64_t g, int q) {
    DalphaPlan pl;
    pl.tiles_k = (int)((K + DA_TILE - 1) / DA_TILE);
    pl.tiles_n = (int)((N + DA_TILE - 1) / DA_TILE);
    const int64_t tiles = (int64_t)pl.tiles_k * pl.tiles_n;
    int64_t s = tiles >= 256 ? 1 : 256 / tiles;       // one round of workgroups on the 256 compute units
    const int64_t max_s = (T + 255) / 256;            // at least 256 tokens (4 steps) per slice
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    pl.per_split = ((T + s - 1) / s + 63) / 64 * 64;
    pl.splits = (int)((T + pl.per_split - 1) / pl.per_split);
    pl.T16 = (T + 63) / 64 * 4;
    pl.xg = (K <= N);
    const int64_t gcols = pl.xg ? K : N;
    pl.frag_bytes = (size_t)(((gcols + 31) / 32) * pl.T16 * 1024);
    pl.fine = (g != K) && (g % DA_TILE != 0);  // groups that are not whole k tiles need per-32-column partials
    pl.part_bytes = (size_t)pl.splits * pl.tiles_k * q * N * sizeof(float) * (pl.fine ? 8 : 1);
    return pl;
}

size_t mfma_bwd_alpha_workspace(int64_t T, int64_t N, int64_t K, int64_t g, int q) {
    const DalphaPlan pl = dalpha_plan(T, N, K, g, q);
    return pl.frag_bytes + pl.part_bytes;
}

hipError_t launch_bwd_alpha_mfma(const uint32_t* packed, const void* x, const void* dy, int64_t T, int64_t N,
                                 int64_t K, int64_t g, int q, int q_train, float grad_scale, float* dalpha,
                                 void* workspace, const AdamWArgs* opt, hipStream_t st) {
    const int lds = 3 * DA_STAGE;
    const DalphaPlan pl = dalpha_plan(T, N, K, g, q);
    u32x4* frag = reinterpret_cast<u32x4*>(workspace);
    float* part = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(workspace) + pl.frag_bytes);
    const bf16_t* gact = (const bf16_t*)(pl.xg ? x : dy);
    const bf16_t* lact = (const bf16_t*)(pl.xg ? dy : x);
    const int64_t gcols = pl.xg ? K : N, lcols = pl.xg ? N : K;
    {
        dim3 grid((unsigned)((gcols + 127) / 128), (unsigned)((pl.T16 * 2 + 15) / 16));
        BCQ_LAUNCH(transpose_frag_kernel, grid, dim3(256), 0, st, gact, T, gcols, pl.T16, frag);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    TileMap tmap;
    const unsigned wgs = make_tile_map(pl.tiles_k, pl.tiles_n, pl.splits, 32, 1.0, 1.0, &tmap);
    dim3 grid(wgs);
    const int qt = q_train <= 4 ? q_train : 8;
#define BCQ_DA_LAUNCH(XGV, QTV, FV)                                                                                   \
    {                                                                                                                 \
        static LdsLimit limit;                                                                                        \
        hipError_t ea = limit.ensure((const void*)dalpha_kernel<XGV, QTV, FV>, (size_t)lds);                           \
        if (ea != hipSuccess) return ea;                                                                              \
        BCQ_LAUNCH((dalpha_kernel<XGV, QTV, FV>), grid, dim3(256), lds, st, lact, lcols, lcols, frag, pl.T16,  \
                           packed, part, T, N, K, q_train, tmap, pl.splits, pl.per_split);                            \
    }
#define BCQ_DA_Q(XGV, FV)                                  \
    switch (qt) {                                          \
        case 1: BCQ_DA_LAUNCH(XGV, 1, FV) break;           \
        case 2: BCQ_DA_LAUNCH(XGV, 2, FV) break;           \
        case 3: BCQ_DA_LAUNCH(XGV, 3, FV) break;           \
        case 4: BCQ_DA_LAUNCH(XGV, 4, FV) break;           \
        default: BCQ_DA_LAUNCH(XGV, 8, FV) break;          \
    }
    if (pl.fine) {
        if (pl.xg) {
            BCQ_DA_Q(true, true)
        } else {
            BCQ_DA_Q(false, true)
        }
    } else {
        if (pl.xg) {
            BCQ_DA_Q(true, false)
        } else {
            BCQ_DA_Q(false, false)
        }
    }
#undef BCQ_DA_Q
#undef BCQ_DA_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t rows = (int64_t)q_train * N, G = K / g;
    const dim3 rgrid((unsigned)((rows * G + 63) / 64));
    AdamWArgs oa = {};
    if (opt) oa = *opt;
    if (pl.fine)
        BCQ_LAUNCH(dalpha_reduce_fine_kernel, rgrid, dim3(256), 0, st, (const float*)part, dalpha, rows, G,
                           pl.splits, (int64_t)pl.tiles_k * 8, (int)(g / 32), grad_scale, oa);
    else
        BCQ_LAUNCH(dalpha_reduce_kernel, rgrid, dim3(256), 0, st, (const float*)part, dalpha, rows, G,
                           pl.splits, pl.tiles_k, (int)(g == K ? pl.tiles_k : g / DA_TILE), grad_scale, oa);
    return hipGetLastError();
}

}  // namespace bcq
