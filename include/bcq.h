/*
 * bcq.h - C ABI of the MI355X (gfx950) library for the binary-coding-quantized (BCQ) linear layer
 * of AlphaTuning (arXiv 2210.03858).
 *
 * Model (Section 3 "BCQ Format", Eq. 1, row-wise quantization g = h_in):
 *     W[N][K] ~= sum_{i=0..q-1} diag(alpha_i) * B_i ,   B_i in {-1,+1}^{N x K},  alpha_i in R^N.
 * N = h_out (rows of W), K = h_in (columns of W, contraction length of the forward), T = n_b tokens.
 * Plane index i is 0-based here (alpha_1 of the paper is alpha[0]).  Shapes follow Table 1:
 * alpha[q][N] (always fp32, Section 4.2), sign planes [q][N][K].
 *
 * Canonical packed layout: packed[i][n][w], w < K/32, one uint32 per 32 consecutive columns;
 * bit j (LSB = 0) of word w is the sign of B_i[n][32w + j]; 1 <=> +1, 0 <=> -1.
 * Transposed twin (optional accelerator for the input gradient): packed_t[i][k][v], v < N/32;
 * bit j of word v is the sign of B_i[32v + j][k].  It holds the same information as `packed`.
 *
 * Group-wise scales (Appendix C, paragraph "group-wise quantization"; Table 1 rows with g < h_in; Section 4.1,
 * remark after Eq. 4): every row is cut into K/g consecutive vectors of length g, each with its own q scales:
 *     What[n][k] = sum_i alpha_i[n][k / g] * B_i[n][k],   alpha[q][N][K/g] fp32.
 * The *_grouped entry points take g (32 <= g <= K, g % 32 == 0, K % g == 0, else BCQ_ERR_SHAPE); with g = K they
 * are the row-wise calls, which forward to them.  The sign planes and their packed layouts do not depend on g.
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *     frees or keeps them.  Arrays are dense row-major with the innermost extent as stride.
 *   - Every data pointer must be 16-byte aligned (BCQ_ERR_ALIGN otherwise).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Arguments are
 *     validated synchronously on the host; the work is enqueued on `stream` and the call returns
 *     without waiting.  Outputs are valid once the stream has reached that point.
 *   - `workspace` is optional device scratch owned by the caller, at least 16-byte aligned; its
 *     contents before the call are ignored and after the call are unspecified (except where an
 *     entry point documents a status word).  Pass NULL / 0 to make the library choose a path that
 *     needs none (always available, possibly slower).  bcq_workspace_bytes() gives the size that
 *     enables the fastest path; a non-NULL workspace smaller than that is BCQ_ERR_WORKSPACE.
 *   - Return value: BCQ_OK or the first problem found; nothing is enqueued unless BCQ_OK.
 *     Order of checks: NULL pointers, shapes, dtype, alignment, workspace, device.
 *   - Limits: 1 <= q <= 8; K % 32 == 0; 1 <= N, K <= 2^17; 1 <= T <= 2^24; N*K and T*max(N,K) at most 2^40.
 *   - No global state besides per-device capability caches; calls on different streams may overlap
 *     as long as their outputs and workspaces do not alias.
 *   - Numerics of the bf16 paths (fp32 accumulation throughout; the bar of the tests is 2e-2 of the largest output):
 *     the matrix-core path (32 tokens and more, workspace given) first sums the planes into What = sum_i alpha_i B_i
 *     and rounds What to bf16 once (relative 2^-9 per weight) - a rounding Eq. 2 / Eq. 3 do not contain; alpha itself
 *     stays fp32.  The streaming paths (few tokens) multiply exact signs with activations split into two FP8 terms:
 *     exact for bf16 activations within 2^-13 of the largest of their 32-element block (forward, scale gradient); the
 *     input gradient re-codes the fp32 product dy * alpha_i and keeps 8 significant bits of it (relative 2^-9 per
 *     term).  Without a workspace, and for fp32 activations, no such rounding happens.
 *   - Non-finite activations: a token row of x or dy that holds an Inf or NaN makes the outputs of that token
 *     non-finite and leaves every other token's outputs untouched (the scale gradient sums over tokens and becomes
 *     non-finite as a whole); the streaming paths return NaN for every output of such a token.
 *   - HIP graphs: every call only launches kernels on `stream` (no allocation, no memset, no
 *     synchronisation), so it can be recorded into a graph.  The first launch of a kernel that
 *     needs more than 64 KiB of LDS raises that kernel's limit (a host-side attribute call), so
 *     run each call once with its shapes before the capture, or call bcq_prepare / bcq_batch_prepare.  A captured call keeps pointing at
 *     the buffers it was recorded with.
 */
#ifndef BCQ_H
#define BCQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BCQ_OK = 0,
    BCQ_ERR_NULL = 1,      /* a required pointer is NULL                                        */
    BCQ_ERR_SHAPE = 2,     /* N,K,T < 1; q outside [1,8]; K % 32 != 0; q_train outside [1,q];
                              N % 32 != 0 with a transposed twin; K above the quantizer's limit;
                              g outside [32,K], g % 32 != 0 or K % g != 0                       */
    BCQ_ERR_DTYPE = 3,     /* dtype is neither BCQ_F32 nor BCQ_BF16, or op code unknown         */
    BCQ_ERR_ALIGN = 4,     /* a data pointer or the workspace is not 16-byte aligned            */
    BCQ_ERR_WORKSPACE = 5, /* workspace non-NULL but smaller than bcq_workspace_bytes()         */
    BCQ_ERR_NONFINITE = 6, /* reserved: reported through bcq_quantize's status word, not returned */
    BCQ_ERR_DEVICE = 7     /* no usable gfx950 device, or a HIP call failed                     */
} bcq_status;

typedef enum { BCQ_F32 = 0, BCQ_BF16 = 1 } bcq_dtype; /* element type of x, y, dy, dx */

typedef enum {
    BCQ_OP_QUANTIZE = 0,
    BCQ_OP_FWD = 1,
    BCQ_OP_BWD_INPUT = 2,
    BCQ_OP_BWD_ALPHA = 3
} bcq_op;

/* Largest K bcq_quantize accepts (a whole row is kept in registers across the q planes). */
#define BCQ_QUANTIZE_MAX_K 16384

/* Static, NUL-terminated description of a status code. */
const char* bcq_status_string(bcq_status s);

/* ABI version, bumped on any signature change or addition (2: *_grouped entry points; 3: bcq_quantize_alternating; 4: AdamW entry points;
 * 5: decode layout; 6: bcq_linear_fwd_static;
 * 7: batched small-token calls; 8: bcq_prepare, bcq_batch_prepare; 9: bcq_linear_fwd_lut). */
int bcq_abi_version(void);

/* Scratch size (bytes) that enables the fastest path of `op` for this problem; *out may be 0.
 * T is ignored for BCQ_OP_QUANTIZE.  Host-only: touches no device. */
bcq_status bcq_workspace_bytes(int op, int64_t T, int64_t N, int64_t K, int q, int dtype, size_t* out);

/* bcq_workspace_bytes for group size g. */
bcq_status bcq_workspace_bytes_grouped(int op, int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype,
                                       size_t* out);

/* Host-side one-time set-up for later calls of `op` (BCQ_OP_*) with these arguments, with or without a workspace and
 * twin and for every q_train: the kernels those calls select get their dynamic-LDS limit raised where they need more
 * than 64 KiB, and bcq_linear_fwd_static's scratch address is looked up.  Nothing is launched, allocated or read.
 * After it the calls only launch kernels, so the very first one may already sit inside a HIP graph capture.
 * Not needed otherwise: every entry point does the same set-up by itself on first use.
 * g = K for row-wise scales.  Errors: BCQ_ERR_DTYPE (op, dtype), BCQ_ERR_SHAPE, BCQ_ERR_DEVICE. */
bcq_status bcq_prepare(int op, int64_t T, int64_t N, int64_t K, int64_t g, int q, int dtype);

/* Greedy BCQ quantizer (Appendix C: Eq. ap1 for the first plane, Eq. ap2-ap3 for the others).
 * Per row n: r = W[n][:] in fp64; for i = 0..q-1: B_i = (r >= 0 ? +1 : -1) (so sign(0) = +1),
 * alpha_i = fp32( sum_k |r_k| / K ) with the sum in fp64, r -= alpha_i * B_i using the ROUNDED alpha_i.
 *   W          [N][K] fp32, in
 *   alpha      [q][N] fp32, out
 *   packed     [q][N][K/32] uint32 canonical layout, out
 *   planes_i8  [q][N][K] int8 holding -1/+1, out; may be NULL
 *   workspace  optional; if non-NULL (>= 16 bytes) its first int32 is a status word, set to the number of
 *              rows of W that hold a NaN or Inf (0 = all finite); outputs of such rows are unspecified.
 * K <= BCQ_QUANTIZE_MAX_K, else BCQ_ERR_SHAPE. */
bcq_status bcq_quantize(const float* W, int64_t N, int64_t K, int q, float* alpha, uint32_t* packed,
                        int8_t* planes_i8, void* workspace, size_t workspace_bytes, void* stream);

/* bcq_quantize on every length-g vector of every row on its own (Appendix C, group-wise paragraph):
 * alpha [q][N][K/g] out; packed and planes_i8 as above.  g <= BCQ_QUANTIZE_MAX_K and N*K/g < 2^31, else
 * BCQ_ERR_SHAPE.  The status word counts vectors (not rows) that hold a NaN or Inf. */
bcq_status bcq_quantize_grouped(const float* W, int64_t N, int64_t K, int64_t g, int q, float* alpha,
                                uint32_t* packed, int8_t* planes_i8, void* workspace, size_t workspace_bytes,
                                void* stream);

/* Alternating quantizer (Appendix C, "Alternating Method", Eq. ap4): the greedy result of every length-g vector
 * is refined by `iters` rounds (the paper uses 15) of (1) least-squares refit alpha = (B^T B)^{-1} B^T w and
 * (2) re-assignment of every element to the nearest of the 2^q levels sum_i +-alpha_i.  fp64 throughout, alpha
 * rounded to fp32 once at the end (it may come out negative or zero).  The loop stops at a fixed point, and before
 * a refit whose B^T B is singular (then the current pair stays, e.g. the greedy pair of an all-zero vector).
 * Ties between two levels go to the larger level.  iters = 0 returns the greedy result.  Arguments, layouts,
 * limits and the status word as bcq_quantize_grouped (g = K: row-wise); 0 <= iters <= BCQ_ALTERNATING_MAX_ITERS. */
#define BCQ_ALTERNATING_MAX_ITERS 1000
bcq_status bcq_quantize_alternating(const float* W, int64_t N, int64_t K, int64_t g, int q, int iters, float* alpha,
                                    uint32_t* packed, int8_t* planes_i8, void* workspace, size_t workspace_bytes,
                                    void* stream);

/* Bit-plane pack (Table 1 gives the index order B:(q, h_out, h_in); footnote of Section 3: contiguous rows).
 *   planes_i8 [q][N][K] int8, in.  Only the sign of each byte is read: v >= 0 -> bit 1 (+1), v < 0 -> bit 0.
 *   packed    [q][N][K/32] uint32 canonical layout, out. */
bcq_status bcq_pack(const int8_t* planes_i8, int64_t N, int64_t K, int q, uint32_t* packed, void* stream);

/* Inverse of bcq_pack: writes exactly -1 or +1 into planes_i8[q][N][K]. */
bcq_status bcq_unpack(const uint32_t* packed, int64_t N, int64_t K, int q, int8_t* planes_i8, void* stream);

/* Builds the transposed twin packed_t[q][K][N/32] from the canonical packed[q][N][K/32] (same signs,
 * bits running along N).  Needs N % 32 == 0.  One-time, like bcq_pack; used by bcq_linear_bwd_input. */
bcq_status bcq_pack_transposed(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* packed_t,
                               void* stream);

/* Decode layout of the sign planes (Section 3 ends with inference through kernels that multiply by the packed binary
 * codes directly instead of dequantising; this is the layout our small-token forward streams fastest): the same bits
 * as the canonical layout, tile-ordered so that every 4 KiB a wave reads is one contiguous run in HBM.
 *   tiled [ceil(N/16)][ceil(K/512)][q][64][4] uint32: row tile rt, 512-column segment seg, plane i, lane l, word j
 *   hold canonical word packed[i][16 rt + l % 16][16 seg + 4 (l / 16) + j]; rows >= N and words >= K/32 read as 0.
 * bcq_decode_layout_bytes gives the size of `tiled`; bcq_pack_decode builds it (one-time, like bcq_pack). */
bcq_status bcq_decode_layout_bytes(int64_t N, int64_t K, int q, size_t* out);
bcq_status bcq_pack_decode(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* tiled, void* stream);

/* Forward (Eq. 2) from the decode layout, for at most 80 tokens of bf16 activations: same result as
 * bcq_linear_fwd_grouped on the canonical planes.
 *   tiled: output of bcq_pack_decode, in; alpha [q][N][K/g] fp32 in (g == K: row-wise; else g % 512 == 0);
 *   x [T][K] bf16 in; y [T][N] bf16 out; workspace REQUIRED, at least
 *   bcq_workspace_bytes_grouped(BCQ_OP_FWD, T, N, K, g, q, BCQ_BF16) bytes.
 * Errors: BCQ_ERR_DTYPE for fp32 activations; BCQ_ERR_SHAPE for T > 80 or a group size the streaming kernels do
 * not take; BCQ_ERR_NULL without workspace; the others as for bcq_linear_fwd. */
bcq_status bcq_linear_fwd_decode(const uint32_t* tiled, const float* alpha, const void* x, int dtype, int64_t T,
                                 int64_t N, int64_t K, int64_t g, int q, void* y, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Forward (Eq. 2) for decode by table look-up (Section 6, "Inference Speed": the route the paper names for fast
 * small-batch inference), a selectable variant of bcq_linear_fwd for 1 .. BCQ_LUT_MAX_TOKENS tokens of bf16
 * activations and row-wise scales.  Every group of 4 columns of x gives a table of its 16 signed sums (8 stored, the
 * rest by sign), built in LDS by every workgroup; the nibbles of the canonical packed words index it; alpha is
 * applied once per plane and row; fp32 accumulation, y rounded to bf16.  No workspace, nothing allocated.
 *   packed [q][N][K/32] in; alpha [q][N] fp32 in; x [T][K] bf16 in; y [T][N] bf16 out.
 * Errors: BCQ_ERR_DTYPE unless dtype == BCQ_BF16; BCQ_ERR_SHAPE for T > BCQ_LUT_MAX_TOKENS or tables larger than
 * BCQ_LUT_MAX_TABLE_BYTES (8 * T * K bytes of LDS: T = 1 any K <= 16384, T = 4 K <= 4096) and the usual shape limits;
 * BCQ_ERR_NULL, BCQ_ERR_ALIGN, BCQ_ERR_DEVICE as for bcq_linear_fwd.
 * On gfx950 the default small-token path (FP4 x FP8 matrix instruction) is the faster one at every token count;
 * this entry point exists so that the two can be compared. */
#define BCQ_LUT_MAX_TOKENS 4
#define BCQ_LUT_MAX_TABLE_BYTES (128 * 1024)
bcq_status bcq_linear_fwd_lut(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                              int64_t N, int64_t K, int q, void* y, void* stream);

/* Forward (Eq. 2): y[t][n] = sum_i alpha_i[n] * sum_k B_i[n][k] * x[t][k], fp32 accumulation,
 * result rounded to `dtype` (bf16: round to nearest even).  The dequantised W exists at most as a transient bf16
 * copy of this one layer inside the caller's workspace (large-token path); without a workspace it never exists.
 *   packed [q][N][K/32] in; alpha [q][N] fp32 in; x [T][K] `dtype` in; y [T][N] `dtype` out. */
bcq_status bcq_linear_fwd(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                          int64_t N, int64_t K, int q, void* y, void* workspace, size_t workspace_bytes,
                          void* stream);

/* bcq_linear_fwd for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as bcq_linear_fwd with a workspace
 * (row-wise scales, bf16 activations, at most BCQ_STATIC_MAX_TOKENS tokens: the streaming kernels), but the scratch
 * of those kernels - the activations re-coded as two block-scaled FP8 terms - lives in a fixed array of
 * BCQ_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing and calls no allocating routine.
 *   packed [q][N][K/32] in; alpha [q][N] fp32 in; x [T][K] bf16 in; y [T][N] bf16 out (caller-owned, as everywhere).
 * Errors: BCQ_ERR_DTYPE unless dtype == BCQ_BF16; BCQ_ERR_SHAPE for T > BCQ_STATIC_MAX_TOKENS (and the usual shape
 * limits); BCQ_ERR_WORKSPACE when the re-coded activations do not fit the array, i.e. when
 * bcq_workspace_bytes(BCQ_OP_FWD, T, N, K, q, BCQ_BF16) > BCQ_STATIC_SCRATCH_BYTES (about 1056 bytes per token rounded
 * up to 8 or a multiple of 16, per 512 columns of K: T <= 8 fits any K <= 2^17 - 4096, T <= 16 K <= 63488, T <= 80 K <= 12288);
 * the others as for bcq_linear_fwd.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different streams or
 * host threads) race on it and give unspecified results; calls on one stream, or ordered by events, are safe.  The
 * array keeps the previous call's contents; every byte a call reads is written by that call first.
 * The first call on a device looks the array's address up (a host-side query): make it before a graph capture. */
#define BCQ_STATIC_SCRATCH_BYTES (2 * 1024 * 1024)
#define BCQ_STATIC_MAX_TOKENS 80
bcq_status bcq_linear_fwd_static(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                                 int64_t N, int64_t K, int q, void* y, void* stream);

/* Eq. 2 with group-wise scales alpha [q][N][K/g]: y[t][n] = sum_k x[t][k] * sum_i alpha_i[n][k/g] * B_i[n][k]. */
bcq_status bcq_linear_fwd_grouped(const uint32_t* packed, const float* alpha, const void* x, int dtype, int64_t T,
                                  int64_t N, int64_t K, int64_t g, int q, void* y, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* Input gradient (Eq. 3): dx[t][k] = sum_n dy[t][n] * sum_i alpha_i[n] * B_i[n][k].
 *   packed [q][N][K/32] in; packed_t [q][K][N/32] in, may be NULL (non-NULL needs N % 32 == 0); alpha [q][N] in;
 *   dy [T][N] `dtype` in; dx [T][K] `dtype` out.
 * Up to 48 tokens the fast path streams the twin and needs BOTH packed_t and the workspace; from 32 tokens on the
 * tiled path needs the workspace only and uses packed_t when given.  Without them a slower path reads `packed`. */
bcq_status bcq_linear_bwd_input(const uint32_t* packed, const uint32_t* packed_t, const float* alpha,
                                const void* dy, int dtype, int64_t T, int64_t N, int64_t K, int q, void* dx,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Eq. 3 with group-wise scales alpha [q][N][K/g]; arguments as bcq_linear_bwd_input. */
bcq_status bcq_linear_bwd_input_grouped(const uint32_t* packed, const uint32_t* packed_t, const float* alpha,
                                        const void* dy, int dtype, int64_t T, int64_t N, int64_t K, int64_t g,
                                        int q, void* dx, void* workspace, size_t workspace_bytes, void* stream);

/* Scale gradient (Eq. 4, read as the gradient of Eq. 2 with the empirical 1/g_L left to the caller):
 *   dalpha[i][n] = grad_scale * sum_t dy[t][n] * sum_k B_i[n][k] * x[t][k]   for i < q_train.
 * grad_scale = 1 gives the true gradient; the paper's damping is grad_scale = 1/K for row-wise scales.
 * q_train = 1 is the paper's recipe (train alpha_1 only, Section 4.2); q_train = q trains all planes.
 *   packed [q][N][K/32] in; x [T][K], dy [T][N] `dtype` in; dalpha [q_train][N] fp32 out, OVERWRITTEN.
 * The result does not depend on the launch order of workgroups (no floating-point atomics). */
bcq_status bcq_linear_bwd_alpha(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                int64_t N, int64_t K, int q, int q_train, float grad_scale, float* dalpha,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Eq. 4 per scale group: dalpha[i][n][c] = grad_scale * sum_t dy[t][n] * sum_{k in group c} B_i[n][k] * x[t][k],
 * dalpha [q_train][N][K/g] fp32 out, OVERWRITTEN.  The paper's damping is grad_scale = 1/g. */
bcq_status bcq_linear_bwd_alpha_grouped(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                        int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                        float* dalpha, void* workspace, size_t workspace_bytes, void* stream);

/* ---- Batched small-token calls: many independent layers in two launches ------------------------------------------
 * Section 3 notes that small-batch inference is memory-bound and Section 6 ("Inference Speed") expects a latency gain
 * in proportion to the memory reduction.  A single layer of the paper's models holds only 0.2 - 13 MB of sign planes
 * (Table 1), less than a microsecond of HBM time, so a call per layer is bound by launches.  These entry points run
 * ONE operation - forward (Eq. 2), input gradient (Eq. 3) or scale gradient (Eq. 4) - for `count` layers at once:
 * one activation re-coding launch and one streaming launch whose workgroups look their share of the work up in a plan.
 * The layers of a batch must be independent of each other (no layer's input is another's output), share T, q, q_train
 * and grad_scale, use bf16 activations and row-wise scales.  Same arithmetic as the single-layer streaming kernels
 * (signs times activations split into two FP8 terms on the block-scaled matrix instruction, fp32 accumulation).
 *
 * The planes are read in the DECODE layout (bcq_pack_decode), which a wave can stream in address order:
 *   tiled    = bcq_pack_decode(packed,   N, K, q)   for the forward and the scale gradient,
 *   tiled_t  = bcq_pack_decode(packed_t, K, N, q)   for the input gradient (the decode layout of the transposed twin,
 *              i.e. of the [q][K][N/32] matrix that bcq_pack_transposed builds; needs N % 32 == 0).
 *
 * Use: fill a HOST array of bcq_batch_layer; bcq_batch_sizes gives the bytes of the plan and of the workspace;
 * bcq_batch_plan writes the plan into caller-owned HOST memory; the caller copies those bytes to device memory once
 * (they are position independent); bcq_linear_batched then runs the batch, any number of times, as long as the device
 * pointers inside the plan stay valid.  Nothing is allocated, copied or retained by the library.
 *
 * Fields a given op reads (all device pointers, 16-byte aligned; the others may be NULL):
 *   BCQ_OP_FWD:       tiled, alpha [q][N], x [T][K] bf16        -> y [T][N] bf16
 *   BCQ_OP_BWD_INPUT: tiled_t, alpha, dy [T][N] bf16            -> dx [T][K] bf16
 *   BCQ_OP_BWD_ALPHA: tiled, x, dy                              -> dalpha [q_train][N] fp32, overwritten
 * Limits: 1 <= T <= BCQ_BATCH_MAX_TOKENS, 1 <= q <= BCQ_BATCH_MAX_Q, 1 <= count <= BCQ_BATCH_MAX_LAYERS, N % 32 == 0
 * for the input gradient; else BCQ_ERR_SHAPE.  dtype must be BCQ_BF16 (BCQ_ERR_DTYPE).  q_train and grad_scale are read
 * for BCQ_OP_BWD_ALPHA only. */
#define BCQ_BATCH_MAX_TOKENS 16
#define BCQ_BATCH_MAX_Q 4
#define BCQ_BATCH_MAX_LAYERS (1 << 20)
typedef struct bcq_batch_layer {
    const uint32_t* tiled;
    const uint32_t* tiled_t;
    const float* alpha;
    const void* x;
    const void* dy;
    void* y;
    void* dx;
    float* dalpha;
    int64_t N, K;
} bcq_batch_layer;

/* Bytes of the plan (same size on the host and on the device) and of the device workspace for these arguments (the
 * same op, layers, T, q, q_train must be given to bcq_batch_plan).  Host-only. */
bcq_status bcq_batch_sizes(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                           int dtype, size_t* table_bytes, size_t* workspace_bytes);

/* Writes the plan for `op` over layers[0 .. count) into table_host (HOST memory, at least table_bytes of
 * bcq_batch_sizes, else BCQ_ERR_WORKSPACE).  Host-only: touches no device.  Checks NULL, shapes, dtype, alignment. */
bcq_status bcq_batch_plan(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                          float grad_scale, int dtype, void* table_host, size_t table_bytes);

/* Runs a planned batch on `stream`: table_host is the plan as written by bcq_batch_plan, table_device a copy of the
 * same bytes in device memory (16-byte aligned; the kernels read it), workspace device scratch of at least the plan's
 * workspace bytes (16-byte aligned, REQUIRED; contents unspecified afterwards; calls that may overlap need their own).
 * BCQ_ERR_DTYPE if table_host does not hold a plan of this library version. */
bcq_status bcq_linear_batched(const void* table_host, const void* table_device, size_t table_bytes, void* workspace,
                              size_t workspace_bytes, void* stream);

/* Host-side one-time set-up of bcq_linear_batched for this plan (see bcq_prepare): after it, the first
 * bcq_linear_batched with the plan only launches kernels and may sit inside a HIP graph capture. */
bcq_status bcq_batch_prepare(const void* table_host, size_t table_bytes);

/* One AdamW step (Appendix A: AdamW with a linear-decay learning rate, the schedule being the caller's: pass the
 * step's lr).  Decoupled weight decay, bias-corrected moments, t = step >= 1:
 *     m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g^2;
 *     alpha <- alpha - lr * ( (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps) + weight_decay * alpha ).
 * BCQ_ERR_SHAPE: beta outside [0,1), step < 1, eps < 0, NaN lr or weight_decay. */
typedef struct bcq_adamw {
    float lr, beta1, beta2, eps, weight_decay;
    int64_t step;
} bcq_adamw;

/* alpha, m, v [count] fp32 in/out (device), dalpha [count] fp32 in: the update above, element-wise.  Only the
 * trained scales take part: with q_train < q pass the first q_train planes (they are contiguous). */
bcq_status bcq_alpha_adamw_step(float* alpha, const float* dalpha, float* m, float* v, int64_t count,
                                const bcq_adamw* opt, void* stream);

/* bcq_linear_bwd_alpha_grouped followed by the AdamW step on alpha[0 .. q_train) in the same call (Section 4.1:
 * only the scales are trained; Section 4.2: alpha_1 only = q_train 1).  dalpha [q_train][N][K/g] is still written;
 * alpha, m, v [q_train][N][K/g] fp32 are updated in place.  On the matrix-core path the update happens inside the
 * final reduction of the gradient (no extra kernel, no re-read of dalpha). */
bcq_status bcq_linear_bwd_alpha_adamw(const uint32_t* packed, const void* x, const void* dy, int dtype, int64_t T,
                                      int64_t N, int64_t K, int64_t g, int q, int q_train, float grad_scale,
                                      float* dalpha, float* alpha, float* m, float* v, const bcq_adamw* opt,
                                      void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BCQ_H */
