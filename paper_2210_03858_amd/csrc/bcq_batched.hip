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
enum { BATCH_MAIN_LDS = 0, BATCH_MAIN_WAVE = 1 };  // shared-activation kernel body / per-wave kernel body

struct BatchHeader {  // 128 bytes
    uint32_t magic, version;
    int32_t op, q, q_used, T, halves, count;
    float scale;
    uint32_t pre_blocks, pre_sets;
    uint32_t main_blocks[2];     // workgroups of the launch of each main-kernel form (0 = none)
    uint32_t pad0;
    // 56 bytes so far
    uint64_t layers_off, pre_map_off, main_map_off[2];
    uint64_t table_bytes, workspace_bytes;
    uint64_t plane_bytes;        // sum of q N K / 8 over the layers (for reporting)
    uint64_t pad1[2];
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
    uint32_t seg_magic;       // ceil(2^32 / segs_act): virtual segment -> plane
    uint64_t pad[3];
};
static_assert(sizeof(BatchLayerDev) == 128, "table layer layout");

// ---- kernels --------------------------------------------------------------------------------------------------------
// blockIdx.x -> (layer, block index inside the layer) through `map`; all loads below are uniform (scalar).
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
    stream_body<STREAM_DX, 1, QP, TWO, true, false, false>(L.planes, ws + L.xq_off, ws + L.sq_off, L.alpha, nullptr, L.out,
                                                           T, L.rows, L.cw, q_used, 1.f, L.spp, L.segs_main,
                                                           (size_t)L.xq_plane, (size_t)L.sq_plane, 127, 1, 1, 0, m.y, 0);
}

constexpr int kWaveFormWaves = 4;

// ---- host: sizes and plan ---------------------------------------------------------------------------------------------
struct BatchShape {  // per layer, derived from (op, T, N, K)
    int64_t rows, cw;
    int32_t segs_act, segs_main, spp;
    int form;
    uint32_t main_blocks, sets;
    size_t xq_bytes, sq_bytes;
};

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static BatchShape batch_shape(int op, int64_t T, int64_t N, int64_t K, int q) {
    BatchShape s;
    const bool dx = (op == BCQ_OP_BWD_INPUT);
    s.rows = dx ? K : N;
    s.cw = (dx ? N : K) / 32;
    s.segs_act = (int32_t)((s.cw + 15) / 16);
    const int halves = T <= 8 ? 1 : 2;
    s.sets = dx ? (uint32_t)q : 1u;
    s.xq_bytes = (size_t)s.segs_act * 4 * halves * QBLK;
    s.sq_bytes = (size_t)s.segs_act * halves * QSCL;
    const int64_t rt = (s.rows + 15) / 16;
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
    uint64_t pre_blocks = 0, main_blocks[2] = {0, 0};
    size_t table_bytes = 0, workspace_bytes = 0;
    uint64_t plane_bytes = 0;
};

static BatchTotals batch_totals(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q) {
    BatchTotals t;
    for (int64_t l = 0; l < count; ++l) {
        const BatchShape s = batch_shape(op, T, layers[l].N, layers[l].K, q);
        t.pre_blocks += (uint64_t)s.segs_act;
        t.main_blocks[s.form] += s.main_blocks;
        t.workspace_bytes += align_up(s.sets * s.xq_bytes, 256) + align_up(s.sets * s.sq_bytes, 256);
        t.plane_bytes += (uint64_t)q * (uint64_t)layers[l].N * (uint64_t)layers[l].K / 8;
    }
    t.table_bytes = sizeof(BatchHeader) + (size_t)count * sizeof(BatchLayerDev) +
                    (size_t)(t.pre_blocks + t.main_blocks[0] + t.main_blocks[1]) * sizeof(uint2);
    t.table_bytes = align_up(t.table_bytes, 256);
    return t;
}

static bcq_status batch_check(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int dtype,
                              bool pointers) {
    using namespace host;
    if (!layers) return BCQ_ERR_NULL;
    if (op != BCQ_OP_FWD && op != BCQ_OP_BWD_INPUT && op != BCQ_OP_BWD_ALPHA) return BCQ_ERR_DTYPE;
    if (count < 1 || count > BCQ_BATCH_MAX_LAYERS || T < 1 || T > BCQ_BATCH_MAX_TOKENS || q < 1 || q > BCQ_BATCH_MAX_Q)
        return BCQ_ERR_SHAPE;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        if (!shape_ok(T, b.N, b.K, q)) return BCQ_ERR_SHAPE;
        // 16-byte plane loads: the streamed plane matrix needs a multiple of 4 words per row
        if ((op == BCQ_OP_BWD_INPUT ? b.N : b.K) % 128 != 0) return BCQ_ERR_SHAPE;
        if (op == BCQ_OP_BWD_INPUT && b.N % 32 != 0) return BCQ_ERR_SHAPE;
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

template <int MODE>
static hipError_t launch_main_lds(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    const bool two = h.halves == 2;
    if constexpr (MODE == STREAM_DX) {  // one virtual plane
        return two ? launch_main_lds_cfg<MODE, 1, true>(h, dev, ws, 1, st) : launch_main_lds_cfg<MODE, 1, false>(h, dev, ws, 1, st);
    } else {
#define BCQ_BATCH_Q(QQ)                                                            \
    return two ? launch_main_lds_cfg<MODE, QQ, true>(h, dev, ws, h.q_used, st)    \
               : launch_main_lds_cfg<MODE, QQ, false>(h, dev, ws, h.q_used, st)
        switch (h.q_used) {
            case 1: BCQ_BATCH_Q(1);
            case 2: BCQ_BATCH_Q(2);
            case 3: BCQ_BATCH_Q(3);
            default: BCQ_BATCH_Q(4);
        }
#undef BCQ_BATCH_Q
    }
}

template <int QP, bool TWO>
static hipError_t launch_main_wave_cfg(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws,
                                       hipStream_t st) {
    hipLaunchKernelGGL((stream_dx_batched_kernel<QP, TWO>), dim3(h.main_blocks[BATCH_MAIN_WAVE]),
                       dim3(64 * kWaveFormWaves), kWaveFormWaves * 1024, st,
                       reinterpret_cast<const BatchLayerDev*>(dev + h.layers_off),
                       reinterpret_cast<const uint2*>(dev + h.main_map_off[BATCH_MAIN_WAVE]), ws, (int64_t)h.T, h.q_used);
    return hipGetLastError();
}

static hipError_t launch_main_wave(const BatchHeader& h, const unsigned char* dev, const unsigned char* ws, hipStream_t st) {
    const bool two = h.halves == 2;
#define BCQ_BATCH_Q(QQ) return two ? launch_main_wave_cfg<QQ, true>(h, dev, ws, st) : launch_main_wave_cfg<QQ, false>(h, dev, ws, st)
    switch (h.q_used) {
        case 1: BCQ_BATCH_Q(1);
        case 2: BCQ_BATCH_Q(2);
        case 3: BCQ_BATCH_Q(3);
        default: BCQ_BATCH_Q(4);
    }
#undef BCQ_BATCH_Q
}

}  // namespace bcq

extern "C" {

bcq_status bcq_batch_sizes(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int dtype,
                           size_t* table_bytes, size_t* workspace_bytes) {
    if (!table_bytes || !workspace_bytes) return BCQ_ERR_NULL;
    const bcq_status s = bcq::batch_check(op, layers, count, T, q, dtype, false);
    if (s != BCQ_OK) return s;
    const bcq::BatchTotals t = bcq::batch_totals(op, layers, count, T, q);
    if (t.pre_blocks > 0x7FFFFFFFull || t.main_blocks[0] > 0x7FFFFFFFull || t.main_blocks[1] > 0x7FFFFFFFull)
        return BCQ_ERR_SHAPE;
    *table_bytes = t.table_bytes;
    *workspace_bytes = t.workspace_bytes;
    return BCQ_OK;
}

bcq_status bcq_batch_plan(int op, const bcq_batch_layer* layers, int64_t count, int64_t T, int q, int q_train,
                          float grad_scale, int dtype, void* table_host, size_t table_bytes) {
    using namespace bcq;
    if (!table_host) return BCQ_ERR_NULL;
    bcq_status s = batch_check(op, layers, count, T, q, dtype, true);
    if (s != BCQ_OK) return s;
    if (op == BCQ_OP_BWD_ALPHA && (q_train < 1 || q_train > q)) return BCQ_ERR_SHAPE;
    const BatchTotals t = batch_totals(op, layers, count, T, q);
    if (t.pre_blocks > 0x7FFFFFFFull || t.main_blocks[0] > 0x7FFFFFFFull || t.main_blocks[1] > 0x7FFFFFFFull)
        return BCQ_ERR_SHAPE;
    if (table_bytes < t.table_bytes) return BCQ_ERR_WORKSPACE;

    unsigned char* base = static_cast<unsigned char*>(table_host);
    memset(base, 0, t.table_bytes);
    BatchHeader h = {};
    h.magic = kBatchMagic;
    h.version = kBatchVersion;
    h.op = op;
    h.q = q;
    h.q_used = (op == BCQ_OP_BWD_ALPHA) ? q_train : q;
    h.T = (int32_t)T;
    h.halves = T <= 8 ? 1 : 2;
    h.count = (int32_t)count;
    h.scale = (op == BCQ_OP_BWD_ALPHA) ? grad_scale : 1.f;
    h.pre_blocks = (uint32_t)t.pre_blocks;
    h.pre_sets = (op == BCQ_OP_BWD_INPUT) ? (uint32_t)q : 1u;
    h.main_blocks[0] = (uint32_t)t.main_blocks[0];
    h.main_blocks[1] = (uint32_t)t.main_blocks[1];
    h.layers_off = sizeof(BatchHeader);
    h.pre_map_off = h.layers_off + (uint64_t)count * sizeof(BatchLayerDev);
    h.main_map_off[0] = h.pre_map_off + t.pre_blocks * sizeof(uint2);
    h.main_map_off[1] = h.main_map_off[0] + t.main_blocks[0] * sizeof(uint2);
    h.table_bytes = t.table_bytes;
    h.workspace_bytes = t.workspace_bytes;
    h.plane_bytes = t.plane_bytes;

    BatchLayerDev* dl = reinterpret_cast<BatchLayerDev*>(base + h.layers_off);
    uint2* pre_map = reinterpret_cast<uint2*>(base + h.pre_map_off);
    struct Item { uint32_t layer, bx; int32_t weight; };
    std::vector<Item> items[2];
    items[0].reserve(t.main_blocks[0]);
    items[1].reserve(t.main_blocks[1]);
    size_t ws_off = 0;
    uint64_t pb = 0;
    for (int64_t l = 0; l < count; ++l) {
        const bcq_batch_layer& b = layers[l];
        const BatchShape sh = batch_shape(op, T, b.N, b.K, q);
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
        d.seg_magic = (uint32_t)((((uint64_t)1 << 32) + (uint64_t)sh.segs_act - 1) / (uint64_t)sh.segs_act);
        dl[l] = d;
        for (int32_t sg = 0; sg < sh.segs_act; ++sg) pre_map[pb++] = make_uint2((uint32_t)l, (uint32_t)sg);
        for (uint32_t bx = 0; bx < sh.main_blocks; ++bx) items[sh.form].push_back(Item{(uint32_t)l, bx, sh.segs_main});
    }
    // The hardware starts workgroups in index order as compute units free up: the longest ones go first, so that the
    // launch does not end with a few long workgroups running alone.
    for (int f = 0; f < 2; ++f) {
        std::stable_sort(items[f].begin(), items[f].end(), [](const Item& a, const Item& b2) { return a.weight > b2.weight; });
        uint2* map = reinterpret_cast<uint2*>(base + h.main_map_off[f]);
        for (size_t i = 0; i < items[f].size(); ++i) map[i] = make_uint2(items[f][i].layer, items[f][i].bx);
    }
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
        case BCQ_OP_FWD:
            e = launch_pre<STREAM_FWD>(h, dev, ws, st);
            if (e == hipSuccess) e = launch_main_lds<STREAM_FWD>(h, dev, ws, st);
            break;
        case BCQ_OP_BWD_ALPHA:
            e = launch_pre<STREAM_DALPHA>(h, dev, ws, st);
            if (e == hipSuccess) e = launch_main_lds<STREAM_DALPHA>(h, dev, ws, st);
            break;
        case BCQ_OP_BWD_INPUT:
            e = launch_pre<STREAM_DX>(h, dev, ws, st);
            if (e == hipSuccess && h.main_blocks[BATCH_MAIN_LDS]) e = launch_main_lds<STREAM_DX>(h, dev, ws, st);
            if (e == hipSuccess && h.main_blocks[BATCH_MAIN_WAVE]) e = launch_main_wave(h, dev, ws, st);
            break;
        default: return BCQ_ERR_DTYPE;
    }
    return e == hipSuccess ? BCQ_OK : BCQ_ERR_DEVICE;
}

}  // extern "C"
