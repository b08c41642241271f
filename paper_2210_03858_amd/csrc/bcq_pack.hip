// Bit-plane pack / unpack and the transposed twin (gfx950, wave64).
// Layout: AlphaTuning Table 1 gives B the index order (q, h_out, h_in); one uint32 holds 32 consecutive
// columns, bit j = column 32w + j, 1 <=> +1.  All three kernels are pure data movement, HBM bound.
#include "bcq_internal.h"

namespace bcq {

// 4 sign bits of 4 packed int8 (bit = 1 where the byte is >= 0), byte 0 -> bit 0
__device__ __forceinline__ uint32_t nonneg_bits4(uint32_t u) {
    uint32_t m = ((~u) >> 7) & 0x01010101u;
    return (m | (m >> 7) | (m >> 14) | (m >> 21)) & 0xFu;
}

// One thread reads 16 int8 (one 16-byte load) and forms 16 bits; an even/odd lane pair forms one word.
__global__ __launch_bounds__(256) void pack_kernel(const int8_t* __restrict__ planes, int64_t total_words,
                                                   uint32_t* __restrict__ packed) {
    int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool live = tid < 2 * total_words;
    uint32_t bits = 0;
    if (live) {
        uint4 v = *reinterpret_cast<const uint4*>(planes + 16 * tid);
        bits = nonneg_bits4(v.x) | (nonneg_bits4(v.y) << 4) | (nonneg_bits4(v.z) << 8) | (nonneg_bits4(v.w) << 12);
    }
    uint32_t hi = __shfl_down(bits, 1);
    if (live && !(threadIdx.x & 1)) packed[tid >> 1] = bits | (hi << 16);
}

__device__ __forceinline__ uint32_t expand4(uint32_t b) {  // 4 bits -> 4 int8 of +1 / -1
    uint32_t r = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) r |= (((b >> j) & 1u) ? 0x01u : 0xFFu) << (8 * j);
    return r;
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ packed, int64_t total_words,
                                                     int8_t* __restrict__ planes) {
    int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tid >= 2 * total_words) return;
    uint32_t b = (packed[tid >> 1] >> ((tid & 1) * 16)) & 0xFFFFu;
    uint4 v;
    v.x = expand4(b);
    v.y = expand4(b >> 4);
    v.z = expand4(b >> 8);
    v.w = expand4(b >> 12);
    *reinterpret_cast<uint4*>(planes + 16 * tid) = v;
}

// In-register transpose of a 32 x 32 bit block, row r = a[r], column c = bit c (LSB = column 0):
// five rounds of swapping the off-diagonal sub-blocks of size s = 16, 8, 4, 2, 1.
__device__ __forceinline__ void transpose32(uint32_t (&a)[32]) {
#pragma unroll
    for (int s = 16; s >= 1; s >>= 1) {
        uint32_t m = 0xFFFFFFFFu / ((1u << s) + 1u);  // columns c with (c & s) == 0
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            if (r & s) continue;
            uint32_t t = ((a[r] >> s) ^ a[r + s]) & m;
            a[r + s] ^= t;
            a[r] ^= t << s;
        }
    }
}

// Tile: 16 row blocks (512 rows of W) x 16 words (512 columns).  Thread (vb, wb) transposes one 32 x 32 block
// read with lanes running along the words of a row (coalesced); results pass through LDS so that the writes
// run along the words of a packed_t row.
constexpr int TR_VB = 16, TR_WB = 16;
__global__ __launch_bounds__(256) void transpose_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                        uint32_t* __restrict__ packed_t) {
    __shared__ uint32_t tile[TR_WB * 32][TR_VB + 1];
    const int64_t Kw = K / 32, Nw = N / 32;
    const int plane = blockIdx.z;
    const uint32_t* src = packed + (int64_t)plane * N * Kw;
    uint32_t* dst = packed_t + (int64_t)plane * K * Nw;
    const int wb = threadIdx.x % TR_WB, vb = threadIdx.x / TR_WB;
    const int64_t w = (int64_t)blockIdx.x * TR_WB + wb, v = (int64_t)blockIdx.y * TR_VB + vb;
    uint32_t a[32];
    const bool live = (w < Kw) && (v < Nw);
#pragma unroll
    for (int r = 0; r < 32; ++r) a[r] = live ? src[(32 * v + r) * Kw + w] : 0u;
    transpose32(a);
#pragma unroll
    for (int r = 0; r < 32; ++r) tile[wb * 32 + r][vb] = a[r];
    __syncthreads();
    // 512 output rows (columns k of W) x 16 words each; thread t handles word t % 16 of rows t / 16 + 16 * pass
    const int ov = threadIdx.x % TR_VB;
    const int64_t gv = (int64_t)blockIdx.y * TR_VB + ov;
    for (int row = threadIdx.x / TR_VB; row < TR_WB * 32; row += 256 / TR_VB) {
        int64_t k = (int64_t)blockIdx.x * TR_WB * 32 + row;
        if (k < K && gv < Nw) dst[k * Nw + gv] = tile[row][ov];
    }
}

hipError_t launch_pack(const int8_t* planes, int64_t total_words, uint32_t* packed, hipStream_t st) {
    int64_t threads = 2 * total_words;
    unsigned blocks = (unsigned)((threads + 255) / 256);
    BCQ_LAUNCH(pack_kernel, dim3(blocks), dim3(256), 0, st, planes, total_words, packed);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t* packed, int64_t total_words, int8_t* planes, hipStream_t st) {
    int64_t threads = 2 * total_words;
    unsigned blocks = (unsigned)((threads + 255) / 256);
    BCQ_LAUNCH(unpack_kernel, dim3(blocks), dim3(256), 0, st, packed, total_words, planes);
    return hipGetLastError();
}

hipError_t launch_pack_transposed(const uint32_t* packed, int64_t N, int64_t K, int q, uint32_t* packed_t,
                                  hipStream_t st) {
    const int64_t Kw = K / 32, Nw = N / 32;
    dim3 grid((unsigned)((Kw + TR_WB - 1) / TR_WB), (unsigned)((Nw + TR_VB - 1) / TR_VB), (unsigned)q);
    BCQ_LAUNCH(transpose_kernel, grid, dim3(256), 0, st, packed, N, K, packed_t);
    return hipGetLastError();
}

}  // namespace bcq
