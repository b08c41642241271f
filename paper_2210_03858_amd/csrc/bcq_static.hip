// Forward for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): bcq_linear_fwd_static is the small-token forward of bcq_linear_fwd with the
// scratch of its streaming kernels (the activations re-coded as two block-scaled FP8 terms) in a fixed array that
// is part of the library's device image instead of a caller's workspace.  See include/bcq.h for the contract.
#include "../../include/bcq.h"

#include "bcq_internal.h"

#include <mutex>

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[BCQ_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the calling thread's current device (the array's name is only a host-side handle:
// host code never passes it anywhere but to HIP_SYMBOL).  Resolved once per device; nullptr on failure.
void* scratch_address() {
    static std::mutex lock;
    static void* address[64];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(lock);
    if (!address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        address[dev] = p;
    }
    return address[dev];
}

}  // namespace

extern "C" bcq_status bcq_linear_fwd_static(const uint32_t* packed, const float* alpha, const void* x, int dtype,
                                            int64_t T, int64_t N, int64_t K, int q, void* y, void* stream) {
    using namespace bcq::host;
    if (!packed || !alpha || !x || !y) return BCQ_ERR_NULL;
    if (!shape_ok(T, N, K, q) || T > BCQ_STATIC_MAX_TOKENS) return BCQ_ERR_SHAPE;
    if (dtype != BCQ_BF16) return BCQ_ERR_DTYPE;
    if (misaligned(packed) || misaligned(alpha) || misaligned(x) || misaligned(y)) return BCQ_ERR_ALIGN;
    if (bcq::stream_fwd_workspace(T, K) > (size_t)BCQ_STATIC_SCRATCH_BYTES) return BCQ_ERR_WORKSPACE;
    if (!device_ok()) return BCQ_ERR_DEVICE;
    void* ws = scratch_address();
    if (!ws) return BCQ_ERR_DEVICE;
    // Every byte of the scratch that the main kernel reads is written by this call's pre-kernel first (padding tokens
    // and columns are written as zeros), so nothing has to be cleared between calls.
    const hipError_t e = bcq::launch_fwd_stream(packed, alpha, x, T, N, K, K, q, y, ws, (hipStream_t)stream);
    return e == hipSuccess ? BCQ_OK : BCQ_ERR_DEVICE;
}
