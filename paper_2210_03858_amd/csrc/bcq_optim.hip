// AdamW step on the trained scales (AlphaTuning Appendix A: AdamW with a linear-decay learning rate; only alpha is
// trained, Section 4.1).  Element-wise over the fp32 scales and their two moment buffers; the matrix-core scale
// gradient applies the same update inside its final reduction instead of launching this kernel.
#include "bcq_internal.h"

namespace bcq {

__global__ __launch_bounds__(256) void adamw_kernel(const float* __restrict__ dalpha, int64_t count, AdamWArgs opt) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < count) adamw_apply(opt, idx, dalpha[idx]);
}

hipError_t launch_adamw(const float* dalpha, int64_t count, AdamWArgs args, hipStream_t st) {
    BCQ_LAUNCH(adamw_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, dalpha, count, args);
    return hipGetLastError();
}

}  // namespace bcq
