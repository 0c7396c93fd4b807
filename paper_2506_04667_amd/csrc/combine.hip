// Kernel and launcher of the combine (task t3 of Sec. 3.1; Eq. "combine 2"); the wavefront's work is in combine_body.h.
#include "combine_body.h"

namespace moe {
namespace {

template <class S>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const void* __restrict__ y, const int32_t* __restrict__ topk_expert,
                                                                  const float* __restrict__ topk_weight,
                                                                  const int32_t* __restrict__ slot, int T, int H, int k, int E,
                                                                  int C, int C_pad, void* __restrict__ out) {
    combine_tokens<S>(y, topk_expert, topk_weight, slot, T, H, k, E, C, C_pad, out,
                      (int)(blockIdx.x * (kCombineThreads / 64) + (threadIdx.x >> 6)), (int)(gridDim.x * (kCombineThreads / 64)));
}

}  // namespace

hipError_t launch_combine(const void* y, const int32_t* topk_expert, const float* topk_weight,
                          const int32_t* slot, int T, int H, int k, int E, int C, int C_pad, int dtype,
                          void* out, hipStream_t stream) {
    // four wavefronts per SIMD on every CU, or one wavefront per token if that is fewer
    const long long per_wg = kCombineThreads / 64;
    long long grid = (long long)device_cu_count() * 4;
    const long long need = (T + per_wg - 1) / per_wg;
    if (grid > need) grid = need;
    const dim3 g((unsigned)grid), b(kCombineThreads);
    if (dtype == 0)
        hipLaunchKernelGGL(combine_kernel<F32>, g, b, 0, stream, y, topk_expert, topk_weight, slot, T, H, k, E, C, C_pad, out);
    else if (dtype == 1)
        hipLaunchKernelGGL(combine_kernel<BF16>, g, b, 0, stream, y, topk_expert, topk_weight, slot, T, H, k, E, C, C_pad, out);
    else
        hipLaunchKernelGGL(combine_kernel<F16>, g, b, 0, stream, y, topk_expert, topk_weight, slot, T, H, k, E, C, C_pad, out);
    return hipGetLastError();
}

}  // namespace moe
