// Combine (task t3 of Sec. 3.1, C <- A (.) S + C; Eq. "combine 2"), built as a
// deterministic gather-reduce: one workgroup per token sums its kept expert
// output rows, scaled by the combine weights, in ascending choice order, in fp32.
#include "common.h"
#include "kernels.h"

namespace moe {
namespace {

template <class S>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ y, const int32_t* __restrict__ topk_expert,
                                                      const float* __restrict__ topk_weight,
                                                      const int32_t* __restrict__ slot, int H, int k, int E,
                                                      int C, int C_pad, void* __restrict__ out) {
    constexpr int VEC = S::kVec;
    const int t = blockIdx.x;
    const int row_chunks = H / VEC;
    for (int c = threadIdx.x; c < row_chunks; c += blockDim.x) {
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        // choices four at a time: first their routing entries, then all their row chunks in flight together,
        // then the sums in ascending choice order
        for (int j0 = 0; j0 < k; j0 += 4) {
            float w[4];
            size_t row[4];
            bool live[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + q;
                live[q] = false;
                w[q] = 0.0f;
                row[q] = 0;
                if (j < k) {
                    const int s = slot[(size_t)t * k + j];
                    const int e = topk_expert[(size_t)t * k + j];
                    w[q] = topk_weight[(size_t)t * k + j];
                    live[q] = s >= 0 && s < C && e >= 0 && e < E;
                    if (live[q]) row[q] = (size_t)e * C_pad + s;
                }
            }
            u32x4 v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (live[q]) v[q] = ((const u32x4*)y)[row[q] * row_chunks + c];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (!live[q]) continue;
                if constexpr (S::kBytes == 4) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t u = v[q][i];   // copy out first: bit_cast of a vector element reads lane 0
                        acc[i] = fmaf(w[q], __builtin_bit_cast(float, u), acc[i]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t u = v[q][i];
                        acc[2 * i] = fmaf(w[q], bits16_to_float<S>((uint16_t)(u & 0xffffu)), acc[2 * i]);
                        acc[2 * i + 1] = fmaf(w[q], bits16_to_float<S>((uint16_t)(u >> 16)), acc[2 * i + 1]);
                    }
                }
            }
        }
        u32x4 o;
        if constexpr (S::kBytes == 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = __builtin_bit_cast(uint32_t, acc[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[i] = (uint32_t)float_to_bits16<S>(acc[2 * i]) | ((uint32_t)float_to_bits16<S>(acc[2 * i + 1]) << 16);
        }
        ((u32x4*)out)[(size_t)t * row_chunks + c] = o;
    }
}

}  // namespace

hipError_t launch_combine(const void* y, const int32_t* topk_expert, const float* topk_weight,
                          const int32_t* slot, int T, int H, int k, int E, int C, int C_pad, int dtype,
                          void* out, hipStream_t stream) {
    if (dtype == 0)
        hipLaunchKernelGGL(combine_kernel<F32>, dim3(T), dim3(256), 0, stream, y, topk_expert, topk_weight, slot, H, k, E, C, C_pad, out);
    else if (dtype == 1)
        hipLaunchKernelGGL(combine_kernel<BF16>, dim3(T), dim3(256), 0, stream, y, topk_expert, topk_weight, slot, H, k, E, C, C_pad, out);
    else
        hipLaunchKernelGGL(combine_kernel<F16>, dim3(T), dim3(256), 0, stream, y, topk_expert, topk_weight, slot, H, k, E, C, C_pad, out);
    return hipGetLastError();
}

}  // namespace moe
