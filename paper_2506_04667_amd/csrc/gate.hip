// Gate stage helpers ("FusedGate" of Alg. 1): the gate projection itself runs on
// the grouped GEMM kernel; this file holds the Wg re-layout that feeds it and the
// top-k selection with the combine weights of Eqs. "combine 1/2".
#include "common.h"
#include "kernels.h"

namespace moe {
namespace {

// WgT[n][h] = Wg[h][n]; rows n >= E are zero.  32 x 32 tiles through LDS.
template <class elem>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const elem* __restrict__ Wg, elem* __restrict__ WgT,
                                                            int H, int E, int E_pad) {
    __shared__ elem tile[32][33];
    const int h0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int h = h0 + r, n = n0 + tx;
        tile[r][tx] = (h < H && n < E) ? Wg[(size_t)h * E + n] : (elem)0;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, h = h0 + tx;
        if (n < E_pad && h < H) WgT[(size_t)n * H + h] = tile[tx][r];
    }
}

// One wavefront per token.  Selection runs k rounds of "largest remaining logit,
// smaller expert index on equal values" (a strict total order, compared as
// floats so that -0.0 and +0.0 tie), where "remaining" means strictly after the
// previous pick in that order, so no per-expert mark is needed and E is
// unbounded.  The rounds run twice: first to get the softmax denominator over the
// k selected logits, then to write experts and weights.  With IN_REGS the row
// (E <= 64 * kRegVals) is read once into registers; otherwise it is re-read.
constexpr int kRegVals = 8;

template <bool IN_REGS>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                   int32_t* __restrict__ topk_expert,
                                                   float* __restrict__ topk_weight) {
    const int token = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    if (token >= T) return;
    const float* l = logits + (size_t)token * E;
    constexpr int kNone = 0x7fffffff;
    float vals[kRegVals];
    if (IN_REGS) {
#pragma unroll
        for (int i = 0; i < kRegVals; ++i) vals[i] = lane + i * kWave < E ? l[lane + i * kWave] : 0.0f;
    }
    float m = 0.0f, sum = 0.0f;
    for (int pass = 0; pass < 2; ++pass) {
        float last_v = 0.0f;
        int last_i = -1;
        for (int j = 0; j < k; ++j) {
            float bv = 0.0f;
            int bi = kNone;
            auto consider = [&](float v, int e) {
                const bool avail = (j == 0) || (v < last_v) || (v == last_v && e > last_i);
                const bool better = (bi == kNone) || (v > bv);  // e ascends: equal values keep the earlier index
                if (avail && better) { bv = v; bi = e; }
            };
            if (IN_REGS) {
#pragma unroll
                for (int i = 0; i < kRegVals; ++i)
                    if (lane + i * kWave < E) consider(vals[i], lane + i * kWave);
            } else {
                for (int e = lane; e < E; e += kWave) consider(l[e], e);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oi = __shfl_xor(bi, off);
                if (oi != kNone && (bi == kNone || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
            }
            if (pass == 0) {
                if (j == 0) m = bv;
                sum += expf(bv - m);
            } else if (lane == 0) {
                topk_expert[(size_t)token * k + j] = bi;
                topk_weight[(size_t)token * k + j] = expf(bv - m) / sum;
            }
            last_v = bv;
            last_i = bi;
        }
    }
}

}  // namespace

hipError_t launch_transpose_pad(const void* Wg, void* WgT, int H, int E, int E_pad, int dtype,
                                hipStream_t stream) {
    dim3 grid((H + 31) / 32, (E_pad + 31) / 32);
    if (dtype == 0)
        hipLaunchKernelGGL(transpose_pad_kernel<float>, grid, dim3(256), 0, stream, (const float*)Wg, (float*)WgT, H, E, E_pad);
    else
        hipLaunchKernelGGL(transpose_pad_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t*)Wg, (uint16_t*)WgT, H, E, E_pad);
    return hipGetLastError();
}

hipError_t launch_topk(const float* logits, int T, int E, int k, int32_t* topk_expert,
                       float* topk_weight, hipStream_t stream) {
    const int tokens_per_block = 256 / kWave;
    const dim3 grid((T + tokens_per_block - 1) / tokens_per_block);
    if (E <= kWave * kRegVals)
        hipLaunchKernelGGL(topk_kernel<true>, grid, dim3(256), 0, stream, logits, T, E, k, topk_expert, topk_weight);
    else
        hipLaunchKernelGGL(topk_kernel<false>, grid, dim3(256), 0, stream, logits, T, E, k, topk_expert, topk_weight);
    return hipGetLastError();
}

}  // namespace moe
