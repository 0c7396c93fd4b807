// Launchers of the fused gate kernel ("FusedGate" of Alg. 1); the kernel body is in gate_fused_body.h.
#include "gate_fused_body.h"

namespace moe {
namespace {

template <class S, int BN_>
__global__ __launch_bounds__(G_THREADS) void gate_fused_kernel(const unsigned char* __restrict__ x, const unsigned char* __restrict__ Wg,
                                                               const float* __restrict__ gate_bias, int T, int H, int E, int k,
                                                               float* __restrict__ logits, int32_t* __restrict__ topk_expert,
                                                               float* __restrict__ topk_weight,
                                                               int32_t* __restrict__ route_counts) {
    gate_fused_tile<S, BN_>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, (int)blockIdx.x);
}

// the kernel's LDS limit on the current device (once per device)
template <class S, int BN>
hipError_t prepare_gate_fused_t() {
    static DeviceFlags limit_raised = {};
    return raise_lds_limit(reinterpret_cast<const void*>(gate_fused_kernel<S, BN>), GateCfg<S, BN>::LDS_BYTES, limit_raised);
}

template <class S, int BN>
hipError_t launch_gate_fused_t(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k,
                               float* logits, int32_t* topk_expert, float* topk_weight, int32_t* route_counts,
                               hipStream_t stream) {
    auto kernel = gate_fused_kernel<S, BN>;
    constexpr int lds_bytes = GateCfg<S, BN>::LDS_BYTES;
    if (hipError_t e = prepare_gate_fused_t<S, BN>(); e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3((unsigned)((T + G_BM - 1) / G_BM)), dim3(G_THREADS), lds_bytes, stream,
                       (const unsigned char*)x, (const unsigned char*)Wg, gate_bias, T, H, E, k, logits, topk_expert,
                       topk_weight, route_counts);
    return hipGetLastError();
}

template <class S>
hipError_t launch_gate_fused_s(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k,
                               float* logits, int32_t* topk_expert, float* topk_weight, int32_t* route_counts,
                               hipStream_t stream) {
    if (S::kBytes == 4 && E <= 64)
        return launch_gate_fused_t<F32, 64>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
    if (E <= 128)
        return launch_gate_fused_t<S, 128>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
    return launch_gate_fused_t<S, 256>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
}

}  // namespace

hipError_t prepare_gate_fused() {
    hipError_t e = prepare_gate_fused_t<F32, 64>();
    if (e == hipSuccess) e = prepare_gate_fused_t<F32, 128>();
    if (e == hipSuccess) e = prepare_gate_fused_t<F32, 256>();
    if (e == hipSuccess) e = prepare_gate_fused_t<BF16, 128>();
    if (e == hipSuccess) e = prepare_gate_fused_t<BF16, 256>();
    if (e == hipSuccess) e = prepare_gate_fused_t<F16, 128>();
    if (e == hipSuccess) e = prepare_gate_fused_t<F16, 256>();
    return e;
}

bool gate_fused_eligible(int T, int H, int E, int k, int dtype) {
    const int el = dtype == 0 ? 4 : 2, vec = 16 / el, kt = 128 / el;
    return E % vec == 0 && E >= vec && E <= 256 && H % kt == 0 && H >= kt && k >= 1 && k <= E &&
           (long long)G_BM * H * el < (1ll << 31) && (long long)kt * E * el < (1ll << 31);
}

hipError_t launch_gate_fused(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k,
                             int dtype, float* logits, int32_t* topk_expert, float* topk_weight,
                             int32_t* route_counts, hipStream_t stream) {
    static_assert(G_BM == 64, "a workgroup's tokens are one chunk of the routing scan");
    switch (dtype) {
        case 0: return launch_gate_fused_s<F32>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
        case 1: return launch_gate_fused_s<BF16>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
        default: return launch_gate_fused_s<F16>(x, Wg, gate_bias, T, H, E, k, logits, topk_expert, topk_weight, route_counts, stream);
    }
}

}  // namespace moe
