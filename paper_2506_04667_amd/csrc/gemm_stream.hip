// Kernels and launchers of the weight-streaming grouped GEMM of the expert FFN tasks; the workgroup's work is in
// gemm_stream_body.h.
#include "gemm_stream_body.h"

namespace moe {
namespace {

template <class S, int ACT0, int NPH>
__global__ __launch_bounds__(THREADS) void ffn_gemm_stream_kernel(StreamArgs a) {
    const int xcd = blockIdx.x % kXcds, wg = blockIdx.x / kXcds, wgs = gridDim.x / kXcds;
    if constexpr (NPH == 1) {
        stream_gemm<S, ACT0, 0, false, false>(a, xcd, wg, wgs);
    } else {
        if (threadIdx.x == 0) check_xcd_placement(a, xcd);
        stream_gemm<S, ACT0, 0, true, false>(a, xcd, wg, wgs);
        __syncthreads();
        stream_gemm<S, 3, 1, false, true>(a, xcd, wg, wgs);
    }
}

__global__ __launch_bounds__(1024) void ffn_units_kernel(const int32_t* __restrict__ rows_dev, int rows_cap, int groups,
                                                         int max_rows, int32_t* __restrict__ w) {
    __shared__ int wave_total[32];
    build_ffn_units(rows_dev, rows_cap, groups, max_rows, w, wave_total, 1024);
}

// the kernel's LDS limit on the current device (once per device)
template <class S, int ACT0, int NPH>
hipError_t prepare_stream_t() {
    static DeviceFlags limit_raised = {};
    return raise_lds_limit(reinterpret_cast<const void*>(ffn_gemm_stream_kernel<S, ACT0, NPH>), LDS_BYTES, limit_raised);
}

// g2 == nullptr: one GEMM.  Otherwise g2's A is g1's C and both share rows/groups/units.
template <class S, int ACT0, int NPH>
hipError_t launch_stream_t(const GemmArgs& g1, const GemmArgs* g2, bool never_met, hipStream_t stream) {
    auto kernel = ffn_gemm_stream_kernel<S, ACT0, NPH>;
    if (hipError_t e = prepare_stream_t<S, ACT0, NPH>(); e != hipSuccess) return e;
    // units the lists can hold: every large row tile of every group, and one small tile per group
    const int nrow_l = ffn_units_nrow_large(g1.max_rows);
    const long long cap = (long long)g1.groups * (nrow_l + 1);
    const long long ncol0 = (g1.N + BN - 1) / BN, ncol1 = g2 ? (g2->N + BN - 1) / BN : 0;
    const long long ncol = ncol0 > ncol1 ? ncol0 : ncol1;
    const long long total = cap * ncol;                                   // upper bound of the live tasks of a GEMM
    if ((long long)g1.groups * ffn_units_nrow_small(g1.max_rows) > 0x7fffffffLL / (ncol > kXcds ? ncol : kXcds))
        return hipErrorInvalidValue;
    // one persistent workgroup per CU, the same number on every XCD, never more workgroups than CUs
    long long grid = device_cu_count() / kXcds * kXcds;
    if (grid < kXcds) return hipErrorInvalidValue;
    const long long need = (total + kXcds - 1) / kXcds * kXcds;
    if (grid > need) grid = need;
    StreamArgs a{};
    a.ph[0] = to_phase(g1);
    if (g2) a.ph[1] = to_phase(*g2);
    a.rows_dev = g1.rows_dev; a.rows_cap = g1.rows_cap; a.max_rows = g1.max_rows;
    a.lists = const_cast<int32_t*>(g1.units);
    a.groups = g1.groups;
    // every wavefront of every first-GEMM column tile of a unit counts once
    a.wait_target = never_met ? 0x7fffffff : (int)ncol0 * (THREADS / 64);
    a.spin_limit = never_met ? 16 : kSpinLimit;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(THREADS), LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class S, int NPH>
hipError_t launch_stream_act(const GemmArgs& g1, const GemmArgs* g2, bool never_met, hipStream_t stream) {
    if constexpr (NPH == 1) {
        if (g1.c_f32) return launch_stream_t<S, kActF32Out, 1>(g1, nullptr, never_met, stream);
    }
    switch (g1.act) {
        case 0: return launch_stream_t<S, 0, NPH>(g1, g2, never_met, stream);
        case 1: return launch_stream_t<S, 1, NPH>(g1, g2, never_met, stream);
        case 2: return launch_stream_t<S, 2, NPH>(g1, g2, never_met, stream);
        default: return launch_stream_t<S, 3, NPH>(g1, g2, never_met, stream);
    }
}

template <class S>
hipError_t prepare_stream_s() {
    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = prepare_stream_t<S, 0, 1>();
    if (e == hipSuccess) e = prepare_stream_t<S, 1, 1>();
    if (e == hipSuccess) e = prepare_stream_t<S, 2, 1>();
    if (e == hipSuccess) e = prepare_stream_t<S, 3, 1>();
    if (e == hipSuccess) e = prepare_stream_t<S, kActF32Out, 1>();
    if (e == hipSuccess) e = prepare_stream_t<S, 0, 2>();
    if (e == hipSuccess) e = prepare_stream_t<S, 1, 2>();
    if (e == hipSuccess) e = prepare_stream_t<S, 2, 2>();
    if (e == hipSuccess) e = prepare_stream_t<S, 3, 2>();
    return e;
}

}  // namespace

int device_cu_count() {
    static std::atomic<int> cus[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

hipError_t prepare_grouped_gemm_stream() {
    const hipError_t e = prepare_stream_s<BF16>();
    return e != hipSuccess ? e : prepare_stream_s<F16>();
}

size_t ffn_units_ints(int groups, int max_rows) { return (size_t)ffn_units_total_ints(groups, max_rows); }

hipError_t launch_ffn_units(const int32_t* rows_dev, int rows_cap, int groups, int max_rows, int32_t* units,
                            hipStream_t stream) {
    hipLaunchKernelGGL(ffn_units_kernel, dim3(1), dim3(1024), 0, stream, rows_dev, rows_cap, groups, max_rows, units);
    return hipGetLastError();
}

void ffn_units_fault_words(int groups, int max_rows, long long* first, long long* second) {
    *second = ffn_units_small_offset(groups, max_rows);
    *first = ffn_units_nrow_large(max_rows) ? 0 : *second;
}

bool stream_gemm_shape_ok(int dtype, int N, int K, int lda, int ldb, int ldc, long long a_rows_total) {
    return dtype != 0 && K % (2 * BK) == 0 && K >= 6 * BK && N % 8 == 0 && N >= 256 && lda % 8 == 0 && ldb % 8 == 0 &&
           ldc % 8 == 0 &&
           // copies address an operand as a 64-bit base plus 32-bit byte offsets
           a_rows_total * lda * 2 < (1ll << 32) && (long long)K * ldb * 2 < (1ll << 32);
}

bool stream_gemm_eligible(const GemmArgs& a) {
    // fp32 output (the weight gradients of the backward pass): identity epilogue only
    if (a.c_f32 && a.act != 3) return false;
    return !a.b_is_nk && a.rows_dev != nullptr && a.units != nullptr &&
           stream_gemm_shape_ok(a.dtype, a.N, a.K, a.lda, a.ldb, a.ldc, a.a_rows_total);
}

hipError_t launch_grouped_gemm_stream(const GemmArgs& a, hipStream_t stream) {
    return a.dtype == 1 ? launch_stream_act<BF16, 1>(a, nullptr, false, stream) : launch_stream_act<F16, 1>(a, nullptr, false, stream);
}

bool ffn_fused_eligible(const GemmArgs& g1, const GemmArgs& g2) {
    return stream_gemm_eligible(g1) && stream_gemm_eligible(g2) && !g1.c_f32 && !g2.c_f32 && g2.act == 3 && g2.a_row_index == nullptr &&
           g1.units == g2.units && g1.rows_dev == g2.rows_dev && g1.rows_cap == g2.rows_cap &&
           g1.groups == g2.groups && g1.max_rows == g2.max_rows && g1.dtype == g2.dtype;
}

hipError_t launch_ffn_stream_fused(const GemmArgs& g1, const GemmArgs& g2, bool never_met, hipStream_t stream) {
    return g1.dtype == 1 ? launch_stream_act<BF16, 2>(g1, &g2, never_met, stream) : launch_stream_act<F16, 2>(g1, &g2, never_met, stream);
}

}  // namespace moe
