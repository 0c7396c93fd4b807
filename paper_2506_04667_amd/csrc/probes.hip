// Yardstick kernels for the benchmark: what this chip reaches on the two resources that bound the layer, measured
// in the same process as the layer itself (see moe_probe_* in include/moe.h).  Not part of the layer.
//   stream read : every workgroup reads a contiguous share of a buffer with 16-byte loads, several in flight per
//                 lane, and folds what it read into one word (so the loads cannot be dropped);
//   stream copy : the same with a 16-byte store per load (the reference kernel for hardware traffic counters);
//   MFMA loop   : register-resident v_mfma_f32_16x16x32 (bf16 / f16) or v_mfma_f32_32x32x2 (fp32) on operand
//                 registers that hold pseudo-random finite values and rotate every step, eight independent
//                 accumulator tiles per wavefront, two wavefronts per SIMD;
//   LDS fill    : how fast a CU can bring L2-resident data into its LDS, by the two routes there are: direct copies
//                 (global_load_lds_dwordx4, what the FFN and gate kernels use) and vector loads into registers
//                 followed by ds_write_b128; and, for reference, the vector loads alone.
#include "../../include/moe.h"

#include "common.h"
#include "kernels.h"
#include "lds_copy.h"

namespace moe {
namespace {

constexpr int kProbeThreads = 256;
constexpr int kUnroll = 8;

template <bool COPY>
__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                     size_t n_vec, uint32_t* __restrict__ sink) {
    // workgroup b owns vectors [b * per, (b + 1) * per); inside it the threads stride by the workgroup size
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n_vec ? lo + per : n_vec;
    u32x4 fold = {0u, 0u, 0u, 0u};
    size_t i = lo + threadIdx.x;
    for (; i + (size_t)(kUnroll - 1) * kProbeThreads < hi; i += (size_t)kUnroll * kProbeThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * kProbeThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (COPY) __builtin_nontemporal_store(v[u], dst + i + (size_t)u * kProbeThreads);
            else fold ^= v[u];
        }
    }
    for (; i < hi; i += kProbeThreads) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        if (COPY) __builtin_nontemporal_store(v, dst + i);
        else fold ^= v;
    }
    if (!COPY) {
        const uint32_t w = fold[0] ^ fold[1] ^ fold[2] ^ fold[3];
        if (w == 0x9e3779b9u) sink[0] = w;              // practically never: keeps the loads alive without a store per thread
    }
}

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
// a finite 16-bit pattern of magnitude about 2^-6 .. 2^-5 with random sign and mantissa
__device__ __forceinline__ uint32_t probe_pair16(uint32_t h, bool bf16) {
    const uint32_t lo = bf16 ? (0x3c80u | (h & 0x807fu)) : (0x2400u | (h & 0x83ffu));
    const uint32_t g = h >> 16;
    const uint32_t hi = bf16 ? (0x3c80u | (g & 0x807fu)) : (0x2400u | (g & 0x83ffu));
    return lo | (hi << 16);
}

template <int DT>                                       // moe_dtype
__global__ __launch_bounds__(512) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
    const uint32_t seed = probe_hash(blockIdx.x * 512u + threadIdx.x + 1u);
    float total = 0.0f;
    if constexpr (DT == 0) {
        f32x16 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;
        float a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            a[j] = __builtin_bit_cast(float, 0x3c000000u | (probe_hash(seed + j) & 0x807fffffu));
            b[j] = __builtin_bit_cast(float, 0x3c000000u | (probe_hash(seed + 7 * j + 3) & 0x807fffffu));
        }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(j + s) & 3], b[(2 * j + s) & 3], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) total += acc[j][q];
    } else {
        f32x4 acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[j][q] = 0.0f;
        u32x4 a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a[j][q] = probe_pair16(probe_hash(seed + 16 * j + q), DT == 1);
                b[j][q] = probe_pair16(probe_hash(seed + 16 * j + q + 8), DT == 1);
            }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const u32x4 av = a[(j + s) & 3], bv = b[(3 * j + s) & 3];
                    if constexpr (DT == 1)
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), acc[j], 0, 0, 0);
                    else
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, av), __builtin_bit_cast(f16x8, bv), acc[j], 0, 0, 0);
                }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) total += acc[j][q];
    }
    if (total == 12345.678f) sink[0] = total;           // keeps the loop alive
}

// One workgroup per CU, 8 wavefronts; per step a wavefront moves 8 KB (eight 1 KB pieces, lane i 16 bytes of each),
// the workgroup 64 KB.  The workgroups of an XCD (block number modulo 8) walk the same region of `region` bytes round
// and round from different starting points, so after the first lap everything comes from that XCD's L2.
// MODE 0: direct copies, the previous step's eight still in flight while this step's are issued.
// MODE 1: vector loads into registers, double-buffered by step, then ds_write_b128.   MODE 2: the loads alone.
constexpr int kFillThreads = 512, kFillPieces = 8, kFillStep = (kFillThreads / 64) * kFillPieces * 1024;
template <int MODE>
__global__ __launch_bounds__(kFillThreads) void lds_fill_probe_kernel(const unsigned char* __restrict__ src, size_t region, int steps,
                                                                      uint32_t* __restrict__ sink) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = uniform((int)(threadIdx.x >> 6));
    const unsigned char* const base = uniform(src + (size_t)(blockIdx.x % 8) * region);
    const size_t steps_per_lap = region / kFillStep;
    size_t at = (size_t)(blockIdx.x / 8) % steps_per_lap;             // step position inside the region
    const uint32_t lds_wave = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)smem + wave * (2 * kFillPieces * 1024);
    const uint32_t lane_off = wave * (kFillPieces * 1024) + lane * 16;
    u32x4 fold = {0u, 0u, 0u, 0u};
    if constexpr (MODE == 0) {
        for (int it = 0; it < steps; ++it) {
            const unsigned char* p = base + at * kFillStep;
#pragma unroll
            for (int j = 0; j < kFillPieces; ++j) copy_to_lds(p, lane_off + j * 1024, lds_wave + ((it & 1) * kFillPieces + j) * 1024);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFillPieces) : "memory");
            at = at + 1 == steps_per_lap ? 0 : at + 1;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        u32x4 a[kFillPieces], b[kFillPieces];
        auto load = [&](u32x4 (&r)[kFillPieces]) __attribute__((always_inline)) {
            const unsigned char* p = base + at * kFillStep + lane_off;
#pragma unroll
            for (int j = 0; j < kFillPieces; ++j) r[j] = *(const u32x4*)(p + j * 1024);
            at = at + 1 == steps_per_lap ? 0 : at + 1;
        };
        auto put = [&](const u32x4 (&r)[kFillPieces], int half) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < kFillPieces; ++j) {
                if constexpr (MODE == 1) {
                    const uint32_t d = lds_wave + (half * kFillPieces + j) * 1024 + lane * 16;
                    asm volatile("ds_write_b128 %0, %1" ::"v"(d), "v"(r[j]) : "memory");
                } else {
                    fold ^= r[j];
                }
            }
        };
        load(a);
        for (int it = 0; it + 1 < steps; it += 2) {
            load(b);
            put(a, 0);
            load(a);
            put(b, 1);
        }
        put(a, 0);
    }
    __syncthreads();
    const uint32_t w = fold[0] ^ fold[1] ^ fold[2] ^ fold[3] ^ ((const uint32_t*)smem)[threadIdx.x];
    if (w == 0x9e3779b9u) sink[0] = w;                  // practically never: keeps the work alive
}

}  // namespace
}  // namespace moe

extern "C" {

moe_status moe_probe_lds_fill(int32_t mode, const void* src, size_t region_bytes, int32_t steps, void* sink, double* bytes_moved,
                              void* stream) {
    if (!src || !sink || mode < 0 || mode > 2 || steps < 2 || (steps & 1) || region_bytes < (size_t)moe::kFillStep ||
        region_bytes % moe::kFillStep || ((uintptr_t)src & 15u))
        return MOE_ERR_INVALID_ARG;
    const int grid = moe::device_cu_count();
    const int lds = 8 * 2 * moe::kFillPieces * 1024;                  // two steps of every wavefront
    auto launch = [&](void (*kernel)(const unsigned char*, size_t, int, uint32_t*)) {
        // a yardstick, not a hot path: the LDS limit is set on every call
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return MOE_ERR_HIP;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(moe::kFillThreads), lds, (hipStream_t)stream, (const unsigned char*)src, region_bytes,
                           steps, (uint32_t*)sink);
        return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
    };
    if (bytes_moved) *bytes_moved = (double)moe::kFillStep * ((mode == 0) ? steps : steps + 1) * grid;
    if (mode == 0) return launch(moe::lds_fill_probe_kernel<0>);
    if (mode == 1) return launch(moe::lds_fill_probe_kernel<1>);
    return launch(moe::lds_fill_probe_kernel<2>);
}

moe_status moe_probe_stream(const void* src, void* dst, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes < 16 || (bytes & 15u) || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return MOE_ERR_INVALID_ARG;
    const size_t n_vec = bytes / 16;
    // eight workgroups per CU keep every memory channel busy
    size_t grid = (size_t)moe::device_cu_count() * 8;
    const size_t need = (n_vec + moe::kProbeThreads - 1) / moe::kProbeThreads;
    if (grid > need) grid = need;
    if (dst)
        hipLaunchKernelGGL(moe::stream_probe_kernel<true>, dim3((unsigned)grid), dim3(moe::kProbeThreads), 0, (hipStream_t)stream,
                           (const moe::u32x4*)src, (moe::u32x4*)dst, n_vec, (uint32_t*)sink);
    else
        hipLaunchKernelGGL(moe::stream_probe_kernel<false>, dim3((unsigned)grid), dim3(moe::kProbeThreads), 0, (hipStream_t)stream,
                           (const moe::u32x4*)src, (moe::u32x4*)nullptr, n_vec, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_probe_mfma(int32_t dtype, int32_t iters, void* sink, double* flops, void* stream) {
    if (!sink || iters <= 0 || dtype < MOE_F32 || dtype > MOE_F16) return MOE_ERR_INVALID_ARG;
    const int grid = moe::device_cu_count();            // 8 wavefronts per CU: two per SIMD
    const double per_wave_step = dtype == MOE_F32 ? 16.0 * (2.0 * 32 * 32 * 2) : 32.0 * (2.0 * 16 * 16 * 32);
    if (flops) *flops = per_wave_step * iters * 8.0 * grid;
    if (dtype == MOE_F32) hipLaunchKernelGGL(moe::mfma_probe_kernel<0>, dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, (float*)sink);
    else if (dtype == MOE_BF16) hipLaunchKernelGGL(moe::mfma_probe_kernel<1>, dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, (float*)sink);
    else hipLaunchKernelGGL(moe::mfma_probe_kernel<2>, dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, (float*)sink);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
