// Shared device-side helpers of the HIP library (storage dtypes, vector types).
// gfx950 only.  Nothing here is used by, or shared with, the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWave = 64;

// Storage element tags.  16-bit types are carried as raw bits.
struct F32 { typedef float store_t; static constexpr int kBytes = 4; static constexpr int kVec = 4; };
struct BF16 { typedef uint16_t store_t; static constexpr int kBytes = 2; static constexpr int kVec = 8; };
struct F16 { typedef uint16_t store_t; static constexpr int kBytes = 2; static constexpr int kVec = 8; };

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// round to nearest even; inputs are finite by contract (NaN kept quiet)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float f16_bits_to_float(uint16_t b) {
    return (float)__builtin_bit_cast(_Float16, b);
}
__device__ __forceinline__ uint16_t float_to_f16_bits(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);  // hardware conversion rounds to nearest even
}

template <class S> __device__ __forceinline__ float load_as_float(const void* p, size_t i);
template <> __device__ __forceinline__ float load_as_float<F32>(const void* p, size_t i) { return ((const float*)p)[i]; }
template <> __device__ __forceinline__ float load_as_float<BF16>(const void* p, size_t i) { return bf16_bits_to_float(((const uint16_t*)p)[i]); }
template <> __device__ __forceinline__ float load_as_float<F16>(const void* p, size_t i) { return f16_bits_to_float(((const uint16_t*)p)[i]); }

template <class S> __device__ __forceinline__ void store_from_float(void* p, size_t i, float v);
template <> __device__ __forceinline__ void store_from_float<F32>(void* p, size_t i, float v) { ((float*)p)[i] = v; }
template <> __device__ __forceinline__ void store_from_float<BF16>(void* p, size_t i, float v) { ((uint16_t*)p)[i] = float_to_bf16_bits(v); }
template <> __device__ __forceinline__ void store_from_float<F16>(void* p, size_t i, float v) { ((uint16_t*)p)[i] = float_to_f16_bits(v); }

template <class S> __device__ __forceinline__ float bits16_to_float(uint16_t b);
template <> __device__ __forceinline__ float bits16_to_float<BF16>(uint16_t b) { return bf16_bits_to_float(b); }
template <> __device__ __forceinline__ float bits16_to_float<F16>(uint16_t b) { return f16_bits_to_float(b); }
template <class S> __device__ __forceinline__ uint16_t float_to_bits16(float f);
template <> __device__ __forceinline__ uint16_t float_to_bits16<BF16>(float f) { return float_to_bf16_bits(f); }
template <> __device__ __forceinline__ uint16_t float_to_bits16<F16>(float f) { return float_to_f16_bits(f); }

// two fp32 values -> two 16-bit storage values packed in a dword (lo in bits 0-15), round to nearest even
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
template <class S> __device__ __forceinline__ uint32_t pack2(float lo, float hi);
template <> __device__ __forceinline__ uint32_t pack2<BF16>(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
template <> __device__ __forceinline__ uint32_t pack2<F16>(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, f16x2));
}

// erf by the rational-exponential form of Abramowitz & Stegun 7.1.26 (absolute error below 1.5e-7),
// with the hardware reciprocal and exponential: about a dozen VALU operations instead of a library call.
__device__ __forceinline__ float erf_as(float x) {
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    const float e = __expf(-ax * ax);
    return copysignf(fmaf(-p * t, e, 1.0f), x);
}
// tanh(u) = 1 - 2 / (1 + exp(2u)); saturates correctly when exp overflows or underflows
__device__ __forceinline__ float tanh_fast(float u) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * u));
}

// phi_1 of the first FFN task, on the fp32 accumulator (act codes of moe_act)
template <int ACT>
__device__ __forceinline__ float apply_act_t(float v) {
    if constexpr (ACT == 0) return fmaxf(v, 0.0f);
    else if constexpr (ACT == 1) return 0.5f * v * (1.0f + tanh_fast(0.7978845608028654f * (v + 0.044715f * v * v * v)));
    else if constexpr (ACT == 2) return 0.5f * v * (1.0f + erf_as(v * 0.7071067811865476f));
    else return v;
}
// GELU (erf form) for results that are rounded to 16-bit storage: erf(v / sqrt 2) = vc P(vc^2) with vc = v
// clamped to +-3 sqrt 2 and P a degree-8 minimax fit, so |erf error| < 2.3e-5 everywhere (the clamp costs
// erfc(3) = 2.2e-5) and the result is within 1.2e-5 |v| of the exact GELU: more than 20 times below half an
// fp16 ulp.  13 full-rate VALU operations and no transcendental, against 13 plus an exp and a reciprocal.
__device__ __forceinline__ float gelu_erf_poly(float v) {
    const float vc = __builtin_amdgcn_fmed3f(v, -4.24264069f, 4.24264069f);
    const float t = vc * vc;
    float p = 1.125445533e-10f;
    p = fmaf(p, t, -1.074439775e-08f);
    p = fmaf(p, t, 4.536786108e-07f);
    p = fmaf(p, t, -1.129272951e-05f);
    p = fmaf(p, t, 1.871838646e-04f);
    p = fmaf(p, t, -2.218813402e-03f);
    p = fmaf(p, t, 1.963627103e-02f);
    p = fmaf(p, t, -1.326938842e-01f);
    p = fmaf(p, t, 7.978062666e-01f);
    const float hv = 0.5f * v;
    return fmaf(hv, vc * p, hv);
}
// phi_1 where the result goes to bf16/fp16 storage
template <int ACT>
__device__ __forceinline__ float apply_act16_t(float v) {
    if constexpr (ACT == 2) return gelu_erf_poly(v);
    else return apply_act_t<ACT>(v);
}
__device__ __forceinline__ float apply_act(float v, int act) {
    switch (act) {
        case 0: return apply_act_t<0>(v);
        case 1: return apply_act_t<1>(v);
        case 2: return apply_act_t<2>(v);
        default: return v;
    }
}

// Host side: a kernel that uses more than 64 KB of dynamic LDS has that limit raised once per device
// (`done` is the kernel's own table of devices already served).  The tables are atomics: two host threads
// making their first call at the same time may both set the attribute (setting it twice is harmless), and
// neither reads a half-written entry.
constexpr int kMaxDevices = 64;
typedef std::atomic<bool> DeviceFlags[kMaxDevices];
inline hipError_t raise_lds_limit(const void* kernel, int bytes, DeviceFlags& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!done[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        done[dev].store(true, std::memory_order_release);
    }
    return hipSuccess;
}

}  // namespace moe
