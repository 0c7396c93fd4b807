// Helper kernels of the layer's backward pass (gradients under a fixed routing; the paper leaves training to
// future work, so this follows the chain rule of Eq. "ffn" and Eqs. "combine 1/2" as stated in include/moe.h).
// The dense contractions of the backward pass run on the grouped GEMM kernels; what is here is the data movement
// and elementwise work between them: gathering rows through the routing table, the activation and its
// derivative, the softmax Jacobian of the gate, transposes that turn weight-gradient products into row-major
// GEMMs, column sums for the bias gradients, and the final gather of dx.  Every reduction has a fixed order, so
// gradients are bit-identical from run to run.
#include "common.h"
#include "kernels.h"

namespace moe {
namespace {

// derivative of phi_1 at the pre-activation v (act codes of moe_act)
__device__ __forceinline__ float act_grad(float v, int act) {
    switch (act) {
        case 0: return v > 0.0f ? 1.0f : 0.0f;
        case 1: {
            const float c = 0.7978845608028654f;
            const float t = tanh_fast(c * (v + 0.044715f * v * v * v));
            return 0.5f * (1.0f + t) + 0.5f * v * (1.0f - t * t) * c * (1.0f + 3.0f * 0.044715f * v * v);
        }
        case 2: return 0.5f * (1.0f + erf_as(v * 0.7071067811865476f)) + v * __expf(-0.5f * v * v) * 0.3989422804014327f;
        default: return 1.0f;
    }
}

// 16 bytes that this kernel reads once: the non-temporal hint (on this chip reads of data that is not in any cache run at
// half the rate without it)
__device__ __forceinline__ u32x4 load_once(const void* base, size_t chunk) { return __builtin_nontemporal_load((const u32x4*)base + chunk); }

// a 16-byte chunk of storage <-> its S::kVec values as floats
template <class S>
__device__ __forceinline__ void chunk_to_floats(const u32x4& v, float (&f)[S::kVec]) {
    if constexpr (S::kBytes == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) { const uint32_t u = v[q]; f[q] = __builtin_bit_cast(float, u); }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t u = v[q];
            f[2 * q] = bits16_to_float<S>((uint16_t)(u & 0xffffu));
            f[2 * q + 1] = bits16_to_float<S>((uint16_t)(u >> 16));
        }
    }
}
template <class S>
__device__ __forceinline__ u32x4 floats_to_chunk(const float (&f)[S::kVec]) {
    u32x4 v;
    if constexpr (S::kBytes == 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = __builtin_bit_cast(uint32_t, f[q]);
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (uint32_t)float_to_bits16<S>(f[2 * q]) | ((uint32_t)float_to_bits16<S>(f[2 * q + 1]) << 16);
    }
    return v;
}

// One workgroup per slot row (e, s), s < C_pad: xe[e, s, :] = x[token, :] and gy[e, s, :] = w * dout[token, :]
// for a live slot, zeros for an empty one (so that the rows beyond an expert's live rows contribute nothing to
// the weight-gradient products, which run over all C_pad rows).  16 bytes per lane.
template <class S>
__global__ __launch_bounds__(256) void bwd_gather_kernel(const void* __restrict__ x, const void* __restrict__ dout,
                                                         const int32_t* __restrict__ slot_token, const float* __restrict__ slot_weight,
                                                         int H, int C, int C_pad, void* __restrict__ xe, void* __restrict__ gy) {
    constexpr int VEC = S::kVec;
    const size_t row = blockIdx.x;
    const int e = (int)(row / C_pad), s = (int)(row % C_pad);
    const int tok = s < C ? slot_token[(size_t)e * C + s] : -1;
    const float w = tok >= 0 ? slot_weight[(size_t)e * C + s] : 0.0f;
    const int row_chunks = H / VEC;
    for (int c = threadIdx.x; c < row_chunks; c += 256) {
        u32x4 xv = {0u, 0u, 0u, 0u}, gv = {0u, 0u, 0u, 0u};
        if (tok >= 0) {
            xv = load_once(x, (size_t)tok * row_chunks + c);
            float f[VEC];
            chunk_to_floats<S>(load_once(dout, (size_t)tok * row_chunks + c), f);
#pragma unroll
            for (int q = 0; q < VEC; ++q) f[q] *= w;
            gv = floats_to_chunk<S>(f);
        }
        ((u32x4*)xe)[row * row_chunks + c] = xv;
        ((u32x4*)gy)[row * row_chunks + c] = gv;
    }
}

// Over [E, C_pad, I]: MODE 0: out = phi(a); MODE 1: out = g * phi'(a); rows at or beyond the expert's live rows give 0.
template <class S, int MODE>
__global__ __launch_bounds__(256) void bwd_act_kernel(const void* __restrict__ a, const void* __restrict__ g,
                                                      const int32_t* __restrict__ expert_demand, int C, int C_pad, int I, int act,
                                                      void* __restrict__ out) {
    constexpr int VEC = S::kVec;
    const size_t row = blockIdx.x;
    const int e = (int)(row / C_pad), s = (int)(row % C_pad);
    const bool live = s < min(expert_demand[e], C);
    const int row_chunks = I / VEC;
    for (int c = threadIdx.x; c < row_chunks; c += 256) {
        u32x4 o = {0u, 0u, 0u, 0u};
        if (live) {
            float av[VEC], v[VEC];
            chunk_to_floats<S>(load_once(a, row * row_chunks + c), av);
            if constexpr (MODE == 0) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) v[q] = apply_act(av[q], act);
            } else {
                float gf[VEC];
                chunk_to_floats<S>(load_once(g, row * row_chunks + c), gf);
#pragma unroll
                for (int q = 0; q < VEC; ++q) v[q] = gf[q] * act_grad(av[q], act);
            }
            o = floats_to_chunk<S>(v);
        }
        ((u32x4*)out)[row * row_chunks + c] = o;
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// One wavefront per token (k <= 64): dL/dw_ij = <dout_i, y_ij> for kept pairs (0 for dropped ones), then the
// Jacobian of the softmax over the k selected logits: dl_ij = w_ij (dL/dw_ij - sum_j' w_ij' dL/dw_ij').
// Writes dl[T, k] (fp32) and the dense matrix dL[T, ld] (storage type, zero where the token did not select the
// expert), which turns dWg = x^T dL into a GEMM.
template <class S>
__global__ __launch_bounds__(256) void bwd_gate_kernel(const void* __restrict__ dout, const void* __restrict__ y,
                                                       const int32_t* __restrict__ topk_expert, const float* __restrict__ topk_weight,
                                                       const int32_t* __restrict__ slot, int T, int T_pad, int H, int k, int E, int C,
                                                       int C_pad, int ld, float* __restrict__ dl, void* __restrict__ dL) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= T) {                                       // rows T .. T_pad - 1 of dL exist for the GEMM's sake: zeros
        if (t < T_pad)
            for (int c = lane; c < ld; c += 64) store_from_float<S>(dL, (size_t)t * ld + c, 0.0f);
        return;
    }
    const int row_chunks = H / S::kVec;
    int e_l = -1, s_l = -1;
    float w_l = 0.0f, dw_l = 0.0f;
    if (lane < k) {
        e_l = topk_expert[(size_t)t * k + lane];
        s_l = slot[(size_t)t * k + lane];
        w_l = topk_weight[(size_t)t * k + lane];
    }
    for (int j = 0; j < k; ++j) {
        const int e = __shfl(e_l, j), s = __shfl(s_l, j);
        if (s < 0 || s >= C || e < 0 || e >= E) continue;      // wave-uniform
        const size_t row = (size_t)e * C_pad + s;
        float part = 0.0f;
        for (int c = lane; c < row_chunks; c += 64) {   // 16 bytes of both rows per lane and step
            float dv[S::kVec], yv[S::kVec];
            chunk_to_floats<S>(load_once(dout, (size_t)t * row_chunks + c), dv);
            chunk_to_floats<S>(load_once(y, row * row_chunks + c), yv);
#pragma unroll
            for (int q = 0; q < S::kVec; ++q) part = fmaf(dv[q], yv[q], part);
        }
        const float d = wave_sum(part);
        if (lane == j) dw_l = d;
    }
    const float mean = wave_sum(w_l * dw_l);
    const float dl_l = w_l * (dw_l - mean);
    if (lane < k) dl[(size_t)t * k + lane] = dl_l;
    for (int c = lane; c < ld; c += 64) {
        float v = 0.0f;
        for (int j = 0; j < k; ++j) {
            const int e = __shfl(e_l, j);
            const float d = __shfl(dl_l, j);
            if (e == c) v = d;
        }
        store_from_float<S>(dL, (size_t)t * ld + c, v);
    }
}

// out[g][c][r] = in[g][r][c] for r < R, c < Cc; out rows have ld_out >= R entries, those at and beyond R are zero.
// 64 x 64 tiles through LDS; 16-bit elements move in pairs (4 bytes per lane on both sides: Cc and ld_out are even).
template <class elem>
__global__ __launch_bounds__(256) void bwd_transpose_kernel(const elem* __restrict__ in, elem* __restrict__ out, int R, int Cc,
                                                            int ld_out) {
    constexpr int TS = 64, PAIR = 4 / (int)sizeof(elem), PITCH = TS + 2;       // elements; rows stay 4-byte aligned
    __shared__ elem tile[TS][PITCH];
    const size_t g = blockIdx.z;
    const int r0 = blockIdx.x * TS, c0 = blockIdx.y * TS;
    constexpr int PER_ROW = TS / PAIR;                  // 4-byte words per tile row
    for (int idx = threadIdx.x; idx < TS * PER_ROW; idx += 256) {
        const int i = idx / PER_ROW, w = idx % PER_ROW;
        const int r = r0 + i, c = c0 + w * PAIR;
        uint32_t v = 0u;
        if (r < R && c < Cc) v = __builtin_nontemporal_load((const uint32_t*)(in + (g * R + r) * Cc + c));
        *(uint32_t*)&tile[i][w * PAIR] = v;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < TS * PER_ROW; idx += 256) {
        const int i = idx / PER_ROW, w = idx % PER_ROW;  // output row c0 + i, entries r0 + w * PAIR ..
        const int c = c0 + i, r = r0 + w * PAIR;
        if (c >= Cc || r >= ld_out) continue;
        uint32_t v;
        if constexpr (PAIR == 2) v = (uint32_t)tile[w * 2][i] | ((uint32_t)tile[w * 2 + 1][i] << 16);
        else v = __builtin_bit_cast(uint32_t, tile[w][i]);
        *(uint32_t*)(out + (g * Cc + c) * ld_out + r) = v;
    }
}

// out[e][c] = sum over the live rows r of in[e][r][c] (fp32).  A workgroup of four wavefronts owns 64 chunks of 16
// bytes of the columns of one expert; wavefront w adds the rows w, w + 4, ... in ascending order, four loads in flight
// per lane, and the four partial sums are added in wavefront order: a fixed order, the same from run to run.
template <class S>
__global__ __launch_bounds__(256) void bwd_colsum_kernel(const void* __restrict__ in, const int32_t* __restrict__ expert_demand, int C,
                                                         int C_pad, int cols, float* __restrict__ out) {
    constexpr int VEC = S::kVec;
    __shared__ float part[3][64][VEC];
    const int e = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row_chunks = cols / VEC, c = blockIdx.x * 64 + lane;
    const int n = min(expert_demand[e], C);
    float acc[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
    if (c < row_chunks) {
        const u32x4* p = (const u32x4*)in + (size_t)e * C_pad * row_chunks + c;
        auto add = [&](const u32x4& v) {
            if constexpr (S::kBytes == 4) {
#pragma unroll
                for (int q = 0; q < 4; ++q) { const uint32_t u = v[q]; acc[q] += __builtin_bit_cast(float, u); }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t u = v[q];
                    acc[2 * q] += bits16_to_float<S>((uint16_t)(u & 0xffffu));
                    acc[2 * q + 1] += bits16_to_float<S>((uint16_t)(u >> 16));
                }
            }
        };
        int r = wave;
        for (; r + 12 < n; r += 16) {
            u32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __builtin_nontemporal_load(p + (size_t)(r + 4 * i) * row_chunks);
#pragma unroll
            for (int i = 0; i < 4; ++i) add(v[i]);
        }
        for (; r < n; r += 4) add(__builtin_nontemporal_load(p + (size_t)r * row_chunks));
    }
    if (wave > 0) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) part[wave - 1][lane][q] = acc[q];
    }
    __syncthreads();
    if (wave == 0 && c < row_chunks) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] += part[w][lane][q];
#pragma unroll
        for (int q = 0; q < VEC; ++q) out[(size_t)e * cols + c * VEC + q] = acc[q];
    }
}

// dgate_bias[e] = sum of dl over the pairs that selected e: one workgroup per expert, fixed reduction tree.
__global__ __launch_bounds__(256) void bwd_gate_bias_kernel(const int32_t* __restrict__ topk_expert, const float* __restrict__ dl,
                                                            long long P, float* __restrict__ dgate_bias) {
    __shared__ float part[256];
    const int e = blockIdx.x;
    float acc = 0.0f;
    const long long P4 = P / 4;                         // four pairs per thread and step (both tables are 16-byte aligned)
    for (long long p = threadIdx.x; p < P4; p += 256) {
        const u32x4 ev = ((const u32x4*)topk_expert)[p];
        const f32x4 dv = ((const f32x4*)dl)[p];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if ((int)ev[q] == e) acc += dv[q];
    }
    for (long long p = P4 * 4 + threadIdx.x; p < P; p += 256)
        if (topk_expert[p] == e) acc += dl[p];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) dgate_bias[e] = part[0];
}

// One wavefront per token: dx_i = sum over kept choices of dxe[e_ij, slot_ij, :] (ascending j), then
// + sum over all k choices of dl_ij * Wg[:, e_ij] (rows of WgT), in fp32.  Lane j holds the routing entries of choice j
// (k <= 64); a lane owns 16-byte chunks lane, lane + 64, ... of the row.
template <class S>
__global__ __launch_bounds__(256) void bwd_dx_kernel(const void* __restrict__ dxe, const void* __restrict__ WgT,
                                                     const int32_t* __restrict__ topk_expert, const int32_t* __restrict__ slot,
                                                     const float* __restrict__ dl, int T, int H, int k, int E, int C, int C_pad,
                                                     float* __restrict__ dx) {
    constexpr int VEC = S::kVec;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= T) return;
    long long row_lane = -1;
    int e_lane = -1;
    float dl_lane = 0.0f;
    if (lane < k) {
        const int s = slot[(size_t)t * k + lane], e = topk_expert[(size_t)t * k + lane];
        if (e >= 0 && e < E) {
            e_lane = e;
            dl_lane = dl[(size_t)t * k + lane];
            if (s >= 0 && s < C) row_lane = (long long)e * C_pad + s;
        }
    }
    const int row_chunks = H / VEC;
    const u32x4* const dv = (const u32x4*)dxe;
    const u32x4* const wv = (const u32x4*)WgT;
    auto fma_chunk = [&](float (&acc)[VEC], float w, const u32x4& v) {
        if constexpr (S::kBytes == 4) {
#pragma unroll
            for (int q = 0; q < 4; ++q) { const uint32_t u = v[q]; acc[q] = fmaf(w, __builtin_bit_cast(float, u), acc[q]); }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t u = v[q];
                acc[2 * q] = fmaf(w, bits16_to_float<S>((uint16_t)(u & 0xffffu)), acc[2 * q]);
                acc[2 * q + 1] = fmaf(w, bits16_to_float<S>((uint16_t)(u >> 16)), acc[2 * q + 1]);
            }
        }
    };
    for (int c = lane; c < row_chunks; c += 64) {
        float acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
        for (int j = 0; j < k; ++j) {
            const long long row = __shfl(row_lane, j);
            if (row >= 0) fma_chunk(acc, 1.0f, __builtin_nontemporal_load(dv + (size_t)row * row_chunks + c));
        }
        for (int j = 0; j < k; ++j) {
            const int e = __shfl(e_lane, j);
            const float d = __shfl(dl_lane, j);
            if (e >= 0) fma_chunk(acc, d, wv[(size_t)e * row_chunks + c]);
        }
#pragma unroll
        for (int q = 0; q < VEC; q += 4)
            *(f32x4*)(dx + (size_t)t * H + (size_t)c * VEC + q) = f32x4{acc[q], acc[q + 1], acc[q + 2], acc[q + 3]};
    }
}

}  // namespace

__global__ __launch_bounds__(256) void bwd_fill_rows_kernel(int32_t* __restrict__ rows, int E, int first, int second) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < 2 * E) rows[i] = i < E ? first : second;
}

hipError_t launch_bwd_fill_rows(int32_t* rows, int E, int first, int second, hipStream_t s) {
    hipLaunchKernelGGL(bwd_fill_rows_kernel, dim3((2 * E + 255) / 256), dim3(256), 0, s, rows, E, first, second);
    return hipGetLastError();
}

hipError_t launch_bwd_gather(const void* x, const void* dout, const int32_t* slot_token, const float* slot_weight, int H, int E,
                             int C, int C_pad, int dtype, void* xe, void* gy, hipStream_t s) {
    const dim3 g((unsigned)((size_t)E * C_pad)), b(256);
    if (dtype == 0) hipLaunchKernelGGL(bwd_gather_kernel<F32>, g, b, 0, s, x, dout, slot_token, slot_weight, H, C, C_pad, xe, gy);
    else if (dtype == 1) hipLaunchKernelGGL(bwd_gather_kernel<BF16>, g, b, 0, s, x, dout, slot_token, slot_weight, H, C, C_pad, xe, gy);
    else hipLaunchKernelGGL(bwd_gather_kernel<F16>, g, b, 0, s, x, dout, slot_token, slot_weight, H, C, C_pad, xe, gy);
    return hipGetLastError();
}

hipError_t launch_bwd_act(const void* a, const void* g_in, const int32_t* expert_demand, int E, int C, int C_pad, int I, int act,
                          int dtype, bool grad, void* out, hipStream_t s) {
    const dim3 g((unsigned)((size_t)E * C_pad)), b(256);
#define MOE_BWD_ACT(S_, M_) hipLaunchKernelGGL((bwd_act_kernel<S_, M_>), g, b, 0, s, a, g_in, expert_demand, C, C_pad, I, act, out)
    if (dtype == 0) { if (grad) MOE_BWD_ACT(F32, 1); else MOE_BWD_ACT(F32, 0); }
    else if (dtype == 1) { if (grad) MOE_BWD_ACT(BF16, 1); else MOE_BWD_ACT(BF16, 0); }
    else { if (grad) MOE_BWD_ACT(F16, 1); else MOE_BWD_ACT(F16, 0); }
#undef MOE_BWD_ACT
    return hipGetLastError();
}

hipError_t launch_bwd_gate(const void* dout, const void* y, const int32_t* topk_expert, const float* topk_weight, const int32_t* slot,
                           int T, int T_pad, int H, int k, int E, int C, int C_pad, int ld, int dtype, float* dl, void* dL,
                           hipStream_t s) {
    const dim3 g((unsigned)((T_pad + 3) / 4)), b(256);
    if (dtype == 0) hipLaunchKernelGGL(bwd_gate_kernel<F32>, g, b, 0, s, dout, y, topk_expert, topk_weight, slot, T, T_pad, H, k, E, C, C_pad, ld, dl, dL);
    else if (dtype == 1) hipLaunchKernelGGL(bwd_gate_kernel<BF16>, g, b, 0, s, dout, y, topk_expert, topk_weight, slot, T, T_pad, H, k, E, C, C_pad, ld, dl, dL);
    else hipLaunchKernelGGL(bwd_gate_kernel<F16>, g, b, 0, s, dout, y, topk_expert, topk_weight, slot, T, T_pad, H, k, E, C, C_pad, ld, dl, dL);
    return hipGetLastError();
}

// out[i] = part[0][i] + part[1][i] + ... in that order, i < n (n a multiple of 4)
__global__ __launch_bounds__(256) void bwd_sum_slices_kernel(const f32x4* __restrict__ part, int slices, long long n4, f32x4* __restrict__ out) {
    const long long i = blockIdx.x * 256ll + threadIdx.x;
    if (i >= n4) return;
    f32x4 acc = part[i];
    for (int g = 1; g < slices; ++g) {
        const f32x4 v = part[(size_t)g * n4 + i];
        acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
    }
    out[i] = acc;
}

hipError_t launch_bwd_sum_slices(const float* part, int slices, long long n, float* out, hipStream_t s) {
    const long long n4 = n / 4;
    hipLaunchKernelGGL(bwd_sum_slices_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (const f32x4*)part, slices, n4, (f32x4*)out);
    return hipGetLastError();
}

hipError_t launch_bwd_transpose(const void* in, void* out, int groups, int R, int Cc, int ld_out, int dtype, hipStream_t s) {
    if (groups <= 0 || R <= 0 || Cc <= 0) return hipSuccess;
    if (groups > 65535 || (Cc + 63) / 64 > 65535 || (Cc & 1) || (ld_out & 1)) return hipErrorInvalidValue;
    const dim3 g((unsigned)((ld_out + 63) / 64), (unsigned)((Cc + 63) / 64), (unsigned)groups), b(256);
    if (dtype == 0) hipLaunchKernelGGL(bwd_transpose_kernel<float>, g, b, 0, s, (const float*)in, (float*)out, R, Cc, ld_out);
    else hipLaunchKernelGGL(bwd_transpose_kernel<uint16_t>, g, b, 0, s, (const uint16_t*)in, (uint16_t*)out, R, Cc, ld_out);
    return hipGetLastError();
}

hipError_t launch_bwd_colsum(const void* in, const int32_t* expert_demand, int E, int C, int C_pad, int cols, int dtype, float* out,
                             hipStream_t s) {
    if (E > 65535) return hipErrorInvalidValue;
    const int chunks = cols / (dtype == 0 ? 4 : 8);      // 16-byte chunks per row (cols is a multiple of 8)
    const dim3 g((unsigned)((chunks + 63) / 64), (unsigned)E), b(256);
    if (dtype == 0) hipLaunchKernelGGL(bwd_colsum_kernel<F32>, g, b, 0, s, in, expert_demand, C, C_pad, cols, out);
    else if (dtype == 1) hipLaunchKernelGGL(bwd_colsum_kernel<BF16>, g, b, 0, s, in, expert_demand, C, C_pad, cols, out);
    else hipLaunchKernelGGL(bwd_colsum_kernel<F16>, g, b, 0, s, in, expert_demand, C, C_pad, cols, out);
    return hipGetLastError();
}

hipError_t launch_bwd_gate_bias(const int32_t* topk_expert, const float* dl, int T, int k, int E, float* dgate_bias, hipStream_t s) {
    hipLaunchKernelGGL(bwd_gate_bias_kernel, dim3((unsigned)E), dim3(256), 0, s, topk_expert, dl, (long long)T * k, dgate_bias);
    return hipGetLastError();
}

hipError_t launch_bwd_dx(const void* dxe, const void* WgT, const int32_t* topk_expert, const int32_t* slot, const float* dl, int T, int H,
                         int k, int E, int C, int C_pad, int dtype, float* dx, hipStream_t s) {
    const dim3 g((unsigned)((T + 3) / 4)), b(256);
    if (dtype == 0) hipLaunchKernelGGL(bwd_dx_kernel<F32>, g, b, 0, s, dxe, WgT, topk_expert, slot, dl, T, H, k, E, C, C_pad, dx);
    else if (dtype == 1) hipLaunchKernelGGL(bwd_dx_kernel<BF16>, g, b, 0, s, dxe, WgT, topk_expert, slot, dl, T, H, k, E, C, C_pad, dx);
    else hipLaunchKernelGGL(bwd_dx_kernel<F16>, g, b, 0, s, dxe, WgT, topk_expert, slot, dl, T, H, k, E, C, C_pad, dx);
    return hipGetLastError();
}

}  // namespace moe
