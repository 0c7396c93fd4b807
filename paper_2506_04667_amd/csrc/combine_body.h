// Combine (task t3 of Sec. 3.1, C <- A (.) S + C; Eq. "combine 2"), built as a
// deterministic gather-reduce: every token's kept expert output rows, scaled by the
// combine weights, are summed in ascending choice order in fp32.
//
// One wavefront per token at a time, persistent: a wavefront walks tokens
// w, w + W, ... and reads the routing entries of its next token while the rows of the
// current one are in flight, so that the dependent chain "routing entry -> row address
// -> row" is paid once per wavefront and not once per token.  A lane owns 16-byte
// chunks lane, lane + 64, ... of the row, four at a time, so a token of 4 KB with two
// kept choices has eight 16-byte loads per lane in flight.  The expert rows are read
// once and the output written once: both bypass the caches' retention (non-temporal).
#pragma once
#include "common.h"
#include "kernels.h"

namespace moe {
namespace {

constexpr int kCombineThreads = 256;                    // four wavefronts per workgroup
constexpr int kChunksPerPass = 4;                       // 16-byte chunks per lane in flight per choice
constexpr int kChoicesPerPass = 2;

// The tokens wave, wave + waves, ... by one wavefront (`wave` is its number among the `waves` that share the work).
template <class S>
__device__ __forceinline__ void combine_tokens(const void* __restrict__ y, const int32_t* __restrict__ topk_expert,
                                               const float* __restrict__ topk_weight, const int32_t* __restrict__ slot, int T,
                                               int H, int k, int E, int C, int C_pad, void* __restrict__ out, int wave, int waves) {
    constexpr int VEC = S::kVec;
    const int lane = threadIdx.x & 63;
    const int row_chunks = H / VEC;
    const u32x4* const yv = (const u32x4*)y;
    u32x4* const ov = (u32x4*)out;

    // routing entries of choice j0 + lane of a token (lanes beyond the choices hold "dropped")
    auto entry = [&](int t, int j0, float& w, long long& row) {
        const int j = j0 + lane;
        w = 0.0f;
        row = -1;
        if (t < T && j < k) {
            const int s = slot[(size_t)t * k + j], e = topk_expert[(size_t)t * k + j];
            w = topk_weight[(size_t)t * k + j];
            if (s >= 0 && s < C && e >= 0 && e < E) row = (long long)e * C_pad + s;
        }
    };
    float w_next;
    long long row_next;
    entry(wave, 0, w_next, row_next);
    for (int t = wave; t < T; t += waves) {
        float w_lane = w_next;                          // entries of choices 0 .. 63, one per lane
        long long row_lane = row_next;
        entry(t + waves, 0, w_next, row_next);          // the next token's, in flight during this one
        for (int c0 = 0; c0 < row_chunks; c0 += 64 * kChunksPerPass) {
            float acc[kChunksPerPass][VEC];
#pragma unroll
            for (int i = 0; i < kChunksPerPass; ++i)
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[i][q] = 0.0f;
            for (int j0 = 0; j0 < k; j0 += kChoicesPerPass) {
                if (j0 > 0 && (j0 & 63) == 0) entry(t, j0, w_lane, row_lane);       // more than 64 choices: fetch the next 64
                float w[kChoicesPerPass];
                long long row[kChoicesPerPass];
#pragma unroll
                for (int q = 0; q < kChoicesPerPass; ++q) {
                    w[q] = __shfl(w_lane, (j0 + q) & 63);
                    row[q] = __shfl(row_lane, (j0 + q) & 63);
                    if (j0 + q >= k) row[q] = -1;
                }
                // all row chunks of these choices in flight together, then the sums in ascending choice order
                u32x4 v[kChoicesPerPass][kChunksPerPass];
#pragma unroll
                for (int q = 0; q < kChoicesPerPass; ++q)
#pragma unroll
                    for (int i = 0; i < kChunksPerPass; ++i) {
                        const int c = c0 + i * 64 + lane;
                        if (row[q] >= 0 && c < row_chunks) v[q][i] = __builtin_nontemporal_load(yv + (size_t)row[q] * row_chunks + c);
                    }
#pragma unroll
                for (int q = 0; q < kChoicesPerPass; ++q) {
                    if (row[q] < 0) continue;
#pragma unroll
                    for (int i = 0; i < kChunksPerPass; ++i) {
                        if (c0 + i * 64 + lane >= row_chunks) continue;
                        if constexpr (S::kBytes == 4) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const uint32_t u = v[q][i][e];   // copy out first: bit_cast of a vector element reads lane 0
                                acc[i][e] = fmaf(w[q], __builtin_bit_cast(float, u), acc[i][e]);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const uint32_t u = v[q][i][e];
                                acc[i][2 * e] = fmaf(w[q], bits16_to_float<S>((uint16_t)(u & 0xffffu)), acc[i][2 * e]);
                                acc[i][2 * e + 1] = fmaf(w[q], bits16_to_float<S>((uint16_t)(u >> 16)), acc[i][2 * e + 1]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kChunksPerPass; ++i) {
                const int c = c0 + i * 64 + lane;
                if (c >= row_chunks) continue;
                u32x4 o;
                if constexpr (S::kBytes == 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = __builtin_bit_cast(uint32_t, acc[i][e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = (uint32_t)float_to_bits16<S>(acc[i][2 * e]) | ((uint32_t)float_to_bits16<S>(acc[i][2 * e + 1]) << 16);
                }
                __builtin_nontemporal_store(o, ov + (size_t)t * row_chunks + c);
            }
        }
    }
}

}  // namespace
}  // namespace moe
