// Dispatch on one GPU (Alg. 1 "Dispatch"): builds the routing table
// T_phi(e, c) = (token, combine weight) with token-order slot assignment and
// drops beyond the capacity C, then packs the kept token rows into the per-expert
// buffer xe[E, C_pad, H] (the one-GPU residue of the symmetric layout's (C, H)
// cells, capacity aligned to the row tile as in Sec. 3.2.1).
//
// Slot assignment is integer work and fully deterministic: the (token, choice)
// pairs, in token-major order, are cut into chunks of 64 tokens (64 k pairs);
//   1. count:   one workgroup per chunk histograms its pairs by expert (LDS integer atomics).
//               The fused gate kernel, whose workgroups own the same 64 tokens, writes these
//               counts itself (the routing table as a by-product of the gate, Alg. 1), and the
//               launch is skipped;
//   2. scan:    one wavefront per expert turns the counts into exclusive chunk bases
//               and the expert's total demand; the launch also empties the routing table;
//   3. scatter: one wavefront per chunk walks its pairs 64 at a time; a lane's
//               slot is base + (pairs of the same expert in earlier steps) +
//               (lower lanes naming the same expert in this step).  One more workgroup of
//               this launch builds the FFN kernels' list of live (expert, row tile) units.
#include "route_body.h"

namespace moe {
namespace {

constexpr int kChunkTokens = 64;                        // tokens per chunk = tokens per fused-gate workgroup

// One workgroup per chunk: per-expert counts in an LDS histogram (integer atomics, so the result does not
// depend on their order).
__global__ __launch_bounds__(256) void route_count_kernel(const int32_t* __restrict__ topk_expert, long long P,
                                                          int chunk_pairs, int T, int k, bool choice_major, int E,
                                                          int32_t* __restrict__ counts) {
    extern __shared__ int32_t hist[];                // [E]
    for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
    __syncthreads();
    const long long p0 = (long long)blockIdx.x * chunk_pairs;
    const long long p1 = p0 + chunk_pairs < P ? p0 + chunk_pairs : P;
    for (long long p = p0 + threadIdx.x; p < p1; p += 256) {
        const int e = topk_expert[pair_index(p, T, k, choice_major)];
        if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) counts[(size_t)blockIdx.x * E + e] = hist[e];
}

// One wavefront per expert: exclusive scan of its per-chunk counts.  The launch also empties the routing table
// (slot_token = -1, slot_weight = 0).
__global__ __launch_bounds__(256) void route_scan_kernel(int32_t* __restrict__ counts, int n_chunks, int E,
                                                         int32_t* __restrict__ expert_demand,
                                                         int32_t* __restrict__ slot_token,
                                                         float* __restrict__ slot_weight, long long EC) {
    route_clear_tables(slot_token, slot_weight, EC, blockIdx.x * (long long)blockDim.x + threadIdx.x, (long long)gridDim.x * blockDim.x);
    const int e = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (e < E) route_scan_expert(counts, n_chunks, E, e, expert_demand);
}

// One wavefront (one workgroup of 64 threads) per chunk; one more workgroup builds the FFN kernels' unit lists.
__global__ __launch_bounds__(64) void route_scatter_kernel(const int32_t* __restrict__ topk_expert,
                                                           const float* __restrict__ topk_weight, long long P,
                                                           int chunk_pairs, int n_chunks, int T, bool choice_major,
                                                           int E, int k, int C, const int32_t* __restrict__ base,
                                                           int32_t* __restrict__ slot,
                                                           int32_t* __restrict__ slot_token,
                                                           float* __restrict__ slot_weight,
                                                           const int32_t* __restrict__ expert_demand,
                                                           int32_t* __restrict__ ffn_units, bool f32_units) {
    extern __shared__ int32_t run[];                 // [E] slots handed out so far, per expert
    __shared__ int wave_total[32];
    if ((int)blockIdx.x == n_chunks) {               // the extra workgroup: list of live FFN units
        if (f32_units) build_row_units(expert_demand, C, E, C, ffn_units, wave_total, 64);
        else build_ffn_units(expert_demand, C, E, C, ffn_units, wave_total, 64);
        return;
    }
    route_scatter_chunk(topk_expert, topk_weight, P, chunk_pairs, T, choice_major, E, k, C, base, slot, slot_token, slot_weight,
                        (int)blockIdx.x, run);
}

// One workgroup per token: the row is read once and written to each kept slot.
__global__ __launch_bounds__(256) void pack_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ topk_expert,
                                                   const int32_t* __restrict__ slot, int row_chunks, int k, int E,
                                                   int C, int C_pad, u32x4* __restrict__ xe) {
    const int t = blockIdx.x;
    for (int c = threadIdx.x; c < row_chunks; c += blockDim.x) {
        const u32x4 v = x[(size_t)t * row_chunks + c];
        for (int j = 0; j < k; ++j) {
            const int s = slot[(size_t)t * k + j];
            if (s < 0 || s >= C) continue;
            const int e = topk_expert[(size_t)t * k + j];
            if (e < 0 || e >= E) continue;
            xe[((size_t)e * C_pad + s) * row_chunks + c] = v;
        }
    }
}

}  // namespace

int route_chunk_tokens() { return kChunkTokens; }
int route_chunks(int T) { return (T + kChunkTokens - 1) / kChunkTokens; }

hipError_t launch_route(const int32_t* topk_expert, const float* topk_weight, int T, int E, int k, int C,
                        bool choice_major, int32_t* counts, bool counts_ready, int32_t* slot, int32_t* expert_demand,
                        int32_t* slot_token, float* slot_weight, int32_t* ffn_units, bool f32_units, hipStream_t stream) {
    const long long P = (long long)T * k;
    const int n_chunks = route_chunks(T);
    const int chunk_pairs = kChunkTokens * k;
    const long long EC = (long long)E * C;
    if (!counts_ready)
        hipLaunchKernelGGL(route_count_kernel, dim3(n_chunks), dim3(256), (size_t)E * sizeof(int32_t), stream,
                           topk_expert, P, chunk_pairs, T, k, choice_major, E, counts);
    hipLaunchKernelGGL(route_scan_kernel, dim3((E + 3) / 4), dim3(256), 0, stream, counts, n_chunks, E,
                       expert_demand, slot_token, slot_weight, EC);
    hipLaunchKernelGGL(route_scatter_kernel, dim3(n_chunks + (ffn_units ? 1 : 0)), dim3(64),
                       (size_t)E * sizeof(int32_t), stream, topk_expert, topk_weight, P, chunk_pairs, n_chunks, T,
                       choice_major, E, k, C, counts, slot, slot_token, slot_weight, expert_demand, ffn_units, f32_units);
    return hipGetLastError();
}

hipError_t launch_pack(const void* x, const int32_t* topk_expert, const int32_t* slot, int T, int H, int k,
                       int E, int C, int C_pad, int dtype, void* xe, hipStream_t stream) {
    const int bytes = dtype == 0 ? 4 : 2;
    const int row_chunks = H * bytes / 16;
    hipLaunchKernelGGL(pack_kernel, dim3(T), dim3(256), 0, stream, (const u32x4*)x, topk_expert, slot,
                       row_chunks, k, E, C, C_pad, (u32x4*)xe);
    return hipGetLastError();
}

}  // namespace moe
