// Wavefront-level pieces of the slot assignment (routing table T_phi with token-order slots and drops beyond
// the capacity; Alg. 1 "Dispatch"), shared by the routing kernels and by the kernel that runs the whole layer in
// one launch.  Integer work only: the result does not depend on scheduling.
#pragma once
#include "common.h"
#include "kernels.h"
#include "ffn_units.h"

namespace moe {
namespace {

// Position q in the order in which pairs claim slots -> index of the pair in the [T, k] tables.
// Token-major: the tables' own order.  Choice-major: q = j * T + token.
__device__ __forceinline__ long long pair_index(long long q, int T, int k, bool choice_major) {
    return choice_major ? (q % T) * k + q / T : q;
}

// slot_token = -1, slot_weight = 0 for all E C entries: thread gid of `stride` threads
__device__ __forceinline__ void route_clear_tables(int32_t* __restrict__ slot_token, float* __restrict__ slot_weight, long long EC,
                                                   long long gid, long long stride) {
    for (long long q = gid; q < EC; q += stride) {
        slot_token[q] = -1;
        slot_weight[q] = 0.0f;
    }
}

// One wavefront: exclusive scan of expert e's per-chunk counts (in place), 64 chunks at a time; its total demand.
__device__ __forceinline__ void route_scan_expert(int32_t* __restrict__ counts, int n_chunks, int E, int e,
                                                  int32_t* __restrict__ expert_demand) {
    const int lane = threadIdx.x % kWave;
    int carry = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += kWave) {
        const int c = c0 + lane;
        const int v = c < n_chunks ? counts[(size_t)c * E + e] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        if (c < n_chunks) counts[(size_t)c * E + e] = carry + incl - v;
        carry += __shfl(incl, kWave - 1);
    }
    if (lane == 0) expert_demand[e] = carry;
}

// this wavefront's LDS writes are complete and visible to its own later reads (also a compiler barrier)
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// One wavefront: the slots of chunk c's pairs, 64 pairs at a time.  `run` is an LDS array of E ints that belongs
// to this wavefront alone: slots handed out so far per expert, starting from the chunk's scanned bases.  A
// lane's slot is base + (pairs of the same expert in earlier steps) + (lower lanes naming the same expert in this
// step): lanes naming the same expert are found by intersecting ballots over the bits of the expert id.
__device__ __forceinline__ void route_scatter_chunk(const int32_t* __restrict__ topk_expert, const float* __restrict__ topk_weight,
                                                    long long P, int chunk_pairs, int T, bool choice_major, int E, int k, int C,
                                                    const int32_t* __restrict__ base, int32_t* __restrict__ slot,
                                                    int32_t* __restrict__ slot_token, float* __restrict__ slot_weight, int c,
                                                    int32_t* run) {
    const int lane = threadIdx.x % kWave;
    for (int e = lane; e < E; e += kWave) run[e] = base[(size_t)c * E + e];
    wave_lds_sync();
    const int nbits = E > 1 ? 32 - __clz(E - 1) : 0;
    const long long p_end = ((long long)c + 1) * chunk_pairs < P ? ((long long)c + 1) * chunk_pairs : P;
    for (long long p0 = (long long)c * chunk_pairs; p0 < p_end; p0 += kWave) {
        const long long p = p0 + lane;
        const long long m = p < p_end ? pair_index(p, T, k, choice_major) : 0;   // index in the [T, k] tables
        int e = p < p_end ? topk_expert[m] : -1;
        const bool valid = (e >= 0 && e < E);
        if (!valid) e = 0;
        unsigned long long same = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long bal = __ballot(valid && bit);
            same &= bit ? bal : ~bal;
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        const int rank = __popcll(same & below);
        const int group = __popcll(same);
        const int s = valid ? run[e] + rank : 0;
        wave_lds_sync();
        if (valid && rank == group - 1) run[e] = s + 1;
        wave_lds_sync();
        if (p < p_end) {
            const bool kept = valid && s < C;
            slot[m] = kept ? s : -1;
            if (kept) {
                slot_token[(size_t)e * C + s] = (int32_t)(m / k);
                slot_weight[(size_t)e * C + s] = topk_weight[m];
            }
        }
    }
}

}  // namespace
}  // namespace moe
