// Direct global -> LDS copies on gfx950 (global_load_lds_dwordx4) and the explicit waits that go
// with them.  The copies are issued from inline asm: a compiler-visible LDS-DMA would make every
// later LDS read wait for all outstanding copies, which defeats prefetching.
#pragma once
#include "common.h"

namespace moe {

// Tell the compiler that a value is the same in every lane (it then lives in scalar registers).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const unsigned char* uniform(const unsigned char* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const unsigned char*)(((uint64_t)hi << 32) | lo);
}

// 64 lanes x 16 bytes from global addresses base + per-lane byte offset to LDS [lds_addr, lds_addr + 1024):
// lane i lands at lds_addr + 16 i.  A wave-uniform base in scalar registers plus 32-bit lane offsets keeps
// the copy cursors out of the vector registers.
__device__ __forceinline__ void copy_to_lds(const unsigned char* base, uint32_t lane_off, uint32_t lds_addr) {
    base = uniform(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}

// The same copy for data that is read once (weights streaming past): the non-temporal hint asks the caches to
// give such lines up first, so that they do not push out lines that other workgroups are about to re-read.
__device__ __forceinline__ void copy_to_lds_stream(const unsigned char* base, uint32_t lane_off, uint32_t lds_addr) {
    base = uniform(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}

// own copies older than the newest N have landed; own LDS reads are complete; then meet the other waves
template <int N>
__device__ __forceinline__ void wait_copies_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

}  // namespace moe
