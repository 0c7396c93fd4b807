// Device-side construction of the list of live (group, row tile) units that the weight-streaming FFN
// kernels walk, shared by the stand-alone launcher and by the routing scatter launch (which appends it as
// one more workgroup so that the whole layer needs no separate launch for it).
#pragma once
#include "common.h"

namespace moe {

// Row tiles of the streaming FFN kernels.  A launch uses one of them for all its units: the large one, unless
// no group can have more rows than the small one (then half the matrix-core work per weight byte goes away).
constexpr int kUnitRowsLarge = 256, kUnitRowsSmall = 128;

// Scratch block `w` of ffn_units_ints() ints: w[0] = fault word (cleared), w[1] = number of live units,
// w[2 + q] = g * nrow + row tile in group order (row tiles of `unit_rows` rows, nrow of them cover the
// capacity), then one completion counter per possible unit (cleared).
// Called by every thread of ONE workgroup of `nthreads` threads (a multiple of 64, at most 1024);
// `wave_total` is an LDS array of 16 ints.
__device__ __forceinline__ void build_ffn_units(const int32_t* __restrict__ rows_dev, int rows_cap, int groups, int unit_rows,
                                                int nrow, int32_t* __restrict__ w, int* wave_total, int nthreads) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int cap = groups * nrow;
    int32_t* units = w + 2;
    int32_t* done = w + 2 + cap;
    for (int i = tid; i < cap; i += nthreads) done[i] = 0;
    int carry = 0;                                      // units of the groups before this pass
    for (int g0 = 0; g0 < groups; g0 += nthreads) {
        const int g = g0 + tid;
        int nt = 0;
        if (g < groups) {
            const int rows = min(rows_dev[g], rows_cap);
            nt = rows > 0 ? (rows + unit_rows - 1) / unit_rows : 0;
        }
        int incl = nt;                                  // inclusive scan inside the wavefront
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
        for (int wv = 0; wv < nwaves; ++wv) {
            const int t = wave_total[wv];
            before += wv < wave ? t : 0;
            total += t;
        }
        const int start = carry + before + incl - nt;
        for (int rt = 0; rt < nt; ++rt) units[start + rt] = g * nrow + rt;
        carry += total;
        __syncthreads();
    }
    if (tid == 0) { w[0] = 0; w[1] = carry; }
}

}  // namespace moe
