// Device-side construction of the lists of live (group, row tile) units that the weight-streaming FFN
// kernels walk, shared by the stand-alone launcher and by the routing scatter launch (which appends it as
// one more workgroup so that the whole layer needs no separate launch for it).
#pragma once
#include "common.h"

namespace moe {

// Row tiles of the streaming FFN kernels.  A group's live rows are cut into large tiles; what remains beyond
// its full large tiles becomes one more large tile if it exceeds the small tile, else one small tile (half the
// matrix-core work and half the activation copies for the same weight bytes).  Each tile size has its own
// list and its own launch.
constexpr int kUnitRowsLarge = 256, kUnitRowsSmall = 128;

// Scratch block: two lists of the same format, the large tiles' first, then kXcds placement words.
//   list = { fault word (cleared), number of live units n, ids[cap] (n used), completion counters[cap] (cleared) }
//   large: cap = groups * nrow_large, id = g * nrow_large + (row tile of 256), nrow_large = ceil(max_rows / 256);
//          absent (0 ints) when max_rows <= 128
//   small: cap = groups, id = g * nrow_small + (row tile of 128), nrow_small = ceil(max_rows / 128)
// both in order of group.  Fault word bits: kFaultWaitGaveUp, kFaultPlacement (single-launch FFN only).
//   placement[x] = -1 (set by the builder); the single-launch FFN records there the hardware XCD that the
//   workgroups with blockIdx % kXcds == x run on, and flags a fault if two of them disagree.
constexpr int kXcds = 8;
constexpr int kFaultWaitGaveUp = 1, kFaultPlacement = 2;
__host__ __device__ inline int ffn_units_nrow_large(int max_rows) {
    return max_rows > kUnitRowsSmall ? (max_rows + kUnitRowsLarge - 1) / kUnitRowsLarge : 0;
}
__host__ __device__ inline int ffn_units_nrow_small(int max_rows) { return (max_rows + kUnitRowsSmall - 1) / kUnitRowsSmall; }
__host__ __device__ inline long long ffn_units_small_offset(int groups, int max_rows) {      // in ints
    const int nl = ffn_units_nrow_large(max_rows);
    return nl ? 2 + 2ll * groups * nl : 0;
}
__host__ __device__ inline long long ffn_units_placement_offset(int groups, int max_rows) {
    return ffn_units_small_offset(groups, max_rows) + 2 + 2ll * groups;
}
__host__ __device__ inline long long ffn_units_total_ints(int groups, int max_rows) {
    return ffn_units_placement_offset(groups, max_rows) + kXcds;
}

// The units of a list that XCD `xcd` works on: unit0, unit0 + unit_step, ... (ux of them).  Every 8th unit
// when an expert has at most one unit in the list (always so for the small tiles), else a contiguous block.
// `large`: the list of 256-row tiles.
__host__ __device__ inline void ffn_xcd_share(bool large, int n_units, int nrow, int xcd, int& unit0, int& unit_step, int& ux) {
    const bool blocks = large && nrow > 1;
    unit0 = blocks ? (int)((long long)n_units * xcd / kXcds) : xcd;
    unit_step = blocks ? 1 : kXcds;
    ux = blocks ? (int)((long long)n_units * (xcd + 1) / kXcds) - unit0
                : (n_units > xcd ? (n_units - xcd + kXcds - 1) / kXcds : 0);
}
// An XCD's tasks of one FFN GEMM over one list, in order: position p = (unit index inside the XCD) * ncol +
// column tile.  Workgroup w of the XCD's wgs takes positions w, w + wgs, ...  For the small list, w is the
// workgroup's number rotated so that the first small-tile task goes to the workgroup after the one that got
// the XCD's last large-tile task.
__host__ __device__ inline void ffn_task_at(int p, int ncol, int unit0, int unit_step, int& list_index, int& col_tile) {
    list_index = unit0 + (p / ncol) * unit_step;
    col_tile = p % ncol;
}
__host__ __device__ inline int ffn_small_list_rotation(int wg, int wgs, int ux_large, int ncol) {
    int w = wg - (int)(((long long)ux_large * ncol) % wgs);
    return w < 0 ? w + wgs : w;
}
// The small-tile tasks even out the large ones: the `handicap` workgroups that got one more large-tile task than the
// others (after the rotation they are the last ones, w >= wgs - handicap) sit out the first round of small-tile
// tasks, so a workgroup's third task, where there is one, is never on top of a large tile.  Workgroup w takes the
// slots w, w + wgs, ... from ffn_first_slot on; a slot's position in the XCD's task sequence is ffn_slot_position
// (the slots of the first round that are sat out do not count).  handicap = 0: position = slot (the large list).
__host__ __device__ inline int ffn_small_list_handicap(int wgs, int ux_large, int ncol) {
    return (int)(((long long)ux_large * ncol) % wgs);
}
__host__ __device__ inline int ffn_first_slot(int w, int wgs, int handicap) { return w < wgs - handicap ? w : w + wgs; }
__host__ __device__ inline int ffn_slot_position(int slot, int wgs, int handicap) { return slot < wgs ? slot : slot - handicap; }
// number of tasks of workgroup w among the XCD's xcd_tasks
__host__ __device__ inline int ffn_slot_count(int w, int wgs, int handicap, int xcd_tasks) {
    int n = 0, start = ffn_first_slot(w, wgs, handicap);
    if (start < wgs) {
        n = start < xcd_tasks ? 1 : 0;
        start += wgs;
    }
    const int left = xcd_tasks + handicap - start;
    return n + (left > 0 ? (left + wgs - 1) / wgs : 0);
}

// Called by every thread of ONE workgroup of `nthreads` threads (a multiple of 64, at most 1024);
// `wave_total` is an LDS array of 32 ints.
__device__ __forceinline__ void build_ffn_units(const int32_t* __restrict__ rows_dev, int rows_cap, int groups, int max_rows,
                                                int32_t* __restrict__ w, int* wave_total, int nthreads) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int nrow_l = ffn_units_nrow_large(max_rows), nrow_s = ffn_units_nrow_small(max_rows);
    int32_t* wl = w;                                    // large list (unused when nrow_l == 0)
    int32_t* ws = w + ffn_units_small_offset(groups, max_rows);
    const int cap_l = groups * nrow_l;
    for (int i = tid; i < cap_l; i += nthreads) wl[2 + cap_l + i] = 0;
    for (int i = tid; i < groups; i += nthreads) ws[2 + groups + i] = 0;
    if (tid < kXcds) w[ffn_units_placement_offset(groups, max_rows) + tid] = -1;
    int carry_l = 0, carry_s = 0;                       // units of the groups before this pass
    for (int g0 = 0; g0 < groups; g0 += nthreads) {
        const int g = g0 + tid;
        int nl = 0, ns = 0, full = 0;
        if (g < groups) {
            const int rows = min(min(rows_dev[g], rows_cap), max_rows);
            if (rows > 0) {
                if (nrow_l) {
                    full = rows / kUnitRowsLarge;
                    const int rem = rows - full * kUnitRowsLarge;
                    nl = full + (rem > kUnitRowsSmall ? 1 : 0);
                    ns = rem > 0 && rem <= kUnitRowsSmall ? 1 : 0;
                } else {
                    ns = 1;
                }
            }
        }
        int incl_l = nl, incl_s = ns;                   // inclusive scans inside the wavefront
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up_l = __shfl_up(incl_l, d), up_s = __shfl_up(incl_s, d);
            if (lane >= d) { incl_l += up_l; incl_s += up_s; }
        }
        if (lane == 63) { wave_total[wave] = incl_l; wave_total[16 + wave] = incl_s; }
        __syncthreads();
        int before_l = 0, total_l = 0, before_s = 0, total_s = 0;
        for (int wv = 0; wv < nwaves; ++wv) {
            const int tl = wave_total[wv], ts = wave_total[16 + wv];
            before_l += wv < wave ? tl : 0;
            total_l += tl;
            before_s += wv < wave ? ts : 0;
            total_s += ts;
        }
        const int start_l = carry_l + before_l + incl_l - nl;
        for (int rt = 0; rt < nl; ++rt) wl[2 + start_l + rt] = g * nrow_l + rt;
        if (ns) ws[2 + carry_s + before_s + incl_s - 1] = g * nrow_s + 2 * full;
        carry_l += total_l;
        carry_s += total_s;
        __syncthreads();
    }
    if (tid == 0) {
        if (nrow_l) { wl[0] = 0; wl[1] = carry_l; }
        ws[0] = 0; ws[1] = carry_s;
    }
}

// ---- fp32 storage: one list of live (group, 256-row tile) units for the kernel whose workgroups each take an equal
// share of the matrix-core work of all live tiles:
//   { n, ids[cap], cum[cap + 1] },  cap = groups * nrow,  id = g * nrow + row tile, in order of group;
//   cum[u] = sum of the weights of the units before u (cum[n] = their total).  A unit's weight is the time one of
//   its iterations takes, in twelfths of a full tile's: its b live 32-row MFMA tiles are dealt to the two wavefront
//   rows in turn, so the matrix cores need ceil(b / 2) / 4 of the full time; an iteration of a unit with one or two
//   live MFMA tiles is bound by its operand copies, which do not shrink with b (measured: 1.95 us against 8.6 us).
constexpr int kF32UnitRows = 256, kF32BlockRows = 32, kF32FullWeight = 12;
__host__ __device__ inline int f32_unit_weight(int live_blocks) {
    const int w = 3 * ((live_blocks + 1) / 2);
    return w > kF32FullWeight ? kF32FullWeight : w;
}
constexpr int kF32MaxWorkgroups = 256;                  // its grid is min(CUs, this); two partial tiles per workgroup
constexpr int kF32TileCols = 256, kF32TileK = 32;       // the kernel's column tile and K-tile
// units and total weight of a group with `rows` live rows
__host__ __device__ inline void f32_group_units(int rows, int& units, int& weight) {
    units = (rows + kF32UnitRows - 1) / kF32UnitRows;
    const int last_blocks = (rows + kF32BlockRows - 1) / kF32BlockRows - (units - 1) * (kF32UnitRows / kF32BlockRows);
    weight = units > 0 ? (units - 1) * kF32FullWeight + f32_unit_weight(last_blocks) : 0;
}
// The list as build_row_units writes it, computed on the host (ids[cap], cum[cap + 1]); returns the number of units.
inline int f32_build_units_host(const int32_t* rows_of, int rows_cap, int groups, int max_rows, int32_t* ids, int32_t* cum) {
    const int nrow = (max_rows + kF32UnitRows - 1) / kF32UnitRows;
    int n = 0, c = 0;
    for (int g = 0; g < groups; ++g) {
        int rows = rows_of[g] < rows_cap ? rows_of[g] : rows_cap;
        rows = rows < max_rows ? rows : max_rows;
        if (rows < 0) rows = 0;
        int nu, wt;
        f32_group_units(rows, nu, wt);
        for (int rt = 0; rt < nu; ++rt) {
            ids[n] = g * nrow + rt;
            cum[n++] = c + rt * kF32FullWeight;
        }
        c += wt;
    }
    cum[n] = c;
    return n;
}
__host__ __device__ inline int f32_units_nrow(int max_rows) { return (max_rows + kF32UnitRows - 1) / kF32UnitRows; }
__host__ __device__ inline long long f32_units_total_ints(int groups, int max_rows) {
    return 2 + 2ll * groups * f32_units_nrow(max_rows);
}

// The live work of one fp32 GEMM and how it is dealt.  Iterations are numbered L = unit * per_unit + column tile *
// nk + K-tile; an iteration of unit u costs cum[u + 1] - cum[u] (the unit's weight).  Workgroup w of G works on the
// iterations [boundary(w), boundary(w + 1)).
struct F32Work {
    const int32_t* ids; const int32_t* cum;
    int n_units, ncol, nk, per_unit;
    long long total_cost;
    __host__ __device__ inline F32Work(const int32_t* ids_, const int32_t* cum_, int n_units_, int ncol_, int nk_)
        : ids(ids_), cum(cum_), n_units(n_units_), ncol(ncol_), nk(nk_), per_unit(ncol_ * nk_),
          total_cost(n_units_ > 0 ? (long long)cum_[n_units_] * (ncol_ * nk_) : 0) {}
    // first iteration of workgroup w of G: where the running cost reaches total * w / G; w == G: the end
    __host__ __device__ inline long long boundary(int w, int G) const {
        if (n_units <= 0) return 0;
        if (w >= G) return (long long)n_units * per_unit;
        const long long c = total_cost / G * w + total_cost % G * w / G;
        int lo = 0, hi = n_units;                       // the unit u with cum[u] * per_unit <= c < cum[u + 1] * per_unit
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long long)cum[mid] * per_unit <= c) lo = mid; else hi = mid;
        }
        return (long long)lo * per_unit + (c - (long long)cum[lo] * per_unit) / (cum[lo + 1] - cum[lo]);
    }
    // The tile (unit * ncol + column tile) whose pieces workgroup w adds up in the second pass, or -1: the tile that
    // range w begins (its first K-tile lies in the range) but does not finish.  Every tile that is cut has exactly
    // one such workgroup; the pieces are those of w, w + 1, ... up to the range that holds the tile's last K-tile.
    __host__ __device__ inline long long tile_to_fix(long long begin, long long end) const {
        if (begin >= end) return -1;
        const long long tile = (end - 1) / nk, tb = tile * nk;
        return (tb + nk <= end || tb < begin) ? -1 : tile;
    }
};

// Called by every thread of ONE workgroup of `nthreads` threads (a multiple of 64, at most 1024);
// `wave_total` is an LDS array of at least 32 ints.
__device__ __forceinline__ void build_row_units(const int32_t* __restrict__ rows_dev, int rows_cap, int groups, int max_rows,
                                                int32_t* __restrict__ out, int* wave_total, int nthreads) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int nrow = f32_units_nrow(max_rows);
    int32_t* ids = out + 1;
    int32_t* cum = out + 1 + (long long)groups * nrow;
    int carry_u = 0, carry_b = 0;                       // units and their weights of the groups before this pass
    for (int g0 = 0; g0 < groups; g0 += nthreads) {
        const int g = g0 + tid;
        const int rows = g < groups ? max(min(min(rows_dev[g], rows_cap), max_rows), 0) : 0;
        int nu, nb;                                     // the group's units and weight
        f32_group_units(rows, nu, nb);
        int incl_u = nu, incl_b = nb;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up_u = __shfl_up(incl_u, d), up_b = __shfl_up(incl_b, d);
            if (lane >= d) { incl_u += up_u; incl_b += up_b; }
        }
        if (lane == 63) { wave_total[wave] = incl_u; wave_total[16 + wave] = incl_b; }
        __syncthreads();
        int before_u = 0, total_u = 0, before_b = 0, total_b = 0;
        for (int wv = 0; wv < nwaves; ++wv) {
            const int tu = wave_total[wv], tb = wave_total[16 + wv];
            before_u += wv < wave ? tu : 0;
            total_u += tu;
            before_b += wv < wave ? tb : 0;
            total_b += tb;
        }
        const int start_u = carry_u + before_u + incl_u - nu, start_b = carry_b + before_b + incl_b - nb;
        for (int rt = 0; rt < nu; ++rt) {
            ids[start_u + rt] = g * nrow + rt;
            cum[start_u + rt] = start_b + rt * kF32FullWeight;
        }
        carry_u += total_u;
        carry_b += total_b;
        __syncthreads();
    }
    if (tid == 0) {
        out[0] = carry_u;
        cum[carry_u] = carry_b;
    }
}

}  // namespace moe
