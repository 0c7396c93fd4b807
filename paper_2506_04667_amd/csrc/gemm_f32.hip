// Expert FFN tasks in fp32 storage (Sec. 3.1 task abstraction; Eq. ffn): a persistent kernel over the live work only.
//
// fp32 MFMAs are sixteen times slower per element than 16-bit ones, so with a 256 x 256 tile these GEMMs are bound by
// the matrix cores, and what a launch of whole tiles loses is balance: a layer with few experts has about as many
// tiles as the chip has CUs (or far fewer), an expert's last row tile may hold a handful of live rows, and tiles
// beyond an expert's live rows are launched only to exit.  Here the work is cut the other way round.  The live
// (expert, 256-row tile) units come from a list built on the device once routing is known, each with its weight:
// the time of one of its iterations, from its live 32-row MFMA tiles (the tile body leaves out the MFMAs of the others).  unit x column tile (256 wide) x
// K-tile (32 deep) is one iteration, numbered unit by unit, K innermost; workgroup w of G (one per CU) starts at
// the iteration where the running weight reaches w / G of the total: about equal matrix-core work for every
// workgroup whatever the routing.  A workgroup's range covers the end of one tile, some whole tiles and the
// beginning of another.  Whole tiles get their epilogue at once; the sums of a partly covered tile go to one of the
// workgroup's two fp32 tiles in the caller's workspace, and a second small launch adds the pieces of each cut tile
// in the order of the workgroups that made them (a fixed order: results are the same run to run) and applies bias
// and activation.  No workgroup ever waits for another.
#include "ffn_units.h"
#include "gemm_body.h"

namespace moe {
namespace {

// 256 x 256 tile: 8 wavefronts (2 x 4), each 128 x 64 (4 x 2 MFMA tiles of 32 x 32); one workgroup per CU
constexpr int F_WM = 2, F_WN = 4, F_TM = 4, F_TN = 2;
using FCfg = Cfg<F32, false, F_WM, F_WN, F_TM, F_TN>;
constexpr int F_BM = FCfg::BM, F_BN = FCfg::BN, F_BK = FCfg::BK, F_THREADS = FCfg::THREADS;
constexpr int F_LDS = 2 * FCfg::STAGE_BYTES;

// upper bound of the workgroups worth launching: the iterations at full capacity, at most kF32MaxWorkgroups
long long f32_workgroups_bound(int groups, int max_rows, int N, int K) {
    const long long t = (long long)groups * f32_units_nrow(max_rows) * ((N + F_BN - 1) / F_BN) * ((K + F_BK - 1) / F_BK);
    return t < kF32MaxWorkgroups ? (t > 0 ? t : 1) : kF32MaxWorkgroups;
}
static_assert(F_BM == kF32UnitRows && F_BN == kF32TileCols && F_BK == kF32TileK, "the unit list and the dealing are cut in the tile's sizes");
constexpr int kFixupSplit = 4;                          // workgroups that share the fix-up of one cut tile, by rows
static_assert(F_BN % 4 == 0 && F_BM * F_BN / 4 % (F_THREADS * kFixupSplit) == 0, "fix-up thread mapping");

struct F32StreamArgs {
    GemmArgs g;
    const int32_t* list;                                // { n_units, ids[cap], cum[cap + 1] }, cap = groups * nrow
    float* partials;                                    // [G][2][F_BM][F_BN]
    int nrow;                                           // row tiles per group the ids are numbered with
};

__device__ __forceinline__ F32Work work_of(const F32StreamArgs& a) {
    const int32_t* ids = a.list + 1;
    return F32Work(ids, ids + (long long)a.g.groups * a.nrow, a.list[0], (a.g.N + F_BN - 1) / F_BN, (a.g.K + F_BK - 1) / F_BK);
}

// One piece of a tile.  Not inlined: inside the loop over a workgroup's pieces the compiler would keep the tile
// body's per-thread addresses alive across iterations and run out of registers.  The LDS array is named here, not
// passed in, so that the body's accesses stay LDS instructions.
__device__ __noinline__ void f32_tile_piece(const GemmArgs& g, int grp, int row0, int n0, int rows, int kt0, int kt1, float* partial) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    gemm_tile<F32, false, F_WM, F_WN, F_TM, F_TN>(g, smem, grp, row0, n0, rows, kt0, kt1, partial);
}

#ifdef MOE_F32_STREAM_CLOCKS
}  // namespace
}  // namespace moe
static __device__ long long f32_dbg[256 * 4];
extern "C" int moe_debug_f32_clocks(long long* host) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(f32_dbg), sizeof(long long) * 256 * 4);
}
namespace moe {
namespace {
#endif

__global__ __launch_bounds__(F_THREADS) void ffn_f32_stream_kernel(F32StreamArgs a) {
#ifdef MOE_F32_STREAM_CLOCKS
    const long long t_start = wall_clock64();
    int n_pieces = 0, n_light = 0;
#endif
    const int w = blockIdx.x, G = gridDim.x;
    const F32Work k = work_of(a);
    const long long begin = k.boundary(w, G), end = k.boundary(w + 1, G);
    bool first = true;
    for (long long it = begin; it < end;) {
        const long long tile = it / k.nk;
        const int kt0 = (int)(it - tile * k.nk);
        const int kt1 = (int)min((long long)k.nk, kt0 + (end - it));
        const int id = k.ids[tile / k.ncol], ct = (int)(tile % k.ncol);
        const int grp = id / a.nrow, rt = id % a.nrow;
        const int rows = min(a.g.rows_dev[grp], a.g.rows_cap);
        const bool whole = kt0 == 0 && kt1 == k.nk;
        float* partial = whole ? nullptr : a.partials + ((size_t)w * 2 + (first ? 0 : 1)) * (F_BM * F_BN);
        f32_tile_piece(a.g, grp, rt * F_BM, ct * F_BN, rows, kt0, kt1, partial);
#ifdef MOE_F32_STREAM_CLOCKS
        ++n_pieces;
        if (rows - rt * F_BM <= 128) n_light += kt1 - kt0;
#endif
        it += kt1 - kt0;
        first = false;
    }
#ifdef MOE_F32_STREAM_CLOCKS
    if (threadIdx.x == 0 && w < 256) {
        f32_dbg[w * 4 + 0] = wall_clock64() - t_start;
        f32_dbg[w * 4 + 1] = end - begin;
        f32_dbg[w * 4 + 2] = n_pieces;
        f32_dbg[w * 4 + 3] = n_light;
    }
#endif
}

// Workgroups (w, 0 .. kFixupSplit - 1) add up the tile that range w begins but does not finish: its own piece, then those of the
// workgroups after it, in order, until the tile's last K-tile; then bias, activation and the store.
__global__ __launch_bounds__(F_THREADS) void ffn_f32_fixup_kernel(F32StreamArgs a, int G) {
    const int w = blockIdx.x;
    const F32Work k = work_of(a);
    const long long begin = k.boundary(w, G), end = k.boundary(w + 1, G);
    const long long tile = k.tile_to_fix(begin, end);
    if (tile < 0) return;                               // nothing cut here, or the cut tile was begun by an earlier workgroup
    const long long tb = tile * k.nk, te = tb + k.nk;
    const int id = k.ids[tile / k.ncol], ct = (int)(tile % k.ncol);
    const int grp = id / a.nrow, rt = id % a.nrow;
    const int rows = min(a.g.rows_dev[grp], a.g.rows_cap);
    const int row0 = rt * F_BM, n0 = ct * F_BN;
    constexpr int V = F_BM * F_BN / 4 / F_THREADS / kFixupSplit;    // float4s per thread
    const int part = blockIdx.y * V * F_THREADS;        // this workgroup's share of the tile: F_BM / kFixupSplit rows
    f32x4 sum[V];
    {
        const f32x4* p = (const f32x4*)(a.partials + ((size_t)w * 2 + (begin == tb ? 0 : 1)) * (F_BM * F_BN));
#pragma unroll
        for (int i = 0; i < V; ++i) sum[i] = p[part + i * F_THREADS + threadIdx.x];
    }
    long long vb = end;                                 // workgroup v's range is [vb, ve)
    for (int v = w + 1; v < G && vb < te; ++v) {
        const long long ve = k.boundary(v + 1, G);
        if (ve > vb) {
            const f32x4* p = (const f32x4*)(a.partials + (size_t)v * 2 * (F_BM * F_BN));   // the tile is v's first piece
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const f32x4 t = p[part + i * F_THREADS + threadIdx.x];
                sum[i][0] += t[0]; sum[i][1] += t[1]; sum[i][2] += t[2]; sum[i][3] += t[3];
            }
        }
        vb = ve;
    }
    const size_t c_base = (size_t)grp * a.g.c_group_stride;
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int idx = part + i * F_THREADS + threadIdx.x;
        const int row = row0 + idx / (F_BN / 4), col = n0 + (idx % (F_BN / 4)) * 4;
        if (row >= rows || col >= a.g.N) continue;      // N is a multiple of 4
        f32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float bias = a.g.bias ? ((const float*)a.g.bias)[(size_t)grp * a.g.bias_group_stride + col + j] : 0.0f;
            o[j] = apply_act(sum[i][j] + bias, a.g.act);
        }
        *(f32x4*)((float*)a.g.C + c_base + (size_t)row * a.g.ldc + col) = o;
    }
}

__global__ __launch_bounds__(1024) void f32_units_kernel(const int32_t* __restrict__ rows_dev, int rows_cap, int groups, int max_rows,
                                                         int32_t* __restrict__ out) {
    __shared__ int wave_total[32];
    build_row_units(rows_dev, rows_cap, groups, max_rows, out, wave_total, 1024);
}

// one workgroup per CU, but never more than the iterations there can be (a workgroup with no work still costs two
// partial tiles of workspace)
int f32_grid(int groups, int max_rows, int N, int K) {
    const long long bound = f32_workgroups_bound(groups, max_rows, N, K);
    const long long g = device_cu_count();
    return (int)(g < bound ? g : bound);
}

}  // namespace

size_t f32_units_ints(int groups, int max_rows) { return (size_t)f32_units_total_ints(groups, max_rows); }
size_t f32_partials_bytes(int groups, int max_rows, int H, int I) {
    const long long g1 = f32_workgroups_bound(groups, max_rows, I, H), g2 = f32_workgroups_bound(groups, max_rows, H, I);
    return (size_t)(g1 > g2 ? g1 : g2) * 2 * F_BM * F_BN * sizeof(float);
}

hipError_t launch_f32_units(const int32_t* rows_dev, int rows_cap, int groups, int max_rows, int32_t* units, hipStream_t stream) {
    hipLaunchKernelGGL(f32_units_kernel, dim3(1), dim3(1024), 0, stream, rows_dev, rows_cap, groups, max_rows, units);
    return hipGetLastError();
}

hipError_t prepare_gemm_f32() {
    static DeviceFlags limit_raised = {};
    return raise_lds_limit(reinterpret_cast<const void*>(ffn_f32_stream_kernel), F_LDS, limit_raised);
}

// Worth it when whole tiles would not fill the chip evenly: fewer than four rounds of 256 x 256 tiles over the CUs at
// full capacity (with more, the plain launch of whole tiles is as fast: its rounding loss is small and it needs no
// second pass), but enough work that the second launch does not show (eight iterations per CU).
bool f32_stream_eligible(const GemmArgs& a) {
    if (a.dtype != 0 || a.b_is_nk || a.c_f32 || !a.units || !a.partials || !a.rows_dev) return false;
    if (a.N % 4 != 0 || a.K % 4 != 0 || a.ldc % 4 != 0) return false;
    const long long units = (long long)a.groups * f32_units_nrow(a.max_rows), ncol = (a.N + F_BN - 1) / F_BN;
    if (units > 0x7fffffffLL / ncol) return false;
    const long long tiles = units * ncol, cus = device_cu_count();
    return tiles < 4 * cus && tiles * ((a.K + F_BK - 1) / F_BK) >= 8 * cus;
}

hipError_t launch_gemm_f32_stream(const GemmArgs& g, hipStream_t stream) {
    if (hipError_t e = prepare_gemm_f32(); e != hipSuccess) return e;
    F32StreamArgs a{};
    a.g = g;
    a.list = g.units;
    a.partials = g.partials;
    a.nrow = f32_units_nrow(g.max_rows);
    const int G = f32_grid(g.groups, g.max_rows, g.N, g.K);
    hipLaunchKernelGGL(ffn_f32_stream_kernel, dim3(G), dim3(F_THREADS), F_LDS, stream, a);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    hipLaunchKernelGGL(ffn_f32_fixup_kernel, dim3(G, kFixupSplit), dim3(F_THREADS), 0, stream, a, G);
    return hipGetLastError();
}

}  // namespace moe
