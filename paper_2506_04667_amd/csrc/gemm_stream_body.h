// Weight-streaming grouped GEMM for the expert FFN tasks in 16-bit storage
// (C1 <- phi1(A B1 + D1), C2 <- C1 B2 + D2; Sec. 3.1).  At the paper's expert-scaling
// shape an expert has only ~256 live rows, so each weight matrix is used by one row
// tile and the kernel is bound by streaming weights from HBM once, not by the
// matrix cores.  The design keeps the copy engine busy without a break:
//
//   * persistent workgroups, one per CU (the paper's processors, Sec. 3, without a
//     scheduler: once routing is known the live tasks are a fixed list, compacted on
//     the device so that empty experts cost nothing and every XCD gets an equal
//     share whatever the routing skew).  A workgroup walks its (expert, row tile,
//     column tile) tasks and treats all their K-tiles as one stream, so the copies
//     of the next task are in flight while the current one finishes and while its
//     epilogue runs -- no drain between tasks;
//   * tile 256 x 256 (8 wavefronts as 2 x 4, 128 rows x 64 columns each, MFMA
//     16x16x32): an expert with <= 256 live rows reads its weights exactly once; a
//     128 x 256 variant of the same loop takes remainders of at most 128 rows;
//   * K-tile 32.  Weights (from HBM) go through a ring of 4 LDS stages of 16 KB
//     (32 x 256), requested 3 K-tiles ahead; activations (re-read from L2 by the 8
//     column tiles of an expert) go through 2 stages of 32 KB that hold two K-tiles
//     each (256 rows x 128 B), so every L2 request is a full 128-byte line;
//   * global -> LDS copies are direct (global_load_lds_dwordx4: no VGPR staging),
//     issued from inline asm and waited for with explicit s_waitcnt vmcnt(n) +
//     s_barrier: a compiler-visible LDS-DMA makes every later LDS read wait for all
//     outstanding copies;
//   * MFMA operand fragments are double-buffered in registers at half-K-tile
//     granularity: while 16 MFMAs run, the LDS reads of the next 16 are in flight,
//     across K-tile and task boundaries too.
//
// A direct copy writes 64 lanes x 16 B to 1024 contiguous LDS bytes (lane i at
// base + 16 i), while each lane picks its own global address; the XOR swizzles below
// are therefore applied on the global side (which 16-byte chunk a lane fetches).
//   A stage: row pitch 128 B; chunk c of row r lives at c ^ ((r >> 1) & 7).
//   B stage: [k][n], row pitch 512 B; chunk c of row k lives at
//            c ^ (((k & 3) << 1) | (((k >> 3) & 1) << 3)); read back in MFMA operand
//            order with ds_read_b64_tr_b16 (the four 16-lane groups of a wavefront
//            read the four k-octets of a K-tile).
// Rows at or beyond the live row count are fetched from the last live row (their
// products land in output rows that are never stored); columns beyond N likewise.
// Because every lane supplies its own global address, the activation rows can be
// gathered straight from the token matrix through the routing table (slot -> token):
// the payload-efficient dispatch of Sec. 3.2.1 without a packed copy.
//
// The MFMAs take the weight fragment as their first operand, so a lane's
// accumulators hold, for ONE token row, runs of four consecutive output columns.
// The epilogue applies bias and activation in registers, packs each run to 8 bytes,
// transposes 32 rows at a time through a wave-private LDS area and stores full
// 128-byte row segments.
//
// Requires K % 64 == 0, K >= 192 and N % 8 == 0; other shapes use the generic kernel.
#pragma once
#include "common.h"
#include "kernels.h"
#include "lds_copy.h"
#include "ffn_units.h"

#include <type_traits>

namespace moe {
namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Layout-study switches: the library is built with all three swizzles on.  Building with one of them set to 0
// (python -m paper_2506_04667_amd.build --define MOE_STREAM_SWIZZLE_A=0 --out <file>) stores that operand in
// LDS unswizzled, which changes nothing but the bank-conflict behaviour: the 16-bit LDS layouts are the part the
// paper's own "FP16 memory throughput" appendix names as its weak spot.
#ifndef MOE_STREAM_SWIZZLE_A
#define MOE_STREAM_SWIZZLE_A 1
#endif
#ifndef MOE_STREAM_SWIZZLE_B
#define MOE_STREAM_SWIZZLE_B 1
#endif
#ifndef MOE_STREAM_SWIZZLE_EPILOGUE
#define MOE_STREAM_SWIZZLE_EPILOGUE 1
#endif
__device__ __forceinline__ int swz_a(int r) { return MOE_STREAM_SWIZZLE_A ? (r >> 1) & 7 : 0; }
__device__ __forceinline__ int swz_b(int k) { return MOE_STREAM_SWIZZLE_B ? ((k & 3) << 1) | (((k >> 3) & 1) << 3) : 0; }
__device__ __forceinline__ int swz_e(int r) { return MOE_STREAM_SWIZZLE_EPILOGUE ? (r >> 1) & 7 : 0; }

constexpr int BN = 256, BK = 32, THREADS = 512;
constexpr int TN = 4, WN = 4;                           // 16-column MFMA tiles per wavefront; wavefronts along N
// Row tile: 128 G rows, G = 2 (the design above) or G = 1 (wavefronts hold 64 x 64: half the MFMAs and half
// the activation copies per weight byte).  An expert's rows are cut into 256-row tiles; a remainder of at
// most 128 rows becomes a 128-row tile.  Each size has its own unit list; one launch walks both (see the
// kernel), so experts with few rows (skewed routing, small capacities, few tokens) do not pay for a
// half-empty large tile.
constexpr int A_STAGE = kUnitRowsLarge * 128;           // up to 256 rows x 64 k (two K-tiles)
constexpr int A_STAGES = 2;
constexpr int B_STAGE = BK * BN * 2;                    // 32 k x 256 columns
constexpr int B_STAGES = 4;
constexpr int B_ROW_BYTES = BN * 2;
constexpr int B_REGION = A_STAGES * A_STAGE;            // weights ring starts after the activation stages
constexpr int EPI_REGION = B_REGION + B_STAGES * B_STAGE;
constexpr int EPI_BYTES_PER_WAVE = 32 * 128;            // 32 rows x 64 columns x 2 B
constexpr int LDS_BYTES = EPI_REGION + 8 * EPI_BYTES_PER_WAVE;
static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");

// v_mfma_f32_16x16x32: a lane holds, of each operand, 8 consecutive k (k = 8 (lane / 16) ..) of row/column
// lane % 16, and of the result rows 4 (lane / 16) .. + 3 of column lane % 16.  Under sustained load with real
// operand values this shape draws less power per flop than 32x32x16 (measured: it sustains a 15-40 % higher
// rate in a register loop), and power is what bounds this kernel beyond its data path.
template <class S> struct Mma16;
template <> struct Mma16<BF16> {
    static __device__ __forceinline__ f32x4 run(s16x8 a, s16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma16<F16> {
    static __device__ __forceinline__ f32x4 run(s16x8 a, s16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// MFMA operands of one K-tile (32 wide), double-buffered in registers: the weights of the wavefront's four
// column tiles (two transpose reads each), and the activations of four of its eight row tiles at a time.
struct WFrags { u32x4 w[TN]; };
struct XFrags { u32x4 x[4]; };                          // four row tiles of 16

struct Task {                                           // wave-uniform description of one output tile
    int unit;                                           // index in the list of live units
    int grp, row0, n0, rows;
};

// One GEMM of the expert FFN: C[g] = act(A[g] B[g] + bias[g]) over the live rows of every group (16-bit storage).
struct StreamPhase {
    const void* A; long long a_group_stride; int lda;
    const int32_t* a_row_index; long long a_index_stride;   // optional gather of the A rows (see GemmArgs)
    const void* B; long long b_group_stride; int ldb;
    void* C; long long c_group_stride; int ldc;
    const void* bias; long long bias_group_stride;
    int N, K;
};
// NPH == 1: the kernel computes ph[0] with activation ACT0.  NPH == 2: also ph[1] (identity), whose A is
// ph[0]'s C: a ph[1] task of a unit starts once all ph[0] column tiles of that unit have been stored.
struct StreamArgs {
    StreamPhase ph[2];
    const int32_t* rows_dev; int rows_cap; int max_rows;
    int32_t* lists;                                     // the scratch block with the two unit lists (see build_ffn_units)
    int groups;
    int wait_target;                                    // NPH == 2: count a unit's completion counter must reach before its ph[1] tasks start
    int spin_limit;                                     // NPH == 2: polls (about 100 ns apart) before a dependency wait gives up
};

constexpr int kSpinLimit = 1 << 21;
constexpr int kActF32Out = 4;                           // template value of ACT: identity with C (and bias) in fp32

// The work of one workgroup on one list for one GEMM (phase PH of the arguments, activation ACT): `list` =
// { fault word, number of live units, ids[cap], completion counters[cap] }; the workgroup is number wg_local of
// the wg_stride workgroups of XCD `xcd` that walk this list.  COUNT: after storing a tile every wavefront adds
// one to its unit's completion counter.  WAIT: before the first copy of a task is requested, its unit's counter
// must have reached a.wait_target (the tiles this task reads are then in the XCD's L2).  `handicap`: see
// ffn_small_list_handicap (0 for the large list).
template <class S, int ACT, int PH, bool COUNT, bool WAIT, int G>
__device__ __forceinline__ void stream_body(const StreamArgs& a, int32_t* list, int cap, int xcd, int wg_local, int wg_stride,
                                            int handicap) {
    typedef uint16_t elem;
    const StreamPhase& P = a.ph[PH];
    int32_t* const fault = list;
    const int32_t* const units = list + 1;              // [0] = live units, [1 + q] = group * nrow + row tile
    int32_t* const done = list + 2 + cap;               // [q] wavefronts that have stored a ph[0] tile of unit q; zero at launch
    constexpr int BM = 128 * G, TM = 4 * G;             // rows of a tile; 16-row MFMA tiles per wavefront
    constexpr int A_COPIES = 2 * G;                     // 1 KB copies per wavefront and activation stage
    static_assert(BM == (G == 2 ? kUnitRowsLarge : kUnitRowsSmall), "the unit list is cut in row tiles of this kernel");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int ncol = (P.N + BN - 1) / BN;
    const int nk = P.K / BK;                            // K-tiles per task (even, >= 6)
    const int nrow = (a.max_rows + BM - 1) / BM;

    // Work is the compact list of live (expert, row tile) units, each one task per column tile.  Each XCD
    // (workgroup ids go round-robin to the 8 XCDs, each with its own L2) takes an equal share of the list, to
    // within one unit whatever the routing skew: the column tiles of a unit run on one XCD at about the same
    // time and share its activation rows through that L2.  When experts can have several row tiles the share is
    // a contiguous block of the list: the row tiles of an expert are neighbours there, so they run on the same
    // XCD at the same time and share the expert's weight panels through that L2 as well (E = 16 at 16K tokens:
    // FFN 0.513 -> 0.455 ms).  With at most one unit per expert the share is every 8th unit, which measured
    // 1.5 % faster than blocks at E = 128 (neighbouring experts' weights, 8 MB apart, stream at the same time
    // instead of regions 128 MB apart).  Inside an XCD the tasks, in order of unit and column tile, are dealt
    // round-robin to its workgroups.
    const int n_units = uniform(units[0]);
    int unit0, unit_step, ux;
    ffn_xcd_share(G == 2, n_units, nrow, xcd, unit0, unit_step, ux);
    const int xcd_tasks = ux * ncol;
    const int my_tasks = ffn_slot_count(wg_local, wg_stride, handicap, xcd_tasks);
    if (my_tasks == 0) return;
    const int first_slot = ffn_first_slot(wg_local, wg_stride, handicap);
    auto position = [&](int slot) __attribute__((always_inline)) { return ffn_slot_position(slot, wg_stride, handicap); };
    // The unit and the live row count of this workgroup's tasks are fetched 64 tasks at a time, one task per
    // lane, so that moving on to the next task costs two lane reads, not two dependent trips to memory.
    int info_unit = 0, info_rows = 0;                   // of this workgroup's task number j0 + lane
    auto load_task_info = [&](int j0) __attribute__((always_inline)) {
        const int p = position(first_slot + (j0 + (int)(threadIdx.x & 63)) * wg_stride);
        if (p < xcd_tasks) {
            int li, ct;
            ffn_task_at(p, ncol, unit0, unit_step, li, ct);
            info_unit = units[1 + li];
            info_rows = min(a.rows_dev[info_unit / nrow], a.rows_cap);
        }
    };
    // task number j of this workgroup, in slot first_slot + j * wg_stride, whose position is < xcd_tasks
    auto task_at = [&](int j, int slot, Task& t) __attribute__((always_inline)) {
        int li, ct;
        ffn_task_at(position(slot), ncol, unit0, unit_step, li, ct);
        t.unit = uniform(li);
        const int unit = __builtin_amdgcn_readlane(info_unit, j & 63);
        t.grp = uniform(unit / nrow);
        t.row0 = uniform((unit % nrow) * BM);
        t.n0 = uniform(ct * BN);
        t.rows = __builtin_amdgcn_readlane(info_rows, j & 63);
    };
    // A second-GEMM task reads what the first-GEMM tasks of its unit stored: wait until all of them (8
    // wavefronts per column tile) have signalled.  First-GEMM tasks never wait, and a workgroup starts on its
    // second-GEMM tasks only after storing all its first-GEMM tiles, so every counter reaches its target
    // whatever the order in which workgroups run; the poll is bounded all the same (a kernel of another stream
    // may hold CUs this launch needs), and a wait that gives up sets the fault word.
    // Producer and consumer run on the same XCD and meet in its L2: the producer's stores are acknowledged
    // by that L2 (vmcnt) before it counts, the counter lives beyond the CU caches (device-scope atomics), and
    // the consumer has never read those lines before, so no cache write-back or invalidate is needed -- an
    // agent-scope release/acquire pair would write back and invalidate the whole L2 on every task.
    auto wait_for_unit = [&](const Task& t) __attribute__((always_inline)) {
        if (WAIT) {
            int spins = 0;
            while (__hip_atomic_load(done + t.unit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < a.wait_target) {
                if (++spins > a.spin_limit) {
                    if (threadIdx.x == 0) __hip_atomic_fetch_or(fault, kFaultWaitGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
            asm volatile("" ::: "memory");
        }
    };
    const int U = uniform(my_tasks * nk);               // K-tiles in this workgroup's whole stream

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- addresses of this wavefront's 1 KB copies, per task: uniform base + per-lane byte offset ----
    // activations: 2 G copies of 8 rows x 128 B per K-tile pair; weights: 2 copies of 2 k-rows x 512 B per K-tile
    auto task_bases = [&](const Task& t, const unsigned char*& base_a, const unsigned char*& base_b) __attribute__((always_inline)) {
        base_a = uniform((const unsigned char*)((const elem*)P.A + (P.a_row_index ? (size_t)0 : (size_t)t.grp * P.a_group_stride)));
        base_b = uniform((const unsigned char*)((const elem*)P.B + (size_t)t.grp * P.b_group_stride));
    };
    auto task_offsets = [&](const Task& t, uint32_t (&oa)[4], uint32_t (&ob)[2]) __attribute__((always_inline)) {
        const int32_t* row_index = P.a_row_index;
        const int lda = P.lda, ldb = P.ldb, N = P.N;
#pragma unroll
        for (int j = 0; j < A_COPIES; ++j) {
            const int r = (wave * A_COPIES + j) * 8 + (lane >> 3), p = lane & 7;
            const int c = p ^ swz_a(r);
            int grow = min(t.row0 + r, t.rows - 1);
            if (row_index) grow = row_index[(size_t)t.grp * P.a_index_stride + grow];
            oa[j] = (uint32_t)grow * (uint32_t)(lda * 2) + c * 16;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = (wave * 2 + j) * 2 + (lane >> 5), p = lane & 31;
            const int c = p ^ swz_b(k);
            const int n = min(t.n0 + c * 8, N - 8);
            ob[j] = (uint32_t)k * (uint32_t)(ldb * 2) + n * 2;
        }
    };

    Task cur, nxt;                                      // task being multiplied; the one after it
    int nxt_j = 0, nxt_p = first_slot;                  // number and slot of `nxt`
    load_task_info(0);
    task_at(nxt_j, nxt_p, cur);
    wait_for_unit(cur);
    const unsigned char *a_base, *b_base;               // copy cursors: bases advance along K
    const unsigned char *na_base, *nb_base;             // bases of the task after `cur`
    uint32_t a_off[4], b_off[2], na_off[4], nb_off[2];
    task_bases(cur, a_base, b_base);
    task_offsets(cur, a_off, b_off);
    nxt = cur;
    ++nxt_j;
    nxt_p += wg_stride;
    if (nxt_j < my_tasks) {
        task_at(nxt_j, nxt_p, nxt);
        wait_for_unit(nxt);
        task_bases(nxt, na_base, nb_base);
        task_offsets(nxt, na_off, nb_off);
    } else {
        na_base = a_base; nb_base = b_base;
#pragma unroll
        for (int j = 0; j < A_COPIES; ++j) na_off[j] = a_off[j];
#pragma unroll
        for (int j = 0; j < 2; ++j) nb_off[j] = b_off[j];
    }
    int a_left = nk / 2, b_left = nk;                   // requests left before a cursor moves to the next task
    const size_t b_step = (size_t)BK * P.ldb * 2;       // bytes between K-tiles of the weights
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const uint32_t lds_a_wave = lds_base + wave * (A_COPIES * 1024);
    const uint32_t lds_b_wave = lds_base + B_REGION + wave * 2048;

    int a_issue_stage = 0, b_issue_stage = 0;
    auto issue_a = [&]() __attribute__((always_inline)) {                              // next pair of K-tiles of the activation rows
        const uint32_t d = lds_a_wave + a_issue_stage * A_STAGE;
#pragma unroll
        for (int j = 0; j < A_COPIES; ++j) copy_to_lds(a_base, a_off[j], d + j * 1024);
        if (--a_left == 0) {
            a_left = nk / 2;
            a_base = na_base;
#pragma unroll
            for (int j = 0; j < A_COPIES; ++j) a_off[j] = na_off[j];
        } else {
            a_base += 128;
        }
        a_issue_stage ^= 1;
    };
    auto issue_b = [&]() __attribute__((always_inline)) {                              // next K-tile of the weights
        const uint32_t d = lds_b_wave + b_issue_stage * B_STAGE;
        copy_to_lds_stream(b_base, b_off[0], d);
        copy_to_lds_stream(b_base, b_off[1], d + 1024);
        if (--b_left == 0) {
            b_left = nk;
            b_base = nb_base;
            b_off[0] = nb_off[0]; b_off[1] = nb_off[1];
        } else {
            b_base += b_step;
        }
        b_issue_stage = b_issue_stage + 1 == B_STAGES ? 0 : b_issue_stage + 1;
    };

    f32x4 acc[TM][TN];                                  // [row tile of 16][column tile of 16]
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[i][j][q] = 0.0f;

    // ---- per-lane LDS read offsets ----
    const int r16 = lane & 15, kq = lane >> 4;          // row/column inside a 16-wide MFMA tile; k-octet of the lane
    const int a_row = wm * TM * 16 + r16;
    const int a_sw = swz_a(a_row);                      // same for every 16-row tile of this lane
    const int bk = kq * 8 + (r16 >> 2);                 // k of the first transpose read; the second is k + 4
    const int b_sw = swz_b(bk);
    int a_rd[2], b_rd[TN];                              // [half of the 64-wide activation stage]
#pragma unroll
    for (int h = 0; h < 2; ++h) a_rd[h] = a_row * 128 + ((((h << 2) | kq) ^ a_sw) << 4);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int chunk = (wn * TN + tn) * 2 + ((r16 & 3) >> 1);
        b_rd[tn] = B_REGION + bk * B_ROW_BYTES + ((chunk ^ b_sw) << 4) + (r16 & 1) * 8;
    }

    // activations of row tiles 4 g .. 4 g + 3, K-tile in activation stage sa, half h: read i of 4
    auto read_x = [&](int i, int g, int sa, int h, XFrags& f) __attribute__((always_inline)) {
        f.x[i] = *(const u32x4*)(smem + sa * A_STAGE + a_rd[h] + (g * 4 + i) * 16 * 128);
    };
    // weights of the K-tile in weight stage sb: read i of 8 (column tile i / 2, k 0-3 or 4-7 of the lane's octet)
    auto read_w = [&](int i, int sb, WFrags& f) __attribute__((always_inline)) {
        const int tn = i >> 1, half = i & 1;
        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                                      (lds_s16x4*)(smem + sb * B_STAGE + b_rd[tn] + half * 4 * B_ROW_BYTES)));
        f.w[tn][2 * half] = t[0];
        f.w[tn][2 * half + 1] = t[1];
    };
    // MFMA i (0..15) of half g of a K-tile: row tile 4 g + i / 4, column tile i % 4
    auto mma_one = [&](int i, int g, const WFrags& wf, const XFrags& xf) __attribute__((always_inline)) {
        const int tm = g * 4 + (i >> 2), tn = i & 3;
        acc[tm][tn] = Mma16<S>::run(__builtin_bit_cast(s16x8, wf.w[tn]), __builtin_bit_cast(s16x8, xf.x[i >> 2]), acc[tm][tn]);
    };

    // ---- epilogue of task `cur`: bias, activation, conversion, transposed store; then advance to the next task ----
    unsigned char* epi = smem + EPI_REGION + wave * EPI_BYTES_PER_WAVE;   // [32 rows][64 columns], 128 B pitch
    auto store_tile = [&]() __attribute__((always_inline)) {
        // the lane number as the epilogue sees it: opaque to the compiler, so that the address arithmetic below
        // is done here and not kept in registers across the main loop
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int r16 = lane_e & 15, kq = lane_e >> 4;
        const int N = P.N;
        const int col_w = cur.n0 + wn * (TN * 16);      // first column of this wavefront
        const size_t c_base = (size_t)cur.grp * P.c_group_stride;
        if constexpr (ACT == kActF32Out) {
            // fp32 output (and fp32 bias), no activation: a lane's four sums of a tile are four consecutive columns of
            // one row, i.e. one 16-byte store straight from the registers
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = cur.row0 + wm * (TM * 16) + tm * 16 + r16;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int col = col_w + tn * 16 + kq * 4;
                    f32x4 v = acc[tm][tn];
                    if (P.bias) {
                        const f32x4 bv = *(const f32x4*)((const float*)P.bias + (size_t)cur.grp * P.bias_group_stride + min(col, N - 4));
                        v[0] += bv[0]; v[1] += bv[1]; v[2] += bv[2]; v[3] += bv[3];
                    }
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[tm][tn][b] = 0.0f;
                    if (row < cur.rows && col < N) *(f32x4*)((float*)P.C + c_base + (size_t)row * P.ldc + col) = v;
                }
            }
            return;
        }
        // accumulator elements 0 .. 3 of tile (tm, tn): columns c .. c + 3 (c = 16 tn + 4 kq) of token row r16
        u32x2 bias_bits[TN];
        if (P.bias) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int c = min(col_w + tn * 16 + kq * 4, N - 4);
                bias_bits[tn] = *(const u32x2*)((const elem*)P.bias + (size_t)cur.grp * P.bias_group_stride + c);
            }
        }
#pragma unroll
        for (int pass = 0; pass < TM / 2; ++pass) {      // 32 rows (two row tiles) at a time
#pragma unroll
            for (int rh = 0; rh < 2; ++rh) {
                const int tm = pass * 2 + rh, rl = rh * 16 + r16;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    float v[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        float bias = 0.0f;
                        if (P.bias) {
                            const uint32_t word = b < 2 ? bias_bits[tn][0] : bias_bits[tn][1];
                            bias = bits16_to_float<S>((uint16_t)((b & 1) ? (word >> 16) : (word & 0xffffu)));
                        }
                        v[b] = apply_act16_t<(ACT == kActF32Out ? 3 : ACT)>(acc[tm][tn][b] + bias);
                        acc[tm][tn][b] = 0.0f;
                    }
                    const int chunk = (tn * 2 + (kq >> 1)) ^ swz_e(rl);
                    *(u32x2*)(epi + rl * 128 + (chunk << 4) + (kq & 1) * 8) = u32x2{pack2<S>(v[0], v[1]), pack2<S>(v[2], v[3])};
                }
            }
            // a wavefront's LDS operations complete in order: the reads below see the writes above, and the
            // writes of the next pass come after these reads
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r_local = i * 8 + (lane_e >> 3), chunk = lane_e & 7;
                const u32x4 v = *(const u32x4*)(epi + r_local * 128 + ((chunk ^ swz_e(r_local)) << 4));
                const int row = cur.row0 + wm * (TM * 16) + pass * 32 + r_local, col = col_w + chunk * 8;
                if (row < cur.rows && col < N) *(u32x4*)((elem*)P.C + c_base + (size_t)row * P.ldc + col) = v;
            }
        }
    };
    auto finish_task = [&]() __attribute__((always_inline)) {
        // Both copy cursors have moved on to `nxt` by now (they run at most 4 K-tiles ahead and K >= 6
        // K-tiles), so the addresses of its successor can replace `nxt`'s.  The loads they need (the gather
        // table) are requested first and used after the tile is stored.
        Task after = nxt;
        ++nxt_j;
        nxt_p += wg_stride;
        if (nxt_j < my_tasks) {
            if ((nxt_j & 63) == 0) load_task_info(nxt_j);
            task_at(nxt_j, nxt_p, after);
            wait_for_unit(after);
            task_bases(after, na_base, nb_base);
            task_offsets(after, na_off, nb_off);
        }
        store_tile();
        if (COUNT) {
            // this wavefront's part of the tile has reached the XCD's L2 before it is counted
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0) __hip_atomic_fetch_add(done + cur.unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        cur = nxt;
        nxt = after;
    };

    // ---- main loop over the stream of K-tiles u = 0 .. U-1 ----
    // K-tile u: weights in stage u % 4, activations in stage (u / 2) % 2, half u % 2; one 32-wide MFMA step
    // per 16 x 16 tile, done as two halves of 16 MFMAs (row tiles 0-3, then 4-7).  Operands are read from
    // LDS one step ahead, slotted between the MFMAs: during the first half the activations of the second
    // half; during the second half the weights and first-half activations of tile u+1.  Early in the second
    // half of tile u the wave waits for tile u+1, then requests weights tile u+4 (into the stage tile u
    // vacated) and, after an odd u, the activation pair (u+3)/2 (into the stage the pair u/2 vacated: every
    // wavefront holds the rest of that pair in registers by then).  Copies of one wave complete in issue
    // order, which in steady state reads
    //   ... B | A B | B | A B | B | A B ...      (A = 2 G copies, B = 2 copies; one group per K-tile)
    // so "tile u+1 has landed" is vmcnt(2 G + 4) before an odd tile (only its weights are new: the newer
    // copies are B A B) and vmcnt(4) before an even tile (its activation pair is new: the newer copies are
    // B B).  Other vector memory operations in flight only make these waits stricter.
    // With G = 1 a wavefront has four row tiles, so a K-tile is one group of 16 MFMAs: the wait and the
    // requests come after its first four, and the twelve reads of tile u+1's operands between the others,
    // with the activations double-buffered by tile (x0 even, x1 odd) instead of by half.
    // requests of the virtual steps -4 .. -1, in steady-state order: B0 A0 B1 B2 A1 B3
    issue_b();
    issue_a();
    issue_b();
    issue_b();
    issue_a();
    issue_b();
    wait_copies_and_barrier<4>();                       // A0 and B0 (and more) have landed
    WFrags w0, w1;                                      // weights of the even / odd tile of a pair
    XFrags x0, x1;                                      // activations of row tiles 0-3 / 4-7 (G = 1: of the even / odd tile)
#pragma unroll
    for (int i = 0; i < 8; ++i) read_w(i, 0, w0);
#pragma unroll
    for (int i = 0; i < 4; ++i) read_x(i, 0, 0, 0, x0);
    int sb = 0;                                         // weight stage of tile u
    int k_done = 0;                                     // K-tiles of `cur` multiplied so far

    // First half of a K-tile (weights wf, activations x0), reading the second half's activations into x1.
    auto first_half = [&](const WFrags& wf, int sa, int h) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            mma_one(i, 0, wf, x0);
            if ((i & 3) == 0) read_x(i >> 2, 1, sa, h, x1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Second half of a K-tile after its first four MFMAs: twelve MFMAs with the twelve reads of the next
    // tile's operands (weights in stage sb_n -> wn_f, activations of its first half -> x0) between them.
    auto second_half_tail = [&](const WFrags& wf, WFrags& wn_f, int sb_n, int sa_n, int h_n) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 4; i < 16; ++i) {
            mma_one(i, 1, wf, x1);
            if (i < 12) read_w(i - 4, sb_n, wn_f);
            else read_x(i - 12, 0, sa_n, h_n, x0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One pair of K-tiles (u even, u + 1).  STEADY: u <= U - 6, so every request below exists and the wait
    // counts above hold; otherwise nothing more is requested and the waits are for everything in flight.
    // LAST: u + 2 == U, nothing follows.
    // G = 1: the twelve MFMAs of a K-tile after its first four (operands wf, xf), with the twelve reads of
    // the next tile's operands (-> wn_f, xn_f) between them.
    auto single_tail = [&](const WFrags& wf, const XFrags& xf, WFrags& wn_f, XFrags& xn_f, int sb_n, int sa_n, int h_n) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 4; i < 16; ++i) {
            mma_one(i, 0, wf, xf);
            if (i < 12) read_w(i - 4, sb_n, wn_f);
            else read_x(i - 12, 0, sa_n, h_n, xn_f);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto pair_of_tiles = [&](int u, auto steady_tag, auto last_tag) __attribute__((always_inline)) {
        constexpr bool STEADY = decltype(steady_tag)::value, LAST = decltype(last_tag)::value;
        constexpr int LAST_G = G - 1;                   // the half of a K-tile whose first four MFMAs cover the wait
        const int sa = (u >> 1) & 1;
        // ---- even tile u ----
        if (G == 2) first_half(w0, sa, 0);
        const int sb1 = (sb + 1) & (B_STAGES - 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) mma_one(i, LAST_G, w0, G == 2 ? x1 : x0);   // these cover the wait for tile u+1
        __builtin_amdgcn_sched_barrier(0);
        wait_copies_and_barrier<STEADY ? A_COPIES + 4 : 0>();
        if (STEADY) issue_b();
        __builtin_amdgcn_sched_barrier(0);
        if (G == 2) second_half_tail(w0, w1, sb1, sa, 1);
        else single_tail(w0, x0, w1, x1, sb1, sa, 1);
        // ---- odd tile u + 1 ----
        if (G == 2) first_half(w1, sa, 1);
        sb = (sb1 + 1) & (B_STAGES - 1);
        if (!LAST) {
#pragma unroll
            for (int i = 0; i < 4; ++i) mma_one(i, LAST_G, w1, x1);
            __builtin_amdgcn_sched_barrier(0);
            wait_copies_and_barrier<STEADY ? 4 : 0>();
            if (STEADY) {
                issue_a();
                issue_b();
            }
            __builtin_amdgcn_sched_barrier(0);
            if (G == 2) second_half_tail(w1, w0, sb, sa ^ 1, 0);
            else single_tail(w1, x1, w0, x0, sb, sa ^ 1, 0);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) mma_one(i, LAST_G, w1, x1);
            __builtin_amdgcn_sched_barrier(0);
        }
        k_done += 2;
        if (k_done == nk) {
            k_done = 0;
            finish_task();
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int u = 0;
    for (; u <= U - 6; u += 2) pair_of_tiles(u, std::true_type{}, std::false_type{});
    pair_of_tiles(u, std::false_type{}, std::false_type{});          // u == U - 4
    pair_of_tiles(u + 2, std::false_type{}, std::true_type{});       // u == U - 2
}

// One persistent workgroup per CU.  A workgroup first walks its share of the XCD's large-tile tasks, then its
// share of the small-tile tasks; nothing separates the two parts but a workgroup barrier, so workgroups with
// few or no large tiles start on the small ones at once.  The small-tile tasks are dealt starting with the
// workgroup after the one that got the XCD's last large-tile task, and the workgroups that got one more large-tile
// task than the others sit out the first round of small ones, which evens out the work (ffn_small_list_handicap).
// NPH == 2 (both FFN GEMMs in one launch): the workgroup then walks its second-GEMM tasks the same way, each
// waiting for its unit's first-GEMM tiles.  Since no workgroup waits for anything before all its own first-GEMM
// tiles are stored, the waits always end (see wait_for_unit).
template <class S, int ACT0, int PH, bool COUNT, bool WAIT>
__device__ __forceinline__ void stream_gemm(const StreamArgs& a, int xcd, int wg, int wgs) {
    const int nrow_l = ffn_units_nrow_large(a.max_rows), nrow_s = ffn_units_nrow_small(a.max_rows);
    int32_t* const list_l = a.lists;
    int32_t* const list_s = a.lists + ffn_units_small_offset(a.groups, a.max_rows);
    const int n_l = nrow_l ? uniform(list_l[1]) : 0, n_s = uniform(list_s[1]);
    int unit0, unit_step, ux_l, ux_s;
    ffn_xcd_share(true, n_l, nrow_l, xcd, unit0, unit_step, ux_l);
    ffn_xcd_share(false, n_s, nrow_s, xcd, unit0, unit_step, ux_s);
    if (ux_l > 0) stream_body<S, ACT0, PH, COUNT, WAIT, 2>(a, list_l, a.groups * nrow_l, xcd, wg, wgs, 0);
    if (ux_s > 0) {
        if (ux_l > 0) __syncthreads();                  // every wavefront is done with the LDS stages of the first part
        const int ncol = (a.ph[PH].N + BN - 1) / BN;
        const int wg_s = ffn_small_list_rotation(wg, wgs, ux_l, ncol);
        stream_body<S, ACT0, PH, COUNT, WAIT, 1>(a, list_s, a.groups, xcd, wg_s, wgs, ffn_small_list_handicap(wgs, ux_l, ncol));
    }
}

// Tiles that one workgroup writes and another reads inside a launch (first-GEMM tiles when both GEMMs share a
// launch) meet in one XCD's L2, which holds only if the workgroups with the same block number modulo 8 really
// share an XCD.  Each workgroup records the hardware XCD it runs on (XCC_ID, bits 3:0 of that hardware register) in
// its class's placement word; a second, different value sets the fault word (the results may then be stale, and
// moe_ffn_status says so).  Called by thread 0 of a workgroup; `xcd` = block number modulo 8.
__device__ __forceinline__ void check_xcd_placement(const StreamArgs& a, int xcd) {
    int32_t* const placement = a.lists + ffn_units_placement_offset(a.groups, a.max_rows);
    int32_t* const fault = a.lists + ffn_units_small_offset(a.groups, a.max_rows);
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    const int mine = (int)(xcc & 15u);
    int expected = -1;
    if (!__hip_atomic_compare_exchange_strong(placement + xcd, &expected, mine, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT) && expected != mine)
        __hip_atomic_fetch_or(fault, kFaultPlacement, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

inline StreamPhase to_phase(const GemmArgs& g) {
    StreamPhase p{};
    p.A = g.A; p.a_group_stride = g.a_group_stride; p.lda = g.lda;
    p.a_row_index = g.a_row_index; p.a_index_stride = g.a_index_stride;
    p.B = g.B; p.b_group_stride = g.b_group_stride; p.ldb = g.ldb;
    p.C = g.C; p.c_group_stride = g.c_group_stride; p.ldc = g.ldc;
    p.bias = g.bias; p.bias_group_stride = g.bias_group_stride;
    p.N = g.N; p.K = g.K;
    return p;
}

}  // namespace
}  // namespace moe
