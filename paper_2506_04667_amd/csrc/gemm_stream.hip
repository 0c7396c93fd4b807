// Weight-streaming grouped GEMM for the expert FFN tasks in 16-bit storage
// (C1 <- phi1(A B1 + D1), C2 <- C1 B2 + D2; Sec. 3.1).  At the paper's expert-scaling
// shape an expert has only ~256 live rows, so each weight matrix is used by one row
// tile and the kernel is bound by streaming weights from HBM once, not by the
// matrix cores.  The design therefore maximises bytes in flight per CU and keeps
// the LDS and MFMA pipes busy at the same time:
//
//   * tile 256 x 256 per workgroup (8 wavefronts as 2 x 4, 128 rows x 64 columns
//     each, MFMA 32x32x16): an expert with <= 256 live rows reads its weights once;
//   * K-tile 32.  Weights (from HBM) go through a ring of NS LDS stages of 16 KB
//     (32 x 256), requested NS-1 K-tiles ahead; activations (re-read from L2 by the
//     8 column tiles of an expert) go through 2 stages of 32 KB that hold two
//     K-tiles each (256 rows x 128 B), so that every L2 request is a full 128-byte
//     line -- the L1's outstanding-request queue, not HBM, is what saturates first;
//     global -> LDS copies are direct (global_load_lds_dwordx4: no VGPR staging);
//   * the copies are issued from inline asm and waited for with explicit
//     s_waitcnt vmcnt(n) + s_barrier, because a compiler-visible LDS-DMA makes every
//     later LDS read wait for all outstanding copies;
//   * MFMA operand fragments are double-buffered in registers at k-step (16)
//     granularity: while the MFMAs of one k-step run, the LDS reads of the next are
//     in flight, across the K-tile boundary too.
//
// A direct copy writes 64 lanes x 16 B to 1024 contiguous LDS bytes (lane i at
// base + 16 i), while each lane picks its own global address; the XOR swizzles below
// are therefore applied on the global side (which 16-byte chunk a lane fetches).
//   A stage: row pitch 128 B; chunk c of row r lives at c ^ ((r >> 1) & 7).
//   B stage: [k][n], row pitch 512 B; chunk c of row k lives at c ^ ((k & 3) << 1);
//            read back in MFMA operand order with ds_read_b64_tr_b16.
// Rows at or beyond the live row count are fetched from the last live row (their
// products land in output rows that are never stored); columns beyond N likewise.
// Because every lane supplies its own global address, the activation rows can be
// gathered straight from the token matrix through the routing table (slot -> token):
// the payload-efficient dispatch of Sec. 3.2.1 without a packed copy.
//
// The MFMAs take the weight fragment as their first operand, so a lane's
// accumulators hold, for ONE token row, runs of four consecutive output columns.
// The epilogue applies bias and activation in registers, packs each run to 8 bytes,
// transposes through the (now idle) LDS and stores full 128-byte row segments.
//
// Requires K % 64 == 0 and N % 8 == 0; other shapes use the generic kernel.
#include "common.h"
#include "kernels.h"

namespace moe {
namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kXcds = 8;
constexpr int BM = 256, BN = 256, BK = 32, THREADS = 512;
constexpr int A_STAGE = BM * 128;                       // 256 rows x 64 k (two K-tiles)
constexpr int A_STAGES = 2;
constexpr int B_STAGE = BK * BN * 2;                    // 32 k x 256 columns
constexpr int B_ROW_BYTES = BN * 2;
constexpr int B_REGION = A_STAGES * A_STAGE;            // weights ring starts after the activation stages
constexpr int TM = 4, TN = 2, WN = 4;                   // 32x32 MFMA tiles per wavefront; wavefronts along N
constexpr int EPI_BYTES_PER_WAVE = 128 * 128;           // 128 rows x 64 columns x 2 B

template <class S> struct Mma16;
template <> struct Mma16<BF16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma16<F16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// 64 lanes x 16 bytes from per-lane global addresses to LDS [lds_addr, lds_addr + 1024)
__device__ __forceinline__ void copy_to_lds(const void* gptr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

// own copies older than the newest N have landed; own LDS reads are complete; then meet the other waves
template <int N>
__device__ __forceinline__ void wait_copies_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

struct Frags {                                          // MFMA operands of one 16-wide k-step
    s16x8 x[TM];                                        // activations, per row tile
    s16x8 w[TN];                                        // weights, per column tile
};

template <class S, int NS, int ACT>
__global__ __launch_bounds__(THREADS) void ffn_gemm_stream_kernel(GemmArgs a) {
    typedef uint16_t elem;
    static_assert(NS == 5, "the wait counts below are derived for five weight stages");
    static_assert(B_REGION + NS * B_STAGE >= 8 * EPI_BYTES_PER_WAVE, "epilogue staging must fit in the rings");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // ---- task decode: all tiles of an expert on one XCD (ids are dealt round-robin to XCDs) ----
    const int ncol = (a.N + BN - 1) / BN;
    const int nrow = (a.max_rows + BM - 1) / BM;
    int grp, rt, ct;
    {
        const int id = blockIdx.x, per_group = nrow * ncol;
        if (a.groups >= kXcds) {
            const int x = id % kXcds, s = id / kXcds;
            grp = (s / per_group) * kXcds + x;
            rt = (s % per_group) / ncol;
            ct = (s % per_group) % ncol;
        } else {
            grp = id / per_group;
            rt = (id % per_group) / ncol;
            ct = (id % per_group) % ncol;
        }
    }
    if (grp >= a.groups) return;
    const int row0 = rt * BM, n0 = ct * BN;
    const int rows = min(a.rows_dev[grp], a.rows_cap);
    if (row0 >= rows) return;
    const int K = a.K, N = a.N;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g2 = lane >> 5;

    // ---- per-lane global addresses of this wavefront's 1 KB copies ----
    const elem* A = (const elem*)a.A + (a.a_row_index ? (size_t)0 : (size_t)grp * a.a_group_stride);
    const elem* B = (const elem*)a.B + (size_t)grp * a.b_group_stride;
    const unsigned char* ga[4];                         // activations: 4 copies of 8 rows x 128 B per K-tile pair
    const unsigned char* gb[2];                         // weights: 2 copies of 2 k-rows x 512 B per K-tile
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (wave * 4 + j) * 8 + (lane >> 3), p = lane & 7;
        const int c = p ^ ((r >> 1) & 7);
        int grow = min(row0 + r, rows - 1);
        if (a.a_row_index) grow = a.a_row_index[(size_t)grp * a.a_index_stride + grow];
        ga[j] = (const unsigned char*)(A + (size_t)grow * a.lda + c * 8);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = (wave * 2 + j) * 2 + (lane >> 5), p = lane & 31;
        const int c = p ^ ((k & 3) << 1);
        const int n = min(n0 + c * 8, N - 8);
        gb[j] = (const unsigned char*)(B + (size_t)k * a.ldb + n);
    }
    const size_t b_step = (size_t)BK * a.ldb * 2;
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const uint32_t lds_a_wave = lds_base + wave * 4096;
    const uint32_t lds_b_wave = lds_base + B_REGION + wave * 2048;

    int a_issue_stage = 0, b_issue_stage = 0;
    auto issue_a = [&]() {                              // next pair of K-tiles of the activation rows
        const uint32_t d = lds_a_wave + a_issue_stage * A_STAGE;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            copy_to_lds(ga[j], d + j * 1024);
            ga[j] += 128;
        }
        a_issue_stage ^= 1;
    };
    auto issue_b = [&]() {                              // next K-tile of the weights
        const uint32_t d = lds_b_wave + b_issue_stage * B_STAGE;
        copy_to_lds(gb[0], d);
        copy_to_lds(gb[1], d + 1024);
        gb[0] += b_step; gb[1] += b_step;
        b_issue_stage = b_issue_stage + 1 == NS ? 0 : b_issue_stage + 1;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

    // ---- per-lane LDS read offsets ----
    const int a_row = wm * TM * 32 + l32;
    const int a_sw = (a_row >> 1) & 7;                  // same for every 32-row MFMA tile of this lane
    const int L = lane & 15, nb = (lane >> 4) & 1;
    const int bk = g2 * 8 + (L >> 2);                   // k of the first transpose read; second is k + 4
    int a_rd[2][2], b_rd[TN];                           // [half of the 64-wide stage][k-step]
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) a_rd[h][ks] = a_row * 128 + ((((h << 2) | (ks << 1) | g2) ^ a_sw) << 4);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int chunk = (wn * TN + tn) * 4 + nb * 2 + ((L & 3) >> 1);
        b_rd[tn] = B_REGION + bk * B_ROW_BYTES + ((chunk ^ ((bk & 3) << 1)) << 4) + (L & 1) * 8;
    }

    // operands of k-step ks of the K-tile in activation stage sa (half h) and weight stage sb
    auto load_frags = [&](int sa, int h, int sb, Frags& f, int ks) {
        const unsigned char* pa = smem + sa * A_STAGE + a_rd[h][ks];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) f.x[tm] = *(const s16x8*)(pa + tm * 32 * 128);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const unsigned char* p = smem + sb * B_STAGE + b_rd[tn] + ks * 16 * B_ROW_BYTES;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * B_ROW_BYTES));
            f.w[tn] = s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    };
    auto mma = [&](const Frags& f) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = Mma16<S>::run(f.w[tn], f.x[tm], acc[tm][tn]);
    };

    // ---- main loop ----
    // K-tile t: weights in stage t % NS, activations in stage (t / 2) % 2, half t % 2; consumed as two
    // 16-wide k-steps.  The operands of the next k-step are read from LDS while the MFMAs of the current one
    // run.  Between the two k-steps of tile t the wave waits for tile t+1, then requests weights tile t+NS
    // (into the stage tile t vacated) and, after an odd t, the activation pair (t+3)/2 (into the stage the
    // pair t/2 vacated).  Copies of one wave complete in issue order, which in steady state reads
    //   ... A B B | A B B | A B B ...        (A = 4 copies, B = 2 copies)
    // so "tile t+1 has landed" is vmcnt(14) before an odd tile (only its weights are new: the newer
    // copies are A B B A B) and vmcnt(4) before an even tile (its activation pair is new: newer are B B).
    const int nk = K / BK;                              // even
    const int npair = nk / 2;
    // requests of the virtual steps -5 .. -1, in steady-state order: B0 B1 A0 B2 B3 A1 B4
    if (0 < nk) issue_b();
    if (1 < nk) issue_b();
    issue_a();
    if (2 < nk) issue_b();
    if (3 < nk) issue_b();
    if (1 < npair) issue_a();
    if (4 < nk) issue_b();
    if (nk >= 6) wait_copies_and_barrier<4>();          // A0 and B0 (and more) have landed
    else wait_copies_and_barrier<0>();
    Frags f0, f1;
    load_frags(0, 0, 0, f0, 0);
    int sb = 0;                                         // weight stage of tile t
    for (int t = 0; t < nk; t += 2) {
        const int sa = (t >> 1) & 1;
        // ---- even tile t ----
        load_frags(sa, 0, sb, f1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(f0);
        __builtin_amdgcn_sched_barrier(0);
        int sb1 = sb + 1 == NS ? 0 : sb + 1;
        if (t <= nk - 5) wait_copies_and_barrier<14>();
        else wait_copies_and_barrier<0>();
        if (t + NS < nk) issue_b();
        load_frags(sa, 1, sb1, f0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(f1);
        __builtin_amdgcn_sched_barrier(0);
        // ---- odd tile t + 1 ----
        load_frags(sa, 1, sb1, f1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(f0);
        __builtin_amdgcn_sched_barrier(0);
        sb = sb1 + 1 == NS ? 0 : sb1 + 1;
        if (t + 2 < nk) {
            if (t + 1 <= nk - 5) wait_copies_and_barrier<4>();
            else wait_copies_and_barrier<0>();
            // every wave holds the rest of the pair in registers: its activation stage can be refilled
            if ((t + 4) / 2 < npair) issue_a();
            if (t + 1 + NS < nk) issue_b();
            load_frags(sa ^ 1, 0, sb, f0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        mma(f1);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue ----
    // All waves must be done reading the ring before it is reused as staging space.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    unsigned char* epi = smem + wave * EPI_BYTES_PER_WAVE;   // [128 rows][64 columns] of this wavefront, 128 B pitch
    const int col_w = n0 + wn * (TN * 32);                   // first column of this wavefront
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
        for (int qa = 0; qa < 4; ++qa) {
            // accumulator elements 4 qa .. 4 qa + 3: columns c .. c + 3 of one token row
            const int c_local = tn * 32 + qa * 8 + g2 * 4;
            float bias[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (a.bias) {
                const int c = min(col_w + c_local, N - 4);
                const u32x2 bv = *(const u32x2*)((const elem*)a.bias + (size_t)grp * a.bias_group_stride + c);
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t word = b < 2 ? bv[0] : bv[1];
                    bias[b] = bits16_to_float<S>((uint16_t)((b & 1) ? (word >> 16) : (word & 0xffffu)));
                }
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                float v[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) v[b] = apply_act_t<ACT>(acc[tm][tn][qa * 4 + b] + bias[b]);
                const int r_local = tm * 32 + l32;
                const int chunk = (c_local >> 3) ^ ((r_local >> 1) & 7);
                *(u32x2*)(epi + r_local * 128 + (chunk << 4) + g2 * 8) = u32x2{pack2<S>(v[0], v[1]), pack2<S>(v[2], v[3])};
            }
        }
    }
    // a wavefront's LDS operations complete in order: the reads below see the writes above
    const size_t c_base = (size_t)grp * a.c_group_stride;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int r_local = i * 8 + (lane >> 3), chunk = lane & 7;
        const u32x4 v = *(const u32x4*)(epi + r_local * 128 + ((chunk ^ ((r_local >> 1) & 7)) << 4));
        const int row = row0 + wm * (TM * 32) + r_local, col = col_w + chunk * 8;
        if (row < rows && col < N) *(u32x4*)((elem*)a.C + c_base + (size_t)row * a.ldc + col) = v;
    }
}

template <class S, int NS, int ACT>
hipError_t launch_stream_t(const GemmArgs& a, hipStream_t stream) {
    auto kernel = ffn_gemm_stream_kernel<S, NS, ACT>;
    constexpr int lds_bytes = B_REGION + NS * B_STAGE;
    static bool attr_set = false;                       // LDS above 64 KB must be requested once per kernel
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long long ncol = (a.N + BN - 1) / BN, nrow = (a.max_rows + BM - 1) / BM;
    const long long groups = a.groups >= kXcds ? (long long)(a.groups + kXcds - 1) / kXcds * kXcds : a.groups;
    const long long blocks = groups * nrow * ncol;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(THREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

template <class S>
hipError_t launch_stream_act(const GemmArgs& a, hipStream_t stream) {
    switch (a.act) {
        case 0: return launch_stream_t<S, 5, 0>(a, stream);
        case 1: return launch_stream_t<S, 5, 1>(a, stream);
        case 2: return launch_stream_t<S, 5, 2>(a, stream);
        default: return launch_stream_t<S, 5, 3>(a, stream);
    }
}

}  // namespace

bool stream_gemm_eligible(const GemmArgs& a) {
    return a.dtype != 0 && !a.b_is_nk && !a.c_f32 && a.rows_dev != nullptr && a.K % (2 * BK) == 0 && a.K >= 2 * BK &&
           a.N % 8 == 0 && a.N >= 256 && a.max_rows > 128 && a.lda % 8 == 0 && a.ldb % 8 == 0 && a.ldc % 8 == 0;
}

hipError_t launch_grouped_gemm_stream(const GemmArgs& a, hipStream_t stream) {
    return a.dtype == 1 ? launch_stream_act<BF16>(a, stream) : launch_stream_act<F16>(a, stream);
}

}  // namespace moe
