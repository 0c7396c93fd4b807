// Grouped tile GEMM on CDNA4 matrix cores: the two FFN tasks of every expert
// (C1 <- phi1(A B1 + D1), C2 <- C1 B2 + D2, Sec. 3.1 task abstraction) and the gate
// projection share this kernel.  One workgroup computes one (group, row tile,
// column tile) task; tasks whose row tile lies beyond the group's live rows exit at
// once, so only ceil(rows/BM) row tiles per expert are ever computed (the in-place
// padding idea of Sec. 3.2.1) and no task list or host round trip is needed.
//
// Two tile shapes, both built from 32 x 32 MFMA tiles:
//   large  256 x 256, 8 wavefronts (2 x 4), 128 x 64 per wavefront  -- expert FFNs
//   small  128 x 128, 4 wavefronts (2 x 2),  64 x 64 per wavefront  -- gate, small shapes
// 16-bit storage uses v_mfma_f32_32x32x16_{bf16,f16} with K-tile 64; fp32 uses
// v_mfma_f32_32x32x2_f32 with K-tile 32 (a stage is 128 bytes per A row either
// way).  With a 256-row tile an expert of up to 256 live rows streams its weight
// matrix from HBM exactly once.
//
// Pipeline: two LDS stages; the global loads of K-tile t+2 are in flight in
// registers while K-tile t is multiplied and K-tile t+1 is written to the other
// stage in the middle of the multiply; one barrier per K-tile.
//
// LDS layouts are unpadded and XOR-swizzled at 16-byte-chunk granularity (64
// banks of 4 bytes):
//   A (and an [n][k] B):  row pitch 128 B, chunk c of row r lives at c ^ ((r >> 1) & 7)
//                         -> 16-byte operand reads of 16 consecutive rows hit 16 distinct chunks.
//   [k][n] B, 16-bit:     chunk c of row k lives at c ^ ((k & 3) << 2); the MFMA B operand
//                         (k contiguous per lane) is produced by the LDS transpose read
//                         ds_read_b64_tr_b16: within 16 lanes, lane i receives, as element j,
//                         element (i % 4) of the 8-byte row addressed by lane 4 j + i / 4.
//   [k][n] B, fp32:       chunk c of row k lives at c ^ (((k >> 2) & 1) << 3) so that the two
//                         half-waves (k and k + 4) use disjoint banks.
//
// Workgroup ids are mapped so that all tiles of one expert run on the same XCD
// (ids are dealt round-robin to the 8 XCDs, each with its own L2): the column
// tiles of an expert then share its activation rows, and its row tiles share
// the weight panels, through that L2.
#include "common.h"
#include "kernels.h"

#include <type_traits>

namespace moe {
namespace {

template <class S> struct Mma;
template <> struct Mma<BF16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<F16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kXcds = 8;

template <class S, bool NT, int WM, int WN, int TM, int TN>
struct Cfg {
    static constexpr bool k16 = (S::kBytes == 2);
    static constexpr int VEC = S::kVec;                 // elements per 16-byte chunk
    static constexpr int BK = 8 * VEC;                  // 64 (16-bit) or 32 (fp32): 128 bytes of k per row
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    static constexpr int THREADS = WM * WN * 64;
    static constexpr int A_BYTES = BM * 128;
    static constexpr int B_ROW_BYTES = NT ? 128 : BN * S::kBytes;
    static constexpr int B_ROWS = NT ? BN : BK;
    static constexpr int B_BYTES = B_ROWS * B_ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_LOADS = BM * 8 / THREADS;    // 16-byte chunks per thread per stage
    static constexpr int B_CPR = B_ROW_BYTES / 16;      // chunks per B tile row
    static constexpr int B_LOADS = B_ROWS * B_CPR / THREADS;
    static_assert(BM * 8 % THREADS == 0 && B_ROWS * B_CPR % THREADS == 0, "tile/threads mismatch");
};

// byte offset of 16-byte chunk c of row r in an A-style tile (row pitch 128 B)
__device__ __forceinline__ int a_off(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }
// byte offset of 16-byte chunk c of row k in a [k][n] B tile
template <bool k16>
__device__ __forceinline__ int b_off(int k, int c, int row_bytes) {
    return k * row_bytes + ((c ^ (k16 ? ((k & 3) << 2) : (((k >> 2) & 1) << 3))) << 4);
}

template <class S, bool NT, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(WM * WN * 64) void grouped_gemm_kernel(GemmArgs a) {
    using C = Cfg<S, NT, WM, WN, TM, TN>;
    typedef typename S::store_t elem;
    constexpr bool k16 = C::k16;
    constexpr int VEC = C::VEC, BK = C::BK, BM = C::BM, BN = C::BN, THREADS = C::THREADS;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // ---- task decode: all tiles of a group on one XCD when there are enough groups ----
    const int ncol = (a.N + BN - 1) / BN;
    const int nrow = (a.max_rows + BM - 1) / BM;
    int grp, rt, ct;
    {
        const int id = blockIdx.x;
        const int per_group = nrow * ncol;
        if (a.groups >= kXcds) {
            const int x = id % kXcds, s = id / kXcds;
            grp = (s / per_group) * kXcds + x;
            const int r = s % per_group;
            rt = r / ncol;
            ct = r % ncol;
        } else {
            grp = id / per_group;
            const int r = id % per_group;
            rt = r / ncol;
            ct = r % ncol;
        }
    }
    if (grp >= a.groups) return;
    const int row0 = rt * BM, n0 = ct * BN;
    const int rows = a.rows_dev ? min(a.rows_dev[grp], a.rows_cap) : a.rows_fixed;
    if (row0 >= rows) return;

    const elem* A = (const elem*)a.A + (a.a_row_index ? (size_t)0 : (size_t)grp * a.a_group_stride);
    const elem* B = (const elem*)a.B + (size_t)grp * a.b_group_stride;
    const int K = a.K, N = a.N;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g2 = lane >> 5;

    // global row of each A chunk this thread loads (through the gather table when there is one)
    int a_grow[C::A_LOADS];
#pragma unroll
    for (int i = 0; i < C::A_LOADS; ++i) {
        const int r = row0 + ((tid + i * THREADS) >> 3);
        a_grow[i] = (a.a_row_index && r < rows) ? a.a_row_index[(size_t)grp * a.a_index_stride + r] : r;
    }

    u32x4 ra[C::A_LOADS], rb[C::B_LOADS];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            const int c = tid + i * THREADS;
            const int r = c >> 3, kc = (c & 7) * VEC;
            const bool ok = (row0 + r < rows) && (k0 + kc < K);
            ra[i] = ok ? *(const u32x4*)(A + (size_t)a_grow[i] * a.lda + k0 + kc) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) {
            const int c = tid + i * THREADS;
            if (NT) {
                const int r = c >> 3, kc = (c & 7) * VEC;
                const bool ok = (n0 + r < N) && (k0 + kc < K);
                rb[i] = ok ? *(const u32x4*)(B + (size_t)(n0 + r) * a.ldb + k0 + kc) : u32x4{0, 0, 0, 0};
            } else {
                const int r = c / C::B_CPR, nc = (c % C::B_CPR) * VEC;
                const bool ok = (k0 + r < K) && (n0 + nc < N);
                rb[i] = ok ? *(const u32x4*)(B + (size_t)(k0 + r) * a.ldb + n0 + nc) : u32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_lds = [&](int stage) {
        unsigned char* sa = smem + stage * C::STAGE_BYTES;
        unsigned char* sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            const int c = tid + i * THREADS;
            *(u32x4*)(sa + a_off(c >> 3, c & 7)) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) {
            const int c = tid + i * THREADS;
            if (NT) *(u32x4*)(sb + a_off(c >> 3, c & 7)) = rb[i];
            else *(u32x4*)(sb + b_off<k16>(c / C::B_CPR, c % C::B_CPR, C::B_ROW_BYTES)) = rb[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

    // per-lane LDS read bases.  A-style tiles: the swizzle term of a row depends on (row >> 1) & 7,
    // which is the same for every 32-row MFMA tile of this lane.
    const int a_row = wm * TM * 32 + l32;
    const int a_sw = (a_row >> 1) & 7;
    const int bn_row = wn * TN * 32 + l32;               // NT: B rows are n
    const int bn_sw = (bn_row >> 1) & 7;

    // one 128-byte slice of k (4 MFMA k-steps for 16-bit, 4 groups of 4 for fp32), steps [s0, s1)
    auto compute = [&](int stage, int s0, int s1) {
        const unsigned char* sa = smem + stage * C::STAGE_BYTES;
        const unsigned char* sb = sa + C::A_BYTES;
        if constexpr (k16) {
#pragma unroll
            for (int ks = s0; ks < s1; ++ks) {           // 16 k per step; chunk = 2 ks + g2
                s16x8 af[TM], bf[TN];
                const int a_chunk = ((ks << 1) | g2) ^ a_sw;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    af[tm] = *(const s16x8*)(sa + (a_row + tm * 32) * 128 + (a_chunk << 4));
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    if (NT) {
                        const int b_chunk = ((ks << 1) | g2) ^ bn_sw;
                        bf[tn] = *(const s16x8*)(sb + (bn_row + tn * 32) * 128 + (b_chunk << 4));
                    } else {
                        // lanes 0-15 / 16-31: columns 0-15 / 16-31 of the 32-wide tile; lanes 32-63: k + 8
                        const int L = lane & 15, nb = (lane >> 4) & 1;
                        const int k = ks * 16 + g2 * 8 + (L >> 2);          // second read: k + 4 (same k & 3)
                        const int chunk = (wn * TN + tn) * 4 + nb * 2 + ((L & 3) >> 1);
                        const unsigned char* p = sb + b_off<true>(k, chunk, C::B_ROW_BYTES) + (L & 1) * 8;
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * C::B_ROW_BYTES));
                        bf[tn] = s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    }
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = Mma<typename std::conditional<k16, S, BF16>::type>::run(af[tm], bf[tn], acc[tm][tn]);
            }
        } else {
#pragma unroll
            for (int ks = s0; ks < s1; ++ks) {           // 8 k per step: lanes 0-31 take k..k+3, lanes 32-63 k+4..k+7
                f32x4 af[TM];
                float bfr[TN][4];
                const int a_chunk = ((ks << 1) | g2) ^ a_sw;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    af[tm] = *(const f32x4*)(sa + (a_row + tm * 32) * 128 + (a_chunk << 4));
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    if (NT) {
                        const int b_chunk = ((ks << 1) | g2) ^ bn_sw;
                        const f32x4 t = *(const f32x4*)(sb + (bn_row + tn * 32) * 128 + (b_chunk << 4));
#pragma unroll
                        for (int j = 0; j < 4; ++j) bfr[tn][j] = t[j];
                    } else {
                        const int n = (wn * TN + tn) * 32 + l32;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int k = ks * 8 + g2 * 4 + j;
                            bfr[tn][j] = *(const float*)(sb + b_off<false>(k, n >> 2, C::B_ROW_BYTES) + (n & 3) * 4);
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[tm][j], bfr[tn][j], acc[tm][tn], 0, 0, 0);
            }
        }
    };

    const int nk = (K + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    if (nk > 1) load_global(BK);
    __syncthreads();
    for (int t = 0; t < nk; ++t) {
        const int cur = t & 1;
        if (t + 1 < nk) {
            store_lds(cur ^ 1);                          // K-tile t+1; that stage was last read before the previous barrier
            if (t + 2 < nk) load_global((t + 2) * BK);   // a whole K-tile of MFMAs to arrive
        }
        compute(cur, 0, 4);
        __syncthreads();
    }

    // epilogue on the accumulator registers: bias, activation, conversion, store
    const size_t c_base = (size_t)grp * a.c_group_stride;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int col = n0 + (wn * TN + tn) * 32 + l32;
        if (col >= N) continue;
        float bias = 0.0f;
        if (a.bias) {
            const size_t bi = (size_t)grp * a.bias_group_stride + col;
            bias = a.c_f32 ? ((const float*)a.bias)[bi] : load_as_float<S>(a.bias, bi);
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = row0 + (wm * TM + tm) * 32 + (q >> 2) * 8 + g2 * 4 + (q & 3);
                if (row >= rows) continue;
                const float v = apply_act(acc[tm][tn][q] + bias, a.act);
                const size_t ci = c_base + (size_t)row * a.ldc + col;
                if (a.c_f32) ((float*)a.C)[ci] = v;
                else store_from_float<S>(a.C, ci, v);
            }
        }
    }
}

// the kernel's LDS limit on the current device (once per device)
template <class S, bool NT, int WM, int WN, int TM, int TN>
hipError_t prepare_cfg() {
    static DeviceFlags limit_raised = {};
    return raise_lds_limit(reinterpret_cast<const void*>(grouped_gemm_kernel<S, NT, WM, WN, TM, TN>),
                           2 * Cfg<S, NT, WM, WN, TM, TN>::STAGE_BYTES, limit_raised);
}

template <class S, bool NT, int WM, int WN, int TM, int TN>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t stream) {
    using C = Cfg<S, NT, WM, WN, TM, TN>;
    auto kernel = grouped_gemm_kernel<S, NT, WM, WN, TM, TN>;
    constexpr int lds_bytes = 2 * C::STAGE_BYTES;
    if (hipError_t e = prepare_cfg<S, NT, WM, WN, TM, TN>(); e != hipSuccess) return e;
    const long long ncol = (a.N + C::BN - 1) / C::BN;
    const long long nrow = (a.max_rows + C::BM - 1) / C::BM;
    const long long groups = a.groups >= kXcds ? (long long)(a.groups + kXcds - 1) / kXcds * kXcds : a.groups;
    const long long blocks = groups * nrow * ncol;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(C::THREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

template <class S>
hipError_t launch_t(const GemmArgs& a, hipStream_t stream) {
    // Tile choice from the row bound alone (live row counts are only known on the device).  A CU works through
    // the tiles it is given at the same rate however many of them are resident, so the time of a launch is about
    // ceil(tiles / CUs) x tile area / efficiency: 256 x 256 (one per CU), 128 x 128 (two per CU, about 0.94 of
    // the large tile's efficiency) and, for fp32 storage, 128 x 64 (three per CU, about 0.85), which evens out
    // launches with fewer 128 x 128 tiles than two per CU.
    const long long cus = device_cu_count();
    auto cost = [&](int bm, int bn, double eff) {
        const long long tiles = (long long)a.groups * ((a.max_rows + bm - 1) / bm) * ((a.N + bn - 1) / bn);
        return (double)((tiles + cus - 1) / cus) * (double)(bm * bn) / eff;
    };
    int pick = 1;                                        // 0: 256 x 256, 1: 128 x 128, 2: 128 x 64, 3: 64 x 128
    double best = cost(128, 128, 0.94);
    if (a.N > 128 && a.max_rows > 128 && cost(256, 256, 1.0) <= best) {
        pick = 0;
        best = cost(256, 256, 1.0);
    }
    if constexpr (S::kBytes == 4) {
        if (!a.b_is_nk && a.N > 64 && cost(128, 64, 0.85) < best) {
            pick = 2;
            best = cost(128, 64, 0.85);
        }
        if (!a.b_is_nk && a.max_rows > 64 && cost(64, 128, 0.85) < best) pick = 3;
    }
    if (a.b_is_nk) {
        return pick == 0 ? launch_cfg<S, true, 2, 4, 4, 2>(a, stream) : launch_cfg<S, true, 2, 2, 2, 2>(a, stream);
    }
    if constexpr (S::kBytes == 4) {
        if (pick == 2) return launch_cfg<S, false, 2, 2, 2, 1>(a, stream);
        if (pick == 3) return launch_cfg<S, false, 1, 4, 2, 1>(a, stream);
    }
    return pick == 0 ? launch_cfg<S, false, 2, 4, 4, 2>(a, stream) : launch_cfg<S, false, 2, 2, 2, 2>(a, stream);
}

template <class S>
hipError_t prepare_t() {
    hipError_t e = prepare_cfg<S, true, 2, 4, 4, 2>();
    if (e == hipSuccess) e = prepare_cfg<S, true, 2, 2, 2, 2>();
    if (e == hipSuccess) e = prepare_cfg<S, false, 2, 4, 4, 2>();
    if (e == hipSuccess) e = prepare_cfg<S, false, 2, 2, 2, 2>();
    if constexpr (S::kBytes == 4) {
        if (e == hipSuccess) e = prepare_cfg<S, false, 2, 2, 2, 1>();
        if (e == hipSuccess) e = prepare_cfg<S, false, 1, 4, 2, 1>();
    }
    return e;
}

}  // namespace

hipError_t prepare_grouped_gemm() {
    hipError_t e = prepare_t<F32>();
    if (e == hipSuccess) e = prepare_t<BF16>();
    if (e == hipSuccess) e = prepare_t<F16>();
    return e;
}

hipError_t launch_grouped_gemm(const GemmArgs& a, hipStream_t stream) {
    if (a.groups <= 0 || a.max_rows <= 0 || a.N <= 0) return hipSuccess;
    if (stream_gemm_eligible(a)) return launch_grouped_gemm_stream(a, stream);
    switch (a.dtype) {
        case 0: return launch_t<F32>(a, stream);
        case 1: return launch_t<BF16>(a, stream);
        default: return launch_t<F16>(a, stream);
    }
}

}  // namespace moe
