// Tile body of the grouped GEMM on CDNA4 matrix cores (see gemm.hip for the layouts), shared by the kernel that
// computes one whole tile per workgroup and by the fp32 kernel whose persistent workgroups each take an equal
// span of the K-tiles of all live tiles.
#pragma once
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

// One workgroup of WM x WN wavefronts: K-tiles [kt0, kt1) of the BM x BN tile at (row0, n0) of group grp, whose live
// rows are `rows`.  partial == nullptr: bias, activation, conversion and the store to C.  Otherwise the raw fp32
// sums go to partial[BM][BN] (row-major) for a later pass to add up.  Ends with a workgroup barrier after the last
// LDS read, so the caller may start another tile at once.
template <class S, bool NT, int WM, int WN, int TM, int TN>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, unsigned char* smem, int grp, int row0, int n0, int rows, int kt0, int kt1,
                                          float* __restrict__ partial) {
    using C = Cfg<S, NT, WM, WN, TM, TN>;
    typedef typename S::store_t elem;
    constexpr bool k16 = C::k16;
    constexpr int VEC = C::VEC, BK = C::BK, BM = C::BM, BN = C::BN, THREADS = C::THREADS;

    // the operands are device (global) memory: said explicitly, so that a caller that is not a kernel (its GemmArgs then
    // come from memory and carry no address space) still gets global loads, which do not count against LDS waits
    typedef const __attribute__((address_space(1))) elem* gelem;
    typedef const __attribute__((address_space(1))) u32x4* gvec;
    const gelem A = (gelem)(const elem*)a.A + (a.a_row_index ? (size_t)0 : (size_t)grp * a.a_group_stride);
    const gelem B = (gelem)(const elem*)a.B + (size_t)grp * a.b_group_stride;
    const int K = a.K, N = a.N;
    const int lda = a.lda, ldb = a.ldb;                  // locals: `a` may live in memory that stores could alias

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
            ra[i] = ok ? *(gvec)(A + (size_t)a_grow[i] * lda + k0 + kc) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) {
            const int c = tid + i * THREADS;
            if (NT) {
                const int r = c >> 3, kc = (c & 7) * VEC;
                const bool ok = (n0 + r < N) && (k0 + kc < K);
                rb[i] = ok ? *(gvec)(B + (size_t)(n0 + r) * ldb + k0 + kc) : u32x4{0, 0, 0, 0};
            } else {
                const int r = c / C::B_CPR, nc = (c % C::B_CPR) * VEC;
                const bool ok = (k0 + r < K) && (n0 + nc < N);
                rb[i] = ok ? *(gvec)(B + (size_t)(k0 + r) * ldb + n0 + nc) : u32x4{0, 0, 0, 0};
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
    // the 32-row MFMA tiles of a workgroup tile are dealt to the WM wavefront rows in turn (tile tm of wavefront row
    // wm is number tm * WM + wm), so that a tile with few live rows still spreads them over all wavefronts
    const int a_row = wm * 32 + l32;
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
                    af[tm] = *(const s16x8*)(sa + (a_row + tm * WM * 32) * 128 + (a_chunk << 4));
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
        }
    };
    // fp32: the same slice with only the first LT of the wavefront's TM 32-row MFMA tiles (the others lie beyond the
    // group's live rows: their sums are never stored, so their MFMAs and operand reads are left out)
    auto compute32 = [&](int stage, auto lt) {
        constexpr int LT = decltype(lt)::value;
        const unsigned char* sa = smem + stage * C::STAGE_BYTES;
        const unsigned char* sb = sa + C::A_BYTES;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {                 // 8 k per step: lanes 0-31 take k..k+3, lanes 32-63 k+4..k+7
            f32x4 af[LT];
            float bfr[TN][4];
            const int a_chunk = ((ks << 1) | g2) ^ a_sw;
#pragma unroll
            for (int tm = 0; tm < LT; ++tm)
                af[tm] = *(const f32x4*)(sa + (a_row + tm * WM * 32) * 128 + (a_chunk << 4));
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
                for (int tm = 0; tm < LT; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[tm][j], bfr[tn][j], acc[tm][tn], 0, 0, 0);
        }
    };
    // live 32-row MFMA tiles of this wavefront (uniform over the wavefront)
    const int live_tm = min(max(((rows - row0 + 31) / 32 - wm + WM - 1) / WM, 0), TM);
    auto compute_tile = [&](int stage) {
        if constexpr (k16) {
            compute(stage, 0, 4);
        } else {
            static_assert(TM <= 4, "one case per count of live MFMA row tiles");
            switch (live_tm) {
                case 0: break;
                case 1: compute32(stage, std::integral_constant<int, 1>{}); break;
                case 2: compute32(stage, std::integral_constant<int, (TM >= 2 ? 2 : TM)>{}); break;
                case 3: compute32(stage, std::integral_constant<int, (TM >= 3 ? 3 : TM)>{}); break;
                default: compute32(stage, std::integral_constant<int, TM>{}); break;
            }
        }
    };

    const int nk = kt1 - kt0;
    load_global(kt0 * BK);
    store_lds(0);
    if (nk > 1) load_global((kt0 + 1) * BK);
    __syncthreads();
    for (int t = 0; t < nk; ++t) {
        const int cur = t & 1;
        if (t + 1 < nk) {
            store_lds(cur ^ 1);                          // K-tile t+1; that stage was last read before the previous barrier
            if (t + 2 < nk) load_global((kt0 + t + 2) * BK);   // a whole K-tile of MFMAs to arrive
        }
        compute_tile(cur);
        __syncthreads();
    }

    if (partial) {                                       // raw sums of a K-slice, [BM][BN] row-major
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int r = (tm * WM + wm) * 32 + (q >> 2) * 8 + g2 * 4 + (q & 3);
                    partial[(size_t)r * BN + (wn * TN + tn) * 32 + l32] = acc[tm][tn][q];
                }
        return;
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
                const int row = row0 + (tm * WM + wm) * 32 + (q >> 2) * 8 + g2 * 4 + (q & 3);
                if (row >= rows) continue;
                const float v = apply_act(acc[tm][tn][q] + bias, a.act);
                const size_t ci = c_base + (size_t)row * a.ldc + col;
                if (a.c_f32) ((float*)a.C)[ci] = v;
                else store_from_float<S>(a.C, ci, v);
            }
        }
    }
}

}  // namespace
}  // namespace moe
