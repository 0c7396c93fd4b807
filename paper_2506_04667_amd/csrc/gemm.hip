// Grouped tile GEMM on CDNA4 matrix cores: the two FFN tasks of every expert
// (C1 <- phi1(A B1 + D1), C2 <- C1 B2 + D2, Sec. 3.1 task abstraction) and the gate
// projection share this kernel.  One workgroup computes one (group, row tile,
// column tile) task; tasks whose row tile lies beyond the group's live rows exit at
// once, so only ceil(rows/bM) row tiles per expert are ever computed (the in-place
// padding idea of Sec. 3.2.1).
//
// Tile: 128 x 128 per workgroup of 4 wavefronts (2 x 2), 64 x 64 per wavefront as
// 2 x 2 MFMA tiles of 32 x 32.  16-bit storage uses v_mfma_f32_32x32x16_{bf16,f16}
// with K-tile 64; fp32 uses v_mfma_f32_32x32x2_f32 with K-tile 32.  Operands are
// staged through LDS.  A weight tile stored [k][n] (n contiguous) is read in MFMA
// operand order (k contiguous per lane) with the LDS transpose read
// ds_read_b64_tr_b16: within 16 lanes, lane i receives, as element j, element
// (i % 4) of the 8-byte row addressed by lane 4 j + i / 4.
#include "common.h"
#include "kernels.h"
#include <type_traits>

namespace moe {
namespace {

constexpr int BM = 128, BN = 128;

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

template <class S, bool NT>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs a) {
    typedef typename S::store_t elem;
    constexpr bool k16 = (S::kBytes == 2);
    constexpr int VEC = S::kVec;            // elements per 16-byte chunk
    constexpr int BK = 8 * VEC;             // 64 (16-bit) or 32 (fp32)
    constexpr int LDA = BK + VEC;           // 144-byte pitch: conflict-free 16-byte row reads
    constexpr int LDB = NT ? LDA : BN + (k16 ? 32 : 8);
    constexpr int B_ROWS = NT ? BN : BK;
    constexpr int B_CPR = NT ? 8 : BN / VEC;  // chunks per B tile row

    __shared__ __attribute__((aligned(16))) elem sA[BM * LDA];
    __shared__ __attribute__((aligned(16))) elem sB[B_ROWS * LDB];

    const int grp = blockIdx.z;
    const int row0 = blockIdx.y * BM;
    const int n0 = blockIdx.x * BN;
    const int rows = a.rows_dev ? min(a.rows_dev[grp], a.rows_cap) : a.rows_fixed;
    if (row0 >= rows) return;

    const elem* A = (const elem*)a.A + (size_t)grp * a.a_group_stride;
    const elem* B = (const elem*)a.B + (size_t)grp * a.b_group_stride;
    const int K = a.K, N = a.N;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, g2 = lane >> 5;

    u32x4 ra[4], rb[4];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            const int r = c >> 3, kc = (c & 7) * VEC;
            const bool ok = (row0 + r < rows) && (k0 + kc < K);
            ra[i] = ok ? *(const u32x4*)(A + (size_t)(row0 + r) * a.lda + k0 + kc) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            if (NT) {
                const int r = c >> 3, kc = (c & 7) * VEC;
                const bool ok = (n0 + r < N) && (k0 + kc < K);
                rb[i] = ok ? *(const u32x4*)(B + (size_t)(n0 + r) * a.ldb + k0 + kc) : u32x4{0, 0, 0, 0};
            } else {
                const int r = c / B_CPR, nc = (c % B_CPR) * VEC;
                const bool ok = (k0 + r < K) && (n0 + nc < N);
                rb[i] = ok ? *(const u32x4*)(B + (size_t)(k0 + r) * a.ldb + n0 + nc) : u32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            *(u32x4*)(sA + (c >> 3) * LDA + (c & 7) * VEC) = ra[i];
            if (NT) *(u32x4*)(sB + (c >> 3) * LDB + (c & 7) * VEC) = rb[i];
            else *(u32x4*)(sB + (c / B_CPR) * LDB + (c % B_CPR) * VEC) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

    load_global(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();              // previous tile fully consumed
        store_lds();
        __syncthreads();
        if (k0 + BK < K) load_global(k0 + BK);

        if constexpr (k16) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                s16x8 af[2], bf[2];
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
                    af[tm] = *(const s16x8*)(sA + (wm * 64 + tm * 32 + l32) * LDA + kk + g2 * 8);
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) {
                    if (NT) {
                        bf[tn] = *(const s16x8*)(sB + (wn * 64 + tn * 32 + l32) * LDB + kk + g2 * 8);
                    } else {
                        // lanes 0-15 / 16-31: columns 0-15 / 16-31 of the 32-wide tile; lanes 32-63: k + 8
                        const int L = lane & 15, nb = (lane >> 4) & 1;
                        const elem* p = sB + (kk + g2 * 8 + (L >> 2)) * LDB + wn * 64 + tn * 32 + nb * 16 + (L & 3) * 4;
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LDB));
                        bf[tn] = s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    }
                }
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn) acc[tm][tn] = Mma<typename std::conditional<k16, S, BF16>::type>::run(af[tm], bf[tn], acc[tm][tn]);
            }
        } else {
            const float* fA = (const float*)sA;
            const float* fB = (const float*)sB;
#pragma unroll
            for (int kk = 0; kk < BK; kk += 8) {
                // lanes 0-31 take k = kk..kk+3, lanes 32-63 take k = kk+4..kk+7, one k per MFMA
                f32x4 af[2];
                float bfr[2][4];
#pragma unroll
                for (int tm = 0; tm < 2; ++tm)
                    af[tm] = *(const f32x4*)(fA + (wm * 64 + tm * 32 + l32) * LDA + kk + g2 * 4);
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) {
                    if (NT) {
                        f32x4 t = *(const f32x4*)(fB + (wn * 64 + tn * 32 + l32) * LDB + kk + g2 * 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) bfr[tn][j] = t[j];
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) bfr[tn][j] = fB[(kk + g2 * 4 + j) * LDB + wn * 64 + tn * 32 + l32];
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                        for (int tn = 0; tn < 2; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[tm][j], bfr[tn][j], acc[tm][tn], 0, 0, 0);
            }
        }
    }

    // epilogue on the accumulator registers: bias, activation, conversion, store
    const size_t c_base = (size_t)grp * a.c_group_stride;
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
        const int col = n0 + wn * 64 + tn * 32 + l32;
        if (col >= N) continue;
        float bias = 0.0f;
        if (a.bias) {
            const size_t bi = (size_t)grp * a.bias_group_stride + col;
            bias = a.c_f32 ? ((const float*)a.bias)[bi] : load_as_float<S>(a.bias, bi);
        }
#pragma unroll
        for (int tm = 0; tm < 2; ++tm) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int row = row0 + wm * 64 + tm * 32 + (q >> 2) * 8 + g2 * 4 + (q & 3);
                if (row >= rows) continue;
                const float v = apply_act(acc[tm][tn][q] + bias, a.act);
                const size_t ci = c_base + (size_t)row * a.ldc + col;
                if (a.c_f32) ((float*)a.C)[ci] = v;
                else store_from_float<S>(a.C, ci, v);
            }
        }
    }
}

template <class S>
hipError_t launch_t(const GemmArgs& a, hipStream_t stream) {
    dim3 grid((a.N + BN - 1) / BN, (a.max_rows + BM - 1) / BM, a.groups);
    if (a.b_is_nk) hipLaunchKernelGGL((grouped_gemm_kernel<S, true>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((grouped_gemm_kernel<S, false>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_grouped_gemm(const GemmArgs& a, hipStream_t stream) {
    if (a.groups <= 0 || a.max_rows <= 0 || a.N <= 0) return hipSuccess;
    switch (a.dtype) {
        case 0: return launch_t<F32>(a, stream);
        case 1: return launch_t<BF16>(a, stream);
        default: return launch_t<F16>(a, stream);
    }
}

}  // namespace moe
