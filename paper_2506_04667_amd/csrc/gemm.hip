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
#include "gemm_body.h"

namespace moe {
namespace {

constexpr int kXcds = 8;

template <class S, bool NT, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(WM * WN * 64) void grouped_gemm_kernel(GemmArgs a) {
    using C = Cfg<S, NT, WM, WN, TM, TN>;
    constexpr int BM = C::BM, BN = C::BN;
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

    gemm_tile<S, NT, WM, WN, TM, TN>(a, smem, grp, row0, n0, rows, 0, (a.K + C::BK - 1) / C::BK, nullptr);
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
    if (f32_stream_eligible(a)) return launch_gemm_f32_stream(a, stream);
    switch (a.dtype) {
        case 0: return launch_t<F32>(a, stream);
        case 1: return launch_t<BF16>(a, stream);
        default: return launch_t<F16>(a, stream);
    }
}

}  // namespace moe
