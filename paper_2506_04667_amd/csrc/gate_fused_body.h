// Fused gate ("FusedGate" of Alg. 1), all storage types: one kernel computes the gate
// logits x Wg (+ bias) on the matrix cores, writes them, and selects each token's top-k
// experts with their combine weights (Eqs. "combine 1/2": softmax over the k selected
// logits) -- no transposed copy of Wg, no second pass over the logits in HBM.
//
// One workgroup (8 wavefronts) owns 64 tokens and all E <= 256 experts.  The token rows
// stream from HBM exactly once; Wg (H x E, a few hundred KB) is re-read by every workgroup
// from L2.  Both go straight to LDS (global_load_lds_dwordx4) through a ring of K-tiles of
// 128 bytes per row (64 elements, or 32 in fp32), several tiles ahead, with explicit waits.
// In 16-bit storage the LDS layouts and swizzles are those of the
// streaming FFN kernel: token rows 128 B per K-tile, chunk c of row r at c ^ ((r >> 1) & 7);
// Wg tile [k][n], chunk c of row k at c ^ ((k & 3) << 2), read in MFMA operand order with
// ds_read_b64_tr_b16.  The MFMAs take the Wg fragment first, so a lane's accumulators hold
// runs of four consecutive experts of ONE token.
//
// Epilogue: logits (+ bias) go to an fp32 LDS tile (it reuses the ring), from there to HBM
// with full-line stores, and the selection reads the same tile: 16 lanes per token, each
// holding a sixteenth of the row in registers; k rounds of "largest remaining logit, smaller expert
// index on equal values" compared as floats (so -0.0 and +0.0 tie), where "remaining" means
// strictly after the previous pick in that order.  The 16 lanes agree on each pick through
// DPP exchanges; the unnormalised weights wait in LDS until the softmax denominator is known.
#pragma once
#include "common.h"
#include "kernels.h"
#include "lds_copy.h"

namespace moe {
namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int G_BM = 64, G_THREADS = 512, G_WAVES = G_THREADS / 64;
constexpr int G_A_STAGE = G_BM * 128;                    // 64 token rows x 128 bytes of k
constexpr bool kRotateK = true;                          // workgroups start their K loops at different K-tiles

// S: storage type; BN: experts covered (64 for fp32 only, 128, 256).  A K-tile is 128 bytes of k per token
// row: 64 elements in 16-bit storage, 32 in fp32.
template <class S, int BN_>
struct GateCfg {
    static constexpr int BN = BN_;
    static constexpr int EL = S::kBytes, VEC = 16 / EL;  // bytes per element; elements per 16-byte chunk
    static constexpr int KT = 128 / EL;                  // k per K-tile
    static constexpr int PITCH = BN * EL;                // bytes per k-row of the Wg tile
    static constexpr int B_STAGE = KT * PITCH;
    static constexpr int STAGE = G_A_STAGE + B_STAGE;    // 16, 24 or 40 KB
    static constexpr int STAGES = 4;                     // measured: 4 stages beat 3, 5 and 6 (19.5 against 21.5-22.4 us at T = 16K, E = 128, bf16)
    static constexpr int LDS_BYTES = STAGES * STAGE;     // at most 160 KB
    static constexpr int B_COPIES = B_STAGE / 1024 / G_WAVES;  // 1 KB copies per wavefront per K-tile
    static constexpr int COPIES = 1 + B_COPIES;
    static constexpr int TN = BN / 64;                   // 32-expert MFMA tiles per wavefront
    static constexpr int LP = BN + 4;                    // row pitch (floats) of the logits tile
    static_assert(PITCH >= 256, "the swizzles of the Wg tile move chunks by up to 12 or 8 places");
    static_assert(G_BM * (LP + BN) * 4 + BN * 4 <= LDS_BYTES,
                  "logits tile, k <= BN weights per token and the expert histogram must fit in the ring they reuse");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");
};

template <class S> struct GateMma;
template <> struct GateMma<BF16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct GateMma<F16> {
    static __device__ __forceinline__ f32x16 run(s16x8 a, s16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// Candidate (value, expert) of the lane selected by a DPP pattern inside a row of 16 lanes; the better of the
// two by (larger value, then smaller expert index) stays.  "No candidate" is (-inf, INT_MAX) and loses to any.
template <int CTRL>
__device__ __forceinline__ void merge_best(float& bv, int& bi) {
    const float ov = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, bv), CTRL, 0xf, 0xf, true));
    const int oi = __builtin_amdgcn_update_dpp(0, bi, CTRL, 0xf, 0xf, true);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
}

// The gate for the 64 tokens of tile number `tile` (tokens 64 tile .. 64 tile + 63), by all G_THREADS threads of a
// workgroup that has GateCfg<S, BN_>::LDS_BYTES of dynamic LDS.  route_counts (optional) receives row `tile`.
template <class S, int BN_>
__device__ __forceinline__ void gate_fused_tile(const unsigned char* __restrict__ x, const unsigned char* __restrict__ Wg,
                                                const float* __restrict__ gate_bias, int T, int H, int E, int k,
                                                float* __restrict__ logits, int32_t* __restrict__ topk_expert,
                                                float* __restrict__ topk_weight, int32_t* __restrict__ route_counts, int tile) {
    using C = GateCfg<S, BN_>;
    constexpr int BN = C::BN, PITCH = C::PITCH, STAGE = C::STAGE, D = C::STAGES, TN = C::TN, LP = C::LP;
    constexpr int EL = C::EL, VEC = C::VEC, KT = C::KT;
    constexpr bool k16 = EL == 2;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = uniform(tid >> 6);
    // two groups of 2 x 2 wavefronts (32 tokens x BN / 2 experts each); group kg multiplies k-steps 2 kg and
    // 2 kg + 1 of every K-tile, and the two partial sums meet in LDS at the end: two wavefronts per SIMD hide
    // each other's LDS latency and barrier waits without reading any operand twice more
    const int kg = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;
    const int l32 = lane & 31, g2 = lane >> 5;
    const int row0 = tile * G_BM;

    // ---- this wavefront's 1 KB copies per K-tile: 1 of token rows (8 rows x 128 B), B_COPIES of Wg ----
    // Workgroup b starts its K loop at K-tile b % nk and wraps around: at any moment the workgroups read
    // different 128-byte columns of their token rows (and different tiles of Wg), so the requests in flight
    // spread over all memory channels instead of marching down one 4 KB-strided column band together.  The
    // order in which a workgroup accumulates its K-tiles depends on its number only: results are the same
    // from run to run.
    const int nk = H / KT;
    const int k_first = kRotateK ? (int)((unsigned)tile % (unsigned)nk) : 0;
    const size_t b_step = (size_t)KT * E * EL;
    const unsigned char* const a_row0 = uniform(x + (size_t)row0 * H * EL);
    const unsigned char* a_base = uniform(a_row0 + (size_t)k_first * 128);
    const unsigned char* b_base = uniform(Wg + (size_t)k_first * b_step);
    int k_issue = k_first;                              // K-tile the next request fetches
    uint32_t a_off, b_off[C::B_COPIES];
    {
        const int r = wave * 8 + (lane >> 3), p = lane & 7;
        const int c = p ^ ((r >> 1) & 7);
        const int rr = min(row0 + r, T - 1) - row0;     // rows beyond T repeat the last token (never stored)
        a_off = (uint32_t)rr * (uint32_t)(H * EL) + c * 16;
    }
    constexpr int CPR = PITCH / 16;                     // 16-byte chunks per k-row
#pragma unroll
    for (int j = 0; j < C::B_COPIES; ++j) {
        const int kk = (wave * C::B_COPIES + j) * (64 / CPR) + lane / CPR, p = lane % CPR;
        const int c = p ^ (k16 ? ((kk & 3) << 2) : (((kk >> 2) & 1) << 3));
        const int n = min(c * VEC, E - VEC);            // columns beyond E repeat the last experts (masked later)
        b_off[j] = (uint32_t)kk * (uint32_t)(E * EL) + n * EL;
    }
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    auto issue = [&](int t) __attribute__((always_inline)) {
        const uint32_t d = lds_base + (t % D) * STAGE;
        copy_to_lds(a_base, a_off, d + wave * 1024);
#pragma unroll
        for (int j = 0; j < C::B_COPIES; ++j)
            copy_to_lds(b_base, b_off[j], d + G_A_STAGE + (wave * C::B_COPIES + j) * 1024);
        a_base += 128;
        b_base += b_step;
        if (++k_issue == nk) {
            k_issue = 0;
            a_base = a_row0;
            b_base = uniform(Wg);
        }
    };

    // ---- per-lane LDS read offsets ----
    const int a_row = wm * 32 + l32;
    const int a_sw = (a_row >> 1) & 7;
    const int L = lane & 15, nb16 = (lane >> 4) & 1;
    const int bk = g2 * 8 + (L >> 2);                   // k of the first transpose read; the second is k + 4
    int a_rd[2], b_rd[TN];                              // this group's two k-steps: 2 kg, 2 kg + 1
#pragma unroll
    for (int i = 0; i < 2; ++i) a_rd[i] = a_row * 128 + (((((2 * kg + i) << 1) | g2) ^ a_sw) << 4);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        if (k16) {
            const int chunk = (wn * TN + tn) * 4 + nb16 * 2 + ((L & 3) >> 1);
            b_rd[tn] = G_A_STAGE + (2 * kg * 16 + bk) * PITCH + ((chunk ^ ((bk & 3) << 2)) << 4) + (L & 1) * 8;
        } else {
            // fp32: a k-step is 8 wide; the lane's 16-byte activation chunk holds k = 8 ks + 4 g2 + 0..3, and the
            // matching weights are four 4-byte reads at those k, column n (v_mfma_f32_32x32x2 takes one k per
            // half-wavefront; which k of the tile that is does not matter as long as both operands agree)
            const int n = (wn * TN + tn) * 32 + l32;
            b_rd[tn] = G_A_STAGE + (2 * kg * 8 + 4 * g2) * PITCH + (((n >> 2) ^ (g2 << 3)) << 4) + (n & 3) * 4;
        }
    }

    f32x16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;

    // ---- main loop ----
    // The operands of a K-tile are read from LDS into registers one iteration ahead, so the reads' latency
    // hides behind the MFMAs of the tile before.  All D stages are requested up front; in iteration u the
    // wavefront waits for tile u + 1 (its operands are read next), meets the others (every wavefront then holds
    // tile u in registers, so stage u % D is free), requests tile u + D into that stage, starts the reads of
    // tile u + 1 and multiplies tile u.
    struct Ops {                                        // one wavefront's operands of one K-tile (its two k-steps)
        u32x4 x[2];
        u32x4 w[2][TN];                                 // 16-bit: one MFMA operand; fp32: four k of column n
    };
    auto load_ops = [&](int t, Ops& o) __attribute__((always_inline)) {
        const unsigned char* st = smem + (t % D) * STAGE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            o.x[ks] = *(const u32x4*)(st + a_rd[ks]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                if constexpr (k16) {
                    const unsigned char* pw = st + b_rd[tn] + ks * 16 * PITCH;
                    const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)pw));
                    const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(pw + 4 * PITCH)));
                    o.w[ks][tn] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) o.w[ks][tn][j] = *(const uint32_t*)(st + b_rd[tn] + (ks * 8 + j) * PITCH);
                }
            }
        }
    };
    auto mma_ops = [&](const Ops& o) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if constexpr (k16) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tn] = GateMma<S>::run(__builtin_bit_cast(s16x8, o.w[ks][tn]), __builtin_bit_cast(s16x8, o.x[ks]), acc[tn]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const uint32_t wb = o.w[ks][tn][j], xb = o.x[ks][j];   // copy out first: bit_cast of a vector element reads element 0
                        acc[tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, wb), __builtin_bit_cast(float, xb), acc[tn], 0, 0, 0);
                    }
            }
        }
    };
    // One iteration: `cur` holds tile u, `nxt` receives tile u + 1.
    auto step = [&](int u, const Ops& cur, Ops& nxt) __attribute__((always_inline)) {
        if (u + 1 < nk) {
            // a wavefront's copies complete in issue order: with tiles up to u + D - 1 requested, "tile u + 1 has
            // landed" leaves the COPIES * (D - 2) newest in flight; near the end everything outstanding is waited for
            if (u + D - 1 < nk) wait_copies_and_barrier<C::COPIES * (D - 2)>();
            else wait_copies_and_barrier<0>();
            if (u + D < nk) issue(u + D);
            load_ops(u + 1, nxt);
        }
        mma_ops(cur);
    };
    for (int t = 0; t < D && t < nk; ++t) issue(t);
    if (D <= nk) wait_copies_and_barrier<C::COPIES * (D - 1)>();   // tile 0 has landed
    else wait_copies_and_barrier<0>();
    Ops o0, o1;
    load_ops(0, o0);
    int u = 0;
    for (; u + 1 < nk; u += 2) {
        step(u, o0, o1);
        step(u + 1, o1, o0);
    }
    if (u < nk) step(u, o0, o1);
    wait_copies_and_barrier<0>();                       // every wavefront is done with the ring: reuse it

    // ---- logits tile [64 tokens][LP] fp32 in LDS: group 1 parks its partial sums, group 0 adds its own and
    // the bias ----
    // accumulator elements 4 qa .. 4 qa + 3 of tile tn: experts e .. e + 3 of token l32
    float* lg = (float*)smem;
#pragma unroll
    for (int pass = 1; pass >= 0; --pass) {
        if (kg == pass) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int qa = 0; qa < 4; ++qa) {
                    const int e = (wn * TN + tn) * 32 + qa * 8 + g2 * 4;
                    float* cell = lg + (wm * 32 + l32) * LP + e;
                    f32x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = acc[tn][qa * 4 + i];
                    if (pass == 0) {
                        f32x4 b = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (gate_bias && e < E) b = *(const f32x4*)(gate_bias + e);
                        const f32x4 other = *(const f32x4*)cell;
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = (v[i] + other[i]) + b[i];
                    }
                    *(f32x4*)cell = v;
                }
        }
        __syncthreads();
    }

    // ---- logits to HBM: each wavefront stores its 8 tokens, full rows ----
    constexpr int TOK = G_BM / G_WAVES;                 // tokens per wavefront from here on
    constexpr int LANES_PER_ROW = BN / 4;               // 32 or 64 lanes x 16 B
    constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
#pragma unroll
    for (int i = 0; i < TOK / ROWS_PER_PASS; ++i) {
        const int r = wave * TOK + i * ROWS_PER_PASS + lane / LANES_PER_ROW, e = (lane % LANES_PER_ROW) * 4;
        if (row0 + r < T && e < E) *(f32x4*)(logits + (size_t)(row0 + r) * E + e) = *(const f32x4*)(lg + r * LP + e);
    }

    // ---- selection: 16 lanes per token ----
    // Round j picks the largest remaining (logit, then smaller index) of the token: every lane proposes the
    // best of its own VL logits, then the 16 lanes agree through four DPP exchanges (no LDS traffic).  The
    // unnormalised weights exp(v_j - v_0) wait in LDS until the sum over the k picks is known.
    constexpr int VL = BN / 16;                          // logits per lane
    constexpr int kNone = 0x7fffffff;
    constexpr int R = TOK / 4;                           // a wavefront's tokens: 4 at a time x R independent chains
    const int s16 = lane & 15;
    float* stash = lg + G_BM * LP;                       // [64 tokens][k]
    int* hist = (int*)(lg + G_BM * (LP + BN));           // [E] picks per expert among this workgroup's tokens
    if (route_counts) {
        for (int e = tid; e < E; e += G_THREADS) hist[e] = 0;
        __syncthreads();
    }
    float vals[R][VL];
    int row[R];
#pragma unroll
    for (int c = 0; c < R; ++c) {
        row[c] = wave * TOK + c * 4 + (lane >> 4);
#pragma unroll
        for (int i = 0; i < VL / 4; ++i) {
            const f32x4 v = *(const f32x4*)(lg + row[c] * LP + i * 64 + s16 * 4);
#pragma unroll
            for (int q = 0; q < 4; ++q) vals[c][i * 4 + q] = v[q];
        }
    }
    float m[R], sum[R], last_v[R];
    int last_i[R];
#pragma unroll
    for (int c = 0; c < R; ++c) { m[c] = 0.0f; sum[c] = 0.0f; last_v[c] = 0.0f; last_i[c] = -1; }
    for (int j = 0; j < k; ++j) {
#pragma unroll
        for (int c = 0; c < R; ++c) {
            float bv = -INFINITY;
            int bi = kNone;
#pragma unroll
            for (int i = 0; i < VL; ++i) {
                const int e = (i >> 2) * 64 + s16 * 4 + (i & 3);   // ascending in i: equal values keep the earlier index
                const float v = vals[c][i];
                const bool avail = (j == 0) || (v < last_v[c]) || (v == last_v[c] && e > last_i[c]);
                const bool better = (bi == kNone) || (v > bv);
                if (e < E && avail && better) { bv = v; bi = e; }
            }
            merge_best<0xB1>(bv, bi);                   // lane ^ 1
            merge_best<0x4E>(bv, bi);                   // lane ^ 2
            merge_best<0x141>(bv, bi);                  // mirror inside 8 lanes: the other quad
            merge_best<0x140>(bv, bi);                  // mirror inside 16 lanes: the other half
            if (j == 0) m[c] = bv;
            const float p = expf(bv - m[c]);
            sum[c] += p;
            if (s16 == 0 && row0 + row[c] < T) {
                topk_expert[(size_t)(row0 + row[c]) * k + j] = bi;
                stash[row[c] * k + j] = p;
                if (route_counts && bi < E) atomicAdd(&hist[bi], 1);   // integer: the order of the additions does not matter
            }
            last_v[c] = bv;
            last_i[c] = bi;
        }
    }
    // a wavefront's LDS operations complete in order: lane 0 of a group wrote what the group's lanes read here
#pragma unroll
    for (int c = 0; c < R; ++c)
        if (row0 + row[c] < T)
            for (int j = s16; j < k; j += 16)
                topk_weight[(size_t)(row0 + row[c]) * k + j] = stash[row[c] * k + j] / sum[c];
    // first step of the slot assignment: this workgroup's tokens are one chunk of the token-order scan
    if (route_counts) {
        __syncthreads();
        for (int e = tid; e < E; e += G_THREADS) route_counts[(size_t)tile * E + e] = hist[e];
    }
}


}  // namespace
}  // namespace moe
