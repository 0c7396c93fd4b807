// Internal launcher interface between the C-ABI translation unit and the kernel
// translation units.  Every launcher enqueues on `stream` and returns the
// hipGetLastError() of its launches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

// Grouped tile GEMM: for each group g (an expert, or the single gate "group")
//   C[g][r][n] = epilogue( sum_k A[g][r][k] * B[g][k][n] + bias[g][n] ),  r < rows(g)
// rows(g) = rows_fixed if rows_dev == nullptr, else min(rows_dev[g], rows_cap).
// B is [K][N] row-major per group ("NN"), or, when b_is_nk, [N][K] row-major
// (K contiguous).  Accumulation is fp32.
struct GemmArgs {
    const void* A; long long a_group_stride; int lda;       // elements
    // optional gather: row r of group g is A[a_row_index[g * a_index_stride + r]] (a_group_stride unused);
    // entries of live rows are valid row numbers of A
    const int32_t* a_row_index; long long a_index_stride;
    long long a_rows_total;                                 // rows of A reachable from one group's base
    const void* B; long long b_group_stride; int ldb;
    void* C; long long c_group_stride; int ldc;
    const void* bias; long long bias_group_stride;          // nullptr = none
    const int32_t* rows_dev; int rows_fixed; int rows_cap;
    // optional scratch block written by launch_ffn_units for the same rows_dev / rows_cap / groups / max_rows
    // (list of live units and completion counters); the weight-streaming kernels need it
    int32_t* units;
    // fp32 storage only, optional: scratch of f32_partials_bytes() for the sums of tiles that two or more workgroups
    // share (units is then the list written by launch_f32_units)
    float* partials;
    int groups; int max_rows;                               // grid extent in rows
    int N; int K;
    int act;                                                // moe_act, applied after the bias
    int dtype;                                              // storage of A, B (and of C, bias unless c_f32)
    bool b_is_nk;
    bool c_f32;                                             // C and bias are fp32 (gate logits)
};
hipError_t launch_grouped_gemm(const GemmArgs& a, hipStream_t stream);

// Kernels that use more than 64 KB of LDS have that limit raised per device before their first launch there;
// the launchers do it on first use, these do it for every instantiation at once (moe_init).
hipError_t prepare_grouped_gemm();
hipError_t prepare_grouped_gemm_stream();
hipError_t prepare_gate_fused();

// compute units of the current device (256 on MI355X)
int device_cu_count();

// Weight-streaming variant for the 16-bit expert FFN tasks (direct-to-LDS, deep prefetch);
// launch_grouped_gemm routes eligible shapes to it.
bool stream_gemm_eligible(const GemmArgs& a);
// the part of the eligibility that depends on the shape alone
bool stream_gemm_shape_ok(int dtype, int N, int K, int lda, int ldb, int ldc, long long a_rows_total);
hipError_t launch_grouped_gemm_stream(const GemmArgs& a, hipStream_t stream);
// Scratch block of the streaming kernels, written by launch_ffn_units for the same rows_dev / rows_cap / groups /
// max_rows: for each of the two row-tile sizes (256 and 128 rows) a fault word, the number of live (group, row
// tile) units, their list in order of group, and one completion counter per unit.  ffn_units_ints() ints;
// GemmArgs::units points at the block.
size_t ffn_units_ints(int groups, int max_rows);
hipError_t launch_ffn_units(const int32_t* rows_dev, int rows_cap, int groups, int max_rows, int32_t* units,
                            hipStream_t stream);
// Both FFN GEMMs in one persistent launch: a unit's second-GEMM tasks start when all its first-GEMM tiles are
// stored (g2.A is g1.C).  Eligible when both GEMMs are and they share rows, groups and units.
// never_met: the dependency waits get a target no counter reaches and a poll limit of 16, so that every
// second-GEMM task gives up at once and the fault word is set (exercises the give-up path; y is then garbage).
bool ffn_fused_eligible(const GemmArgs& g1, const GemmArgs& g2);
hipError_t launch_ffn_stream_fused(const GemmArgs& g1, const GemmArgs& g2, bool never_met, hipStream_t stream);
// Offsets (in ints) of the scratch block's two fault words (equal when there is no large-tile list).
void ffn_units_fault_words(int groups, int max_rows, long long* first, long long* second);

// fp32 expert FFN tasks over the live work only: persistent workgroups that each take an equal span of the K-tiles of
// all live 64-row tiles (gemm_f32.hip); launch_grouped_gemm routes eligible calls to it.  GemmArgs::units is the list
// written by launch_f32_units (f32_units_ints() ints) for the same rows_dev / rows_cap / groups / max_rows.
bool f32_stream_eligible(const GemmArgs& a);
hipError_t launch_gemm_f32_stream(const GemmArgs& a, hipStream_t stream);
size_t f32_units_ints(int groups, int max_rows);
size_t f32_partials_bytes(int groups, int max_rows, int H, int I);   // shared by the H -> I and the I -> H GEMM
hipError_t launch_f32_units(const int32_t* rows_dev, int rows_cap, int groups, int max_rows, int32_t* units, hipStream_t stream);
hipError_t prepare_gemm_f32();

// WgT[n][h] = Wg[h][n] for n < E, zero rows for E <= n < E_pad.
hipError_t launch_transpose_pad(const void* Wg, void* WgT, int H, int E, int E_pad, int dtype,
                                hipStream_t stream);

// Fused gate for 16-bit storage: logits = x Wg (+ gate_bias) in fp32, top-k experts and combine weights,
// one kernel; Wg is read as stored ([H][E]).  gate_fused_eligible tells whether the shape is covered.
bool gate_fused_eligible(int T, int H, int E, int k, int dtype);
// route_counts (optional): [ceil(T / 64)][E] picks per expert among each workgroup's 64 tokens, the first step
// of the slot assignment (launch_route with counts_ready).
hipError_t launch_gate_fused(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k,
                             int dtype, float* logits, int32_t* topk_expert, float* topk_weight,
                             int32_t* route_counts, hipStream_t stream);

// Top-k selection and combine weights from fp32 logits.
hipError_t launch_topk(const float* logits, int T, int E, int k, int32_t* topk_expert,
                       float* topk_weight, hipStream_t stream);

// Token-order slot assignment.  The pairs are cut into chunks of route_chunk_tokens() tokens; `counts` is
// scratch of route_chunks(T) * E ints.  With counts_ready the per-chunk expert counts are already there (the
// fused gate wrote them).  With ffn_units != nullptr the last launch also builds the FFN kernels' unit list
// for rows_cap = max_rows = C (see launch_ffn_units), or with f32_units the fp32 kernel's list (launch_f32_units).
int route_chunk_tokens();
int route_chunks(int T);
// choice_major: the pairs are taken in the order (choice rank, token) instead of (token, choice rank).
hipError_t launch_route(const int32_t* topk_expert, const float* topk_weight, int T, int E, int k, int C,
                        bool choice_major, int32_t* counts, bool counts_ready, int32_t* slot, int32_t* expert_demand,
                        int32_t* slot_token, float* slot_weight, int32_t* ffn_units, bool f32_units, hipStream_t stream);

// xe[e][slot][:] = x[token][:] for every kept (token, choice).
hipError_t launch_pack(const void* x, const int32_t* topk_expert, const int32_t* slot, int T, int H,
                       int k, int E, int C, int C_pad, int dtype, void* xe, hipStream_t stream);

// out[t][:] = sum_j w[t][j] * y[e][slot][:] over kept choices, fp32.
hipError_t launch_combine(const void* y, const int32_t* topk_expert, const float* topk_weight,
                          const int32_t* slot, int T, int H, int k, int E, int C, int C_pad,
                          int dtype, void* out, hipStream_t stream);

// The whole layer in one persistent launch (layer_fused.hip): gate, slot assignment, both FFN GEMMs and the combine,
// separated by device-wide barriers.  16-bit storage, E <= 128, shapes that the fused gate and the weight-streaming
// FFN kernels take, token-order drop priority.  g1 / g2 describe the FFN GEMMs as for launch_ffn_stream_fused
// (g1.A = x gathered through slot_token, g2.C = y); counts = route_chunks(T) * E ints.
bool layer_fused_eligible(int T, int H, int I, int ldh, int E, int k, int C_pad, int dtype);
hipError_t launch_layer_fused(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k, int C, int C_pad,
                              int dtype, float* logits, int32_t* topk_expert, float* topk_weight, int32_t* counts, int32_t* slot,
                              int32_t* expert_demand, int32_t* slot_token, float* slot_weight, const GemmArgs& g1, const GemmArgs& g2,
                              void* out, hipStream_t stream);
hipError_t prepare_layer_fused();
// zero the barrier words of the single-launch layer on the current device (after a launch that gave up)
hipError_t reset_layer_sync(hipStream_t stream);
// Workgroup 0's stage times (ms) of the last single-launch layer on the current device; synchronises the stream.
hipError_t layer_stage_ms(double* ms, int n, hipStream_t stream);

// ---- backward pass helpers (backward.hip); buffers per expert have C_pad rows ----------------------------
// rows[0 .. E) = first, rows[E .. 2 E) = second
hipError_t launch_bwd_fill_rows(int32_t* rows, int E, int first, int second, hipStream_t s);
// xe[e, s, :] = x[token] and gy[e, s, :] = weight * dout[token] for live slots, zeros for empty ones (s < C_pad)
hipError_t launch_bwd_gather(const void* x, const void* dout, const int32_t* slot_token, const float* slot_weight, int H, int E,
                             int C, int C_pad, int dtype, void* xe, void* gy, hipStream_t s);
// over [E, C_pad, I]: out = phi(a), or with grad: out = g_in * phi'(a); rows beyond an expert's live rows give 0
hipError_t launch_bwd_act(const void* a, const void* g_in, const int32_t* expert_demand, int E, int C, int C_pad, int I, int act,
                          int dtype, bool grad, void* out, hipStream_t s);
// dl[T, k] (fp32) and dL[T_pad, ld] (storage type, dense; rows at and beyond T zero): gradient with respect to the
// selected gate logits (k <= 64)
hipError_t launch_bwd_gate(const void* dout, const void* y, const int32_t* topk_expert, const float* topk_weight, const int32_t* slot,
                           int T, int T_pad, int H, int k, int E, int C, int C_pad, int ld, int dtype, float* dl, void* dL, hipStream_t s);
// out[i] = sum over g < slices of part[g * n + i], in ascending g (n a multiple of 4, 16-byte aligned buffers)
hipError_t launch_bwd_sum_slices(const float* part, int slices, long long n, float* out, hipStream_t s);
// out[g][c][r] = in[g][r][c], r < R, c < Cc; rows of out have ld_out entries, zero at and beyond R
hipError_t launch_bwd_transpose(const void* in, void* out, int groups, int R, int Cc, int ld_out, int dtype, hipStream_t s);
// out[e][c] = sum over live rows of in[e][r][c] (fp32)
hipError_t launch_bwd_colsum(const void* in, const int32_t* expert_demand, int E, int C, int C_pad, int cols, int dtype, float* out,
                             hipStream_t s);
hipError_t launch_bwd_gate_bias(const int32_t* topk_expert, const float* dl, int T, int k, int E, float* dgate_bias, hipStream_t s);
// dx[t, :] = sum of the kept choices' rows of dxe + sum over choices of dl * WgT[expert, :]
hipError_t launch_bwd_dx(const void* dxe, const void* WgT, const int32_t* topk_expert, const int32_t* slot, const float* dl, int T, int H,
                         int k, int E, int C, int C_pad, int dtype, float* dx, hipStream_t s);

}  // namespace moe
