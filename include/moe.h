/*
 * moe.h -- C ABI of the MI355X (gfx950) forward pass of one GPU's share of a
 * capacity-bounded top-k Mixture-of-Experts layer.
 *
 * The layer follows the problem statement of the FlashMoE paper: token matrix
 * A in R^{S x H} -> output O in R^{S x H}, local expert weights X in
 * R^{E x H x D} (Alg. 1 inputs; Sec. 3 notation), a gate that yields the routing
 * table T_phi(e, c) = (token, combine weight) and the affinity scores G_phi,
 * expert FFNs (Eq. "ffn") and the expert-combine (Eqs. "combine 1/2").  Here
 * S = T tokens, D = I.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  `cfg` is a HOST pointer.  The library
 *     allocates nothing and touches only the caller's buffers and workspace;
 *     between calls it keeps nothing but a few facts per device (its CU
 *     count, and that a kernel's LDS limit has been raised there).  That
 *     function attribute is set by moe_init(), or else by the first launch of
 *     each kernel on a device: call moe_init() (or run one call) before
 *     capturing calls into a HIP graph.  The per-device facts are kept in
 *     atomics, so host threads may call concurrently (each on its own stream
 *     and workspace).  Calls act on the current device, which must be the
 *     one that owns the buffers.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No host synchronisation, no device-to-host copy:
 *     ragged per-expert sizes stay on the device.
 *   - Errors are return codes; nothing is thrown.  Arguments are checked before
 *     anything is enqueued; MOE_ERR_HIP (a launch failed) can leave earlier
 *     stages of the call enqueued.  Inputs are assumed finite; NaN/Inf logits
 *     give unspecified routing.
 *   - Identical inputs give bit-identical outputs, run to run (no floating-point
 *     atomics, token-order slot assignment).
 *   - Storage dtype `cfg->dtype` applies to x, Wg, W1, W2, b1, b2, xe, y and
 *     out.  Accumulation, softmax, activation and combine are fp32.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1,         /* null required pointer, dim <= 0, k > E, bad cf, misaligned pointer */
    MOE_ERR_UNSUPPORTED = -2,         /* H or I not a multiple of 8, E > MOE_MAX_EXPERTS, unknown dtype/act */
    MOE_ERR_WORKSPACE_TOO_SMALL = -3,
    MOE_ERR_HIP = -4,                 /* a launch failed (hipGetLastError) */
    /* reported by moe_ffn_status only (the single-launch FFN's bounded waits and placement check): */
    MOE_ERR_FFN_DEPENDENCY_TIMEOUT = -5,
    MOE_ERR_FFN_PLACEMENT = -6,
    /* moe_dispatch_noalloc only: the configuration needs more scratch than its fixed array holds */
    MOE_ERR_STATIC_SCRATCH_TOO_SMALL = -7
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1, MOE_F16 = 2 } moe_dtype;

typedef enum {
    MOE_ACT_RELU = 0,
    MOE_ACT_GELU_TANH = 1,            /* 0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3))) */
    MOE_ACT_GELU_ERF = 2,             /* 0.5 v (1 + erf(v / sqrt 2)) */
    MOE_ACT_IDENTITY = 3
} moe_act;

/* Who keeps a slot when more than C pairs name an expert (the paper leaves it open): */
typedef enum {
    MOE_DROP_TOKEN_MAJOR = 0,         /* pairs ordered by token, then choice rank (the default) */
    MOE_DROP_CHOICE_MAJOR = 1         /* every token's j-th choice before any (j+1)-th choice */
} moe_drop_policy;

/* Which expert capacity capacity_factor scales (the paper's text admits both): */
typedef enum {
    MOE_CAPACITY_PER_CHOICE = 0,      /* ceil(cf k T / E): cf = 1 holds every pair under balanced routing (default) */
    MOE_CAPACITY_LAYOUT = 1           /* ceil(cf T / E): the symmetric layout's C E W = S' (Sec. 3.2), no factor k */
} moe_capacity_mode;

/* moe_config.flags (bit set; unknown bits are MOE_ERR_INVALID_ARG) */
typedef enum {
    /* Both FFN tasks in one persistent launch: a t2 (second-GEMM) tile starts as soon as the t1 tiles it
     * reads are stored, tracked by per-row-tile completion counters (the tile-level dependency of the
     * paper's processors, Alg. 2) instead of a launch boundary.  Same arithmetic in the same order, so the
     * results are bit-identical to the default two launches, which are no slower on one MI355X.
     * 16-bit storage with H, I multiples of 64, at least 256: other configurations are
     * MOE_ERR_UNSUPPORTED.  First-task tiles never wait and a workgroup starts on its second-task tiles
     * only after storing all its first-task tiles, so the waits end whatever order the workgroups run in;
     * they are bounded all the same (about 0.3 s), and producer and consumer tiles meet in one XCD's L2,
     * which assumes that workgroup ids go round-robin to the XCDs -- the kernel checks that from the
     * hardware XCD number.  Either failure is recorded in the workspace, the call has already returned
     * MOE_OK by then, and moe_ffn_status reports it. */
    MOE_FLAG_FFN_SINGLE_LAUNCH = 1,
    /* Test aid, with MOE_FLAG_FFN_SINGLE_LAUNCH only: every dependency wait gets a target that cannot be
     * met and gives up after 16 polls, so that the give-up path runs with every kernel exiting normally;
     * y and out are then meaningless and moe_ffn_status returns MOE_ERR_FFN_DEPENDENCY_TIMEOUT. */
    MOE_FLAG_DEBUG_DEPENDENCY_NEVER_MET = 2,
    /* moe_forward only, on its own (no other flag): the whole layer from ONE persistent launch, the paper's
     * single-kernel operator (Alg. 1) on one GPU: gate, slot assignment, both FFN tasks and the combine are
     * stages of one kernel, one workgroup per CU, separated by four device-wide barriers (where the paper has
     * its scheduler and subscriber: on one GPU the stage boundaries are the only global dependencies), with
     * the FFN tasks ordered by the completion counters of MOE_FLAG_FFN_SINGLE_LAUNCH.  The stages are the
     * default path's device functions, so all outputs are bit-identical to it; it is no faster (back-to-back
     * launches leave no gaps on this GPU).  16-bit storage, E <= 128 (a multiple of 8), H and I multiples of
     * 64 and at least 256, token-order drop priority: otherwise MOE_ERR_UNSUPPORTED.  The barriers' state is
     * a few words inside the library, shared by every launch on a GPU: calls with this flag must not overlap on
     * one GPU.  All workgroups must be resident together (never more than one per CU is launched); the
     * barriers' polls are bounded all the same, and moe_ffn_status reports a give-up (and resets the barrier). */
    MOE_FLAG_LAYER_SINGLE_LAUNCH = 4
} moe_flags;

#define MOE_MAX_EXPERTS 8192

typedef struct {
    int32_t T;                        /* tokens on this GPU (the paper's S) */
    int32_t H;                        /* embedding dimension */
    int32_t I;                        /* FFN intermediate dimension (the paper's D) */
    int32_t E;                        /* local experts */
    int32_t k;                        /* experts selected per token, 1 <= k <= E */
    float capacity_factor;            /* used when capacity_override == 0 */
    int32_t capacity_override;        /* > 0: slots per expert given directly */
    int32_t dtype;                    /* moe_dtype */
    int32_t act;                      /* moe_act: phi_1 of the first FFN task */
    int32_t drop_policy;              /* moe_drop_policy */
    int32_t capacity_mode;            /* moe_capacity_mode, used when capacity_override == 0 */
    int32_t flags;                    /* moe_flags, 0 = defaults */
} moe_config;

const char* moe_status_string(moe_status s);

/* Optional set-up for the current device: raises the LDS limit of every kernel of the library there (a
 * function attribute that the launchers otherwise set on a kernel's first use) and reads the device's CU
 * count, so that later calls change no state and can be captured into a HIP graph without a warm-up call.
 * Idempotent; may be called from several host threads. */
moe_status moe_init(void);

/* Row-tile height bM to which per-expert buffers are aligned (in-place padding,
 * Sec. 3.2.1). */
int32_t moe_row_tile(void);

/* Expert capacity.  C = capacity_override if > 0, else
 * max(1, ceil(capacity_factor * k * T / E)), or without the factor k under
 * MOE_CAPACITY_LAYOUT: the drop threshold (slots per expert
 * in T_phi, Sec. 3 notation).  C_pad = C aligned up to moe_row_tile(): the row
 * stride of the per-expert buffers xe, y.  Alignment pads the buffer only.
 * Pure host arithmetic.  Either output may be NULL. */
moe_status moe_capacity(const moe_config* cfg, int32_t* C, int32_t* C_pad);

/* Bytes of device workspace that moe_forward and the staged calls need for this
 * configuration (gate scratch, routing tables, the lists of live FFN row tiles,
 * the FFN intermediate h and the expert outputs y; for fp32 storage also up to
 * 128 MiB of partial output tiles of the FFN kernel that deals equal shares of
 * the live work; the staged calls take xe and y from the caller). */
moe_status moe_workspace_bytes(const moe_config* cfg, size_t* bytes);

/* The whole layer (Alg. 1 restricted to one GPU: gate -> dispatch -> expert FFN
 * tasks -> combine), enqueued on `stream`.
 *   in : x[T,H], Wg[H,E], gate_bias[E] fp32 or NULL, W1[E,H,I], b1[E,I] or NULL,
 *        W2[E,I,H], b2[E,H] or NULL
 *   out: out[T,H]              out_i = sum over kept choices j of w_ij * FFN_{e_ij}(x_i),
 *                              zero row if every choice was dropped
 *        gate_logits[T,E] fp32 x Wg (+ bias); may be NULL (kept in the workspace)
 *        topk_expert[T,k]      experts by descending logit, equal logits -> smaller index
 *        topk_weight[T,k] fp32 softmax over the k selected logits (Eq. combine 1/2)
 *        slot[T,k]             slot of (token, choice) in its expert's buffer, -1 = dropped;
 *                              slots are handed out in token order, then choice order
 *                              (or choice rank first: cfg->drop_policy)
 *        expert_demand[E]      pairs that named each expert, before the capacity cut
 * All outputs except gate_logits are required.  On this path the packed copy xe
 * is not materialised: the first FFN task reads its rows from x through the
 * routing table (slot -> token), which is what the payload-efficient dispatch of
 * Sec. 3.2.1 amounts to on one GPU. */
moe_status moe_forward(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                       const void* x, const void* Wg, const float* gate_bias,
                       const void* W1, const void* b1, const void* W2, const void* b2,
                       void* out, float* gate_logits, int32_t* topk_expert, float* topk_weight,
                       int32_t* slot, int32_t* expert_demand, void* stream);

/* Measurement aid: moe_forward with HIP events recorded on `stream` at its stage boundaries, so that a
 * benchmark can price each stage (Alg. 1: gate, dispatch, the two FFN tasks, combine) inside the whole-layer
 * call and not in isolation.  events: MOE_FORWARD_EVENTS hipEvent_t created by the caller with timing
 * enabled, recorded in this order: before the gate, after the gate, after the routing launches, after the
 * first FFN launch, after the second (recorded right after [3] when one launch does both), after the
 * combine.  Everything else as moe_forward; the same kernels run in the same order. */
#define MOE_FORWARD_EVENTS 6
moe_status moe_forward_timed(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                             const void* x, const void* Wg, const float* gate_bias,
                             const void* W1, const void* b1, const void* W2, const void* b2,
                             void* out, float* gate_logits, int32_t* topk_expert, float* topk_weight,
                             int32_t* slot, int32_t* expert_demand, void* const* events, void* stream);

/* Yardsticks for the same benchmark: what this chip sustains on the two resources that bound the layer,
 * measured in the same process (the roofline's published peaks are never reached by any kernel).
 * moe_probe_stream: one kernel reads `bytes` (a multiple of 16) from src with 16-byte loads; with dst != NULL it
 *   also writes them there (a plain copy: the reference for hardware traffic counters).  sink: 4 bytes.
 * moe_probe_mfma: a register-resident loop of `iters` steps of dense MFMAs of the dtype (bf16 / f16:
 *   v_mfma_f32_16x16x32, fp32: v_mfma_f32_32x32x2) on pseudo-random finite operands, on every CU; *flops
 *   (host, may be NULL) receives the floating-point operations of the launch.  sink: 4 bytes.
 * Time them with events on `stream`. */
moe_status moe_probe_stream(const void* src, void* dst, size_t bytes, void* sink, void* stream);
moe_status moe_probe_mfma(int32_t dtype, int32_t iters, void* sink, double* flops, void* stream);

/* Yardstick, not part of the layer: the rate at which the CUs bring L2-resident data into LDS.  One workgroup per
 * CU walks a region of region_bytes (a multiple of 64 KiB; the workgroups of an XCD share one region, so `src` must
 * hold 8 * region_bytes, 16-byte aligned, device) round and round, 64 KiB per step, `steps` steps (even, >= 2).
 * mode 0: direct global-to-LDS copies (global_load_lds_dwordx4, the route the FFN and gate kernels use);
 * mode 1: vector loads into registers, then ds_write_b128; mode 2: the vector loads alone.  *bytes_moved (host,
 * optional) receives the bytes all workgroups moved; time the call with events.  `sink`: 4 bytes of device memory. */
moe_status moe_probe_lds_fill(int32_t mode, const void* src, size_t region_bytes, int32_t steps, void* sink,
                              double* bytes_moved, void* stream);

/* ---- staged entry points: the same kernels, one stage each ------------------- */

/* Gate ("FusedGate", Alg. 1): gate_logits = x Wg (+ gate_bias) with fp32
 * accumulation, then top-k and combine weights as in moe_route.  gate_logits is
 * required here. */
moe_status moe_gate(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                    const void* x, const void* Wg, const float* gate_bias,
                    float* gate_logits, int32_t* topk_expert, float* topk_weight, void* stream);

/* Selection only: caller-supplied gate_logits[T,E] -> topk_expert, topk_weight
 * (affinity scores G_phi -> the k experts E_{i,j} and weights g/C_i of
 * Eq. combine 1/2).  Lets tests drive tie-heavy logits through the selection
 * code. */
moe_status moe_route(const moe_config* cfg, const float* gate_logits,
                     int32_t* topk_expert, float* topk_weight, void* stream);

/* Dispatch on one GPU (Alg. 1 "Dispatch"; routing table T_phi; in-place
 * padding of Sec. 3.2.1): per-expert demand count, token-order slot
 * assignment with drops beyond C, then packing of the kept rows of x into
 * xe[E, C_pad, H] in slot order (rows at and beyond min(demand, C) are not
 * written).
 *   out: slot[T,k], expert_demand[E], slot_token[E,C] (-1 = empty),
 *        slot_weight[E,C] fp32 (0 = empty), xe[E,C_pad,H].
 * xe may be NULL to skip packing (routing tables only). */
moe_status moe_dispatch(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                        const void* x, const int32_t* topk_expert, const float* topk_weight,
                        int32_t* slot, int32_t* expert_demand, int32_t* slot_token,
                        float* slot_weight, void* xe, void* stream);

/* moe_dispatch for callers that can neither allocate nor bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels,
 * same results bit for bit.  Its scratch (the routing scan's per-chunk expert counts, ceil(T / 64) * E ints)
 * lives in a fixed array of MOE_STATIC_SCRATCH_BYTES that each GPU holds from the time the library's code is
 * loaded there until the process ends; configurations that need more return MOE_ERR_STATIC_SCRATCH_TOO_SMALL
 * before anything is enqueued (T = 16384 with E = 128 needs 128 KiB).  The call allocates nothing and frees
 * nothing.  The array's address on the current device is looked up on the first call there, or by moe_init():
 * call moe_init() first when the calls are to be captured.  All calls on one GPU share the one array: calls
 * that overlap there (two streams, two host threads) race on it and give wrong slots -- serialise them, or
 * use moe_dispatch with a workspace each. */
#define MOE_STATIC_SCRATCH_BYTES (4u << 20)
moe_status moe_dispatch_noalloc(const moe_config* cfg, const void* x, const int32_t* topk_expert,
                                const float* topk_weight, int32_t* slot, int32_t* expert_demand,
                                int32_t* slot_token, float* slot_weight, void* xe, void* stream);

/* Where the time of the last MOE_FLAG_LAYER_SINGLE_LAUNCH call on the current device went, as seen by its
 * workgroup 0 (wall-clock stamps at the stage boundaries of the one kernel; HIP events cannot look inside a
 * launch).  Waits for `stream`, then writes n <= MOE_LAYER_STAGES intervals in milliseconds to host_ms (host):
 *   0 gate tiles              1 wait at barrier 1
 *   2 table clearing + scan   3 wait at barrier 2
 *   4 scatter (+ unit lists)  5 wait at barrier 3
 *   6 first-GEMM tasks        7 second-GEMM tasks (their dependency waits included)
 *   8 wait at barrier 4       9 combine
 * A wait is short for the workgroup that arrives last and long for one that ran out of work early.  Meaningless
 * before the first such call.  MOE_ERR_INVALID_ARG for a null pointer or n outside 0..MOE_LAYER_STAGES. */
#define MOE_LAYER_STAGES 10
moe_status moe_layer_stage_ms(double* host_ms, int32_t n, void* stream);

/* Expert FFNs (tasks t1, t2 of Sec. 3.1; Eq. ffn in row-vector form): for each
 * expert e and each row r < min(expert_demand[e], C):
 *   y[e,r,:] = phi(xe[e,r,:] W1[e] + b1[e]) W2[e] + b2[e].
 * Only ceil(rows/bM) row tiles per expert are computed; rows beyond are left
 * untouched.  The intermediate h[E,C_pad,I] lives in the workspace.
 * cfg->flags & MOE_FLAG_FFN_SINGLE_LAUNCH runs both tasks in one persistent
 * launch (see moe_flags); follow it with moe_ffn_status when convenient. */
moe_status moe_expert_ffn(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                          const void* xe, const int32_t* expert_demand,
                          const void* W1, const void* b1, const void* W2, const void* b2,
                          void* y, void* stream);

/* Combine (task t3 of Sec. 3.1; Eq. combine 2):
 *   out[i,:] = sum_{j : slot[i,j] >= 0, ascending j} topk_weight[i,j] * y[topk_expert[i,j], slot[i,j], :]
 * in fp32, stored in the storage dtype. */
moe_status moe_combine(const moe_config* cfg, const void* y, const int32_t* topk_expert,
                       const float* topk_weight, const int32_t* slot, void* out, void* stream);

/* ---- backward pass ---------------------------------------------------------------------------------------
 * Gradients of the layer for training.  The paper runs the forward pass only and names training support as
 * future work ("Limitations and Future Work"), so it defines no backward; this is the chain rule applied to
 * Eq. ffn and Eqs. combine 1/2 with these readings: the routing (which k experts a token selected, which pairs
 * kept a slot) is a constant of the differentiation; the combine weights are differentiated as the softmax over
 * the k selected logits (all k enter the normalisation, dropped or not); a dropped pair sends no gradient
 * anywhere.  With dout = dL/dout for a scalar L:
 *   per kept pair (i, j), expert e, a = x_i W1_e + b1_e, h = phi(a), y = h W2_e + b2_e:
 *     dL/dw_ij = <dout_i, y>,  gy = w_ij dout_i,  db2_e += gy,  dW2_e += h^T gy,  da = (gy W2_e^T) * phi'(a),
 *     db1_e += da,  dW1_e += x_i^T da,  dx_i += da W1_e^T;
 *   per token: dl_ij = w_ij (dL/dw_ij - sum_j' w_ij' dL/dw_ij'),  dgate_bias[e_ij] += dl_ij,
 *     dWg[:, e_ij] += x_i dl_ij,  dx_i += dl_ij Wg[:, e_ij].
 * in : x, Wg, W1, b1 (or NULL), W2, b2 (or NULL) as in moe_forward; topk_expert[T,k], topk_weight[T,k] as
 *      moe_forward returned them (slots and drops are recomputed from them under cfg's capacity and drop
 *      policy); dout[T,H] in the storage dtype.
 * out: fp32, all required: dx[T,H], dWg[H,E], dgate_bias[E], dW1[E,H,I], db1[E,I], dW2[E,I,H], db2[E,H]
 *      (every element is written; experts without kept rows get zeros).
 * The expert activations are recomputed (nothing of the forward call's workspace is needed) and kept in the
 * storage dtype between kernels; accumulation is fp32; every reduction has a fixed order.  k <= 64 and
 * cfg->flags == 0, else MOE_ERR_UNSUPPORTED.  Workspace: moe_backward_workspace_bytes. */
moe_status moe_backward_workspace_bytes(const moe_config* cfg, size_t* bytes);
moe_status moe_backward(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                        const void* x, const void* Wg, const void* W1, const void* b1, const void* W2, const void* b2,
                        const int32_t* topk_expert, const float* topk_weight, const void* dout,
                        float* dx, float* dWg, float* dgate_bias, float* dW1, float* db1, float* dW2, float* db2,
                        void* stream);

/* Host arithmetic only (no device work): the tasks of one workgroup of the weight-streaming FFN kernels for
 * one GEMM over one of the two lists of live (expert, row tile) units (Sec. 3.1 tasks; the static stand-in for
 * the paper's scheduler, Alg. 3), in the order the workgroup runs them.  The same inline functions deal the
 * tasks inside the kernels.  large_list: 1 = the list of 256-row tiles (n_units_large units, nrow_large row
 * tiles per expert at most), 0 = the list of 128-row tiles (n_units_small units), whose dealing starts after
 * the XCD's last large-tile task; ncol = column tiles of the GEMM; workgroup `wg` of the `wgs` workgroups of
 * XCD `xcd` (0..7).  Writes up to max_tasks (index in the list, column tile) pairs and returns the
 * workgroup's task count, or -1 on invalid arguments.  For tests and for sizing launches. */
int32_t moe_ffn_schedule(int32_t large_list, int32_t n_units_large, int32_t n_units_small, int32_t nrow_large,
                         int32_t ncol, int32_t xcd, int32_t wg, int32_t wgs, int32_t* list_index, int32_t* col_tile,
                         int32_t max_tasks);

/* Host arithmetic only (no device work): how the fp32 FFN kernel that gives every workgroup an equal share of the
 * live work deals one GEMM (Sec. 3.1 tasks, cut along K as well; the same inline functions run inside the kernels).
 * rows[groups] (host): live rows per expert (values above `capacity` count as capacity); N, K: the GEMM's width and
 * depth; `workgroups`: the grid.  Writes the list of live (expert, 256-row tile) units as the device builds it:
 * unit_id[u] = expert * ceil(capacity / 256) + row tile, unit_cum[u] = sum of the weights of the units before u
 * (n + 1 entries; a unit's weight is the time of one of its iterations in twelfths of a full tile's).  Iterations are
 * numbered unit * ncol * nk + column tile * nk + K-tile (ncol = ceil(N / 256), nk = ceil(K / 32));
 * first_iteration[w] (workgroups + 1 entries) is where workgroup w starts, fix_tile[w] the tile (unit * ncol + column
 * tile) whose pieces the second pass adds up in workgroup w's name, or -1.  Returns the number of units, or -1 on
 * invalid arguments (null pointers, non-positive sizes, max_units < groups * ceil(capacity / 256)).  For tests. */
int32_t moe_f32_ffn_schedule(const int32_t* rows, int32_t groups, int32_t capacity, int32_t N, int32_t K,
                             int32_t workgroups, int64_t* first_iteration, int64_t* fix_tile, int32_t* unit_id,
                             int32_t* unit_cum, int32_t max_units);

/* Outcome of the single-launch FFN of the last moe_forward / moe_expert_ffn enqueued on `stream` with this
 * configuration and workspace (Alg. 2's dependency between t1 and t2 tiles, resolved by bounded waits).
 * Unlike every other call this one SYNCHRONISES: it copies the two fault words of the workspace to the host
 * and waits for `stream`.  MOE_OK, or MOE_ERR_FFN_DEPENDENCY_TIMEOUT (a wait gave up: y and out of that call
 * are invalid), or MOE_ERR_FFN_PLACEMENT (workgroups that must share an XCD's L2 did not: results may be
 * stale).  After calls without MOE_FLAG_FFN_SINGLE_LAUNCH, and for fp32 storage, it returns MOE_OK. */
moe_status moe_ffn_status(const moe_config* cfg, const void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
