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
 *     count, and that a kernel's LDS limit has been raised there: the first
 *     launch of each kernel on a device sets that function attribute, so run
 *     one call before capturing calls into a HIP graph).  Calls act on the
 *     current device, which must be the one that owns the buffers.
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
    MOE_ERR_HIP = -4                  /* a launch failed (hipGetLastError) */
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
} moe_config;

const char* moe_status_string(moe_status s);

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
 * configuration (gate scratch, routing tables, the FFN intermediate h and the
 * expert outputs y; the staged calls take xe and y from the caller). */
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

/* Expert FFNs (tasks t1, t2 of Sec. 3.1; Eq. ffn in row-vector form): for each
 * expert e and each row r < min(expert_demand[e], C):
 *   y[e,r,:] = phi(xe[e,r,:] W1[e] + b1[e]) W2[e] + b2[e].
 * Only ceil(rows/bM) row tiles per expert are computed; rows beyond are left
 * untouched.  The intermediate h[E,C_pad,I] lives in the workspace.
 * With the environment variable MOE_FFN_FUSED=1 (read at each call) eligible
 * 16-bit shapes run both tasks in one persistent launch, a t2 tile starting
 * when the t1 tiles it reads are stored (Alg. 2's tile-level dependency);
 * the results are identical, the two-launch default is faster on one GPU. */
moe_status moe_expert_ffn(const moe_config* cfg, void* workspace, size_t workspace_bytes,
                          const void* xe, const int32_t* expert_demand,
                          const void* W1, const void* b1, const void* W2, const void* b2,
                          void* y, void* stream);

/* Combine (task t3 of Sec. 3.1; Eq. combine 2):
 *   out[i,:] = sum_{j : slot[i,j] >= 0, ascending j} topk_weight[i,j] * y[topk_expert[i,j], slot[i,j], :]
 * in fp32, stored in the storage dtype. */
moe_status moe_combine(const moe_config* cfg, const void* y, const int32_t* topk_expert,
                       const float* topk_weight, const int32_t* slot, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif
