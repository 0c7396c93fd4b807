/*
 * CPU oracle for one GPU's share of a capacity-bounded top-k MoE layer forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This library is the checker the HIP path is judged
 * against.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may load it; the product path never does.  It shares no source, header, table
 * or helper with the HIP library.
 *
 * What it computes is the plain definition of the layer (the paper's novelty is
 * scheduling and communication, not an approximation), in double precision:
 *
 *   O1  logits[i,e] = sum_h x[i,h] * Wg[h,e] (+ gate_bias[e])      -> float
 *       (gate, Alg. 1 "FusedGate"; affinity scores G_phi, Sec. 3 notation)
 *   O2  sel(i) = the k experts with the largest logits[i,.], by descending
 *       logit, equal logits -> smaller expert index first (compared as floats)
 *   O3  w[i,j] = exp(l_ij - m_i) / sum_j' exp(l_ij' - m_i), m_i = largest
 *       selected logit  (Eqs. "combine 1/2": g_{i,e_j} / C_i with
 *       C_i = sum_{j<=k} g_{i,e_j}; g = softmax over all E logits, so the ratio
 *       is the softmax over the k selected logits)                  -> float
 *   O4  C = capacity_override if > 0 else max(1, ceil(cf * k * T / E))
 *   O5  slots in token-major order (token 0 choice 0, token 0 choice 1, ...):
 *       the s-th pair that names expert e gets slot s if s < C, else is dropped
 *       (routing table T_phi(e,c) = (token, combine weight), Sec. 3 notation)
 *   O6  y_ij = phi(x_i W1_e + b1_e) W2_e + b2_e                     (Eq. "ffn")
 *   O7  out_i = sum_{j kept, ascending j} w[i,j] * y_ij, zero if none kept
 *       (Eq. "combine 2"; combine task C <- A (.) S + C)
 *
 * Readings taken where the paper is silent or garbled (each also listed in the
 * design notes of the repository):
 *   - gate = softmax over all E logits, no noise, optional additive bias;
 *   - Eq. combine 1/2 read as sums over the k selected experts e_j = E_{i,j};
 *   - normalisation is over all k selected experts, before any drop, so the
 *     kept weights of a token sum to <= 1;
 *   - capacity carries the factor k (cf = 1 is "just enough under perfectly
 *     balanced routing"); the layout section's C = S/E reading (no factor k)
 *     is oracle_capacity_layout, or any value through capacity_override;
 *   - aligning C up to the tile height pads the buffer only, never the drop
 *     threshold;
 *   - drop priority is token order; top-k ties go to the smaller expert index;
 *   - Eq. ffn is read in row-vector form phi(x W1 + b1) W2 + b2 with
 *     W1[E,H,I], W2[E,I,H];
 *   - "GELU" without qualifier is the erf form; the tanh form is a separate
 *     activation code;
 *   - 16-bit inputs are widened exactly; no intermediate is rounded; only the
 *     stored `out` is rounded (round to nearest even) to the storage dtype.
 *
 * Every function below is pinned by a CPU test against something other than
 * itself (closed forms, library routines on special cases, brute force, the
 * values of the paper's memory-overhead table).  Nothing here is
 * "parity unpinned".
 *
 * All pointers are HOST pointers.  Tensors are row-major and contiguous.
 * dtype codes: 0 = fp32, 1 = bf16, 2 = fp16 (storage of x, Wg, W1, W2, b1, b2,
 * out).  act codes: 0 = ReLU, 1 = GELU(tanh), 2 = GELU(erf), 3 = identity.
 */
#ifndef MOE_ORACLE_H
#define MOE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* threads used by the FFN / gate loops (OpenMP); returns the value in force */
int oracle_set_threads(int n);
int oracle_get_threads(void);

/* O4. Returns C, or -1 on invalid arguments. */
int32_t oracle_capacity(int32_t T, int32_t E, int32_t k, float capacity_factor,
                        int32_t capacity_override);

/* The other reading of the capacity, from the symmetric layout of Sec. 3.2
 * (C E W = S', uniform case S' = S): max(1, ceil(cf * T / E)), independent of k.
 * Returns C, or -1 on invalid arguments.  Feed it to the other functions as
 * capacity_override. */
int32_t oracle_capacity_layout(int32_t T, int32_t E, float capacity_factor);

/* In-place padding (Sec. 3.2.1): smallest multiple of bM that is >= C. */
int32_t oracle_align_up(int32_t C, int32_t bM);

/* Size in bytes of the symmetric tensor layout of Sec. 3.2 / Sec. 3.2.1 and the
 * memory-overhead table: 4 staging copies (2 rounds x 2 buffers) of E cells of
 * align_up(ceil(S/E), bM) rows of H elements of elem_bytes each. */
double oracle_symmetric_layout_bytes(int64_t S, int64_t E, int64_t H, int64_t bM,
                                     int64_t elem_bytes);

/* scalar activation in double, for pins */
double oracle_activation(double v, int32_t act);

/* O1 */
void oracle_gate_logits(const void* x, const void* Wg, const float* gate_bias,
                        int32_t T, int32_t H, int32_t E, int32_t dtype,
                        float* logits /* [T,E] */);

/* O2 + O3 */
void oracle_topk(const float* logits /* [T,E] */, int32_t T, int32_t E, int32_t k,
                 int32_t* topk_expert /* [T,k] */, float* topk_weight /* [T,k] */);

/* O5. slot_token[e,c] = -1 and slot_weight[e,c] = 0 for unused slots. */
void oracle_slots(const int32_t* topk_expert, const float* topk_weight,
                  int32_t T, int32_t E, int32_t k, int32_t C,
                  int32_t* slot /* [T,k], -1 = dropped */,
                  int32_t* expert_demand /* [E], pre-capacity counts */,
                  int32_t* slot_token /* [E,C] */, float* slot_weight /* [E,C] */);

/* O5 under the other drop priority the paper leaves open (it does not say who loses a slot when an
 * expert overflows): choice rank first, then token order -- every token's first choice is served
 * before any second choice.  Same outputs as oracle_slots; with k = 1 the two coincide. */
void oracle_slots_choice_major(const int32_t* topk_expert, const float* topk_weight,
                               int32_t T, int32_t E, int32_t k, int32_t C,
                               int32_t* slot, int32_t* expert_demand,
                               int32_t* slot_token, float* slot_weight);

/* O6 for n given (token, expert) pairs: y[p,:] in double. */
void oracle_ffn_rows(const void* x, const void* W1, const void* b1,
                     const void* W2, const void* b2,
                     const int32_t* pair_token, const int32_t* pair_expert, int32_t n,
                     int32_t H, int32_t I, int32_t act, int32_t dtype,
                     double* y /* [n,H] */);

/* O6 + O7 under a given routing, for the tokens listed in `tokens`
 * (n_tokens entries; NULL = all T tokens in order).
 * out_f64 [n_tokens,H] unrounded (may be NULL); out [n_tokens,H] in the storage
 * dtype (may be NULL). */
void oracle_ffn_combine(const void* x, const void* W1, const void* b1,
                        const void* W2, const void* b2,
                        const int32_t* topk_expert, const float* topk_weight,
                        const int32_t* slot,
                        int32_t T, int32_t H, int32_t I, int32_t E, int32_t k,
                        int32_t act, int32_t dtype,
                        const int32_t* tokens, int32_t n_tokens,
                        double* out_f64, void* out);

/* O1..O7 in one call. Any output pointer may be NULL except none is required.
 * slot_token / slot_weight have C columns where C = oracle_capacity(...). */
int32_t oracle_forward(const void* x, const void* Wg, const float* gate_bias,
                       const void* W1, const void* b1, const void* W2, const void* b2,
                       int32_t T, int32_t H, int32_t I, int32_t E, int32_t k,
                       float capacity_factor, int32_t capacity_override,
                       int32_t act, int32_t dtype,
                       float* gate_logits, int32_t* topk_expert, float* topk_weight,
                       int32_t* slot, int32_t* expert_demand,
                       int32_t* slot_token, float* slot_weight,
                       double* out_f64, void* out);

/* Gradients of the layer (the paper leaves training to future work and states no backward pass; this is
 * the chain rule applied to O1..O7, i.e. to Eq. ffn and Eqs. combine 1/2, with the reading below).
 * Reading: the routing -- which k experts a token selected (topk_expert) and which pairs kept a slot (slot) --
 * is a constant of the differentiation; the combine weights are differentiated as the softmax over the k
 * selected logits l_ij = x_i Wg[:, e_ij] + gate_bias[e_ij] (every selected logit enters the normalisation,
 * dropped or not, as in O3); a dropped pair contributes nothing to out, so nothing flows into its expert and
 * dL/dw_ij = 0.  Everything is evaluated in double on the exactly widened inputs (the float roundings of
 * O1 and O3 are not differentiable and are not applied).  With L any scalar with dL/dout = dout:
 *   B1  w_ij   = softmax_j(l_i,.)
 *   B2  per kept pair: a = x_i W1_e + b1_e, h = phi(a), y = h W2_e + b2_e;
 *       dL/dw_ij = <dout_i, y>;  gy = w_ij dout_i
 *   B3  db2_e += gy;  dW2_e += h^T gy;  da = (gy W2_e^T) * phi'(a);  db1_e += da;  dW1_e += x_i^T da;
 *       dx_i += da W1_e^T
 *   B4  dl_ij = w_ij (dL/dw_ij - sum_j' w_ij' dL/dw_ij')
 *   B5  dgate_bias[e_ij] += dl_ij;  dWg[:, e_ij] += x_i dl_ij;  dx_i += dl_ij Wg[:, e_ij]
 * dout is [T,H] in double.  Every output is in double and may be NULL: dx [T,H], dWg [H,E], dgate_bias [E],
 * dW1 [E,H,I], db1 [E,I], dW2 [E,I,H], db2 [E,H]. */
void oracle_backward(const void* x, const void* Wg, const float* gate_bias,
                     const void* W1, const void* b1, const void* W2, const void* b2,
                     const int32_t* topk_expert, const int32_t* slot, const double* dout,
                     int32_t T, int32_t H, int32_t I, int32_t E, int32_t k,
                     int32_t act, int32_t dtype,
                     double* dx, double* dWg, double* dgate_bias,
                     double* dW1, double* db1, double* dW2, double* db2);

/* derivative of the activation, for pins */
double oracle_activation_grad(double v, int32_t act);

/* storage-dtype helpers (exact widening; round-to-nearest-even narrowing) */
double oracle_load_elem(const void* p, int64_t idx, int32_t dtype);
void   oracle_store_elem(void* p, int64_t idx, int32_t dtype, double v);

#ifdef __cplusplus
}
#endif
#endif
