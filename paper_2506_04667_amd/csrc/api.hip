// C ABI of the MoE layer forward (see include/moe.h): argument validation,
// capacity arithmetic, workspace carving and the launch sequence
// gate -> dispatch -> expert FFN -> combine (Alg. 1 restricted to one GPU).
// Host code only; every step of the path runs in the kernels it launches.
#include "../../include/moe.h"

#include <cmath>
#include <initializer_list>

#include "ffn_units.h"
#include "kernels.h"

// Scratch of moe_dispatch_noalloc, the entry point for callers that cannot allocate: a fixed array in device
// memory that every GPU the library runs on holds from the moment the code object is loaded there.  In host code
// this name is only a handle for hipGetSymbolAddress; the address it yields (one per device) is what kernels,
// fills and copies get.
constexpr size_t kStaticScratchBytes = 4u << 20;
static_assert(kStaticScratchBytes == MOE_STATIC_SCRATCH_BYTES, "the limit stated in the header");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` on the current device, looked up once per device with that device current.
hipError_t static_scratch(void** out) {
    static std::atomic<void*> ptr[moe::kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= moe::kMaxDevices) return hipErrorInvalidDevice;
    void* p = ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

constexpr int kRowTile = 128;     // bM: per-expert buffers are aligned to this many rows
constexpr int kGatePad = 128;     // WgT rows are padded to a multiple of the gate GEMM's column tile
constexpr size_t kAlign = 256;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
    int C, C_pad, E_pad, elem;
    size_t off_wgt, off_logits, off_slot_token, off_slot_weight, off_counts, off_units, off_partials, off_h, off_y, total;
    int ldh;                                             // row pitch of h in elements
};

moe_status check_config(const moe_config* c) {
    if (!c) return MOE_ERR_INVALID_ARG;
    if (c->T <= 0 || c->H <= 0 || c->I <= 0 || c->E <= 0 || c->k <= 0 || c->k > c->E) return MOE_ERR_INVALID_ARG;
    if (c->capacity_override < 0) return MOE_ERR_INVALID_ARG;
    if (c->capacity_override == 0 && !(c->capacity_factor > 0.0f && std::isfinite(c->capacity_factor)))
        return MOE_ERR_INVALID_ARG;
    if (c->dtype < MOE_F32 || c->dtype > MOE_F16) return MOE_ERR_UNSUPPORTED;
    if (c->act < MOE_ACT_RELU || c->act > MOE_ACT_IDENTITY) return MOE_ERR_UNSUPPORTED;
    if (c->H % 8 != 0 || c->I % 8 != 0) return MOE_ERR_UNSUPPORTED;
    if (c->E > MOE_MAX_EXPERTS) return MOE_ERR_UNSUPPORTED;
    if (c->drop_policy < MOE_DROP_TOKEN_MAJOR || c->drop_policy > MOE_DROP_CHOICE_MAJOR) return MOE_ERR_UNSUPPORTED;
    if (c->capacity_mode < MOE_CAPACITY_PER_CHOICE || c->capacity_mode > MOE_CAPACITY_LAYOUT) return MOE_ERR_UNSUPPORTED;
    if (c->flags & ~(MOE_FLAG_FFN_SINGLE_LAUNCH | MOE_FLAG_DEBUG_DEPENDENCY_NEVER_MET | MOE_FLAG_LAYER_SINGLE_LAUNCH))
        return MOE_ERR_INVALID_ARG;
    if ((c->flags & MOE_FLAG_LAYER_SINGLE_LAUNCH) && (c->flags & ~MOE_FLAG_LAYER_SINGLE_LAUNCH)) return MOE_ERR_INVALID_ARG;
    if ((c->flags & MOE_FLAG_DEBUG_DEPENDENCY_NEVER_MET) && !(c->flags & MOE_FLAG_FFN_SINGLE_LAUNCH)) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

moe_status capacity_of(const moe_config* c, int* C, int* C_pad) {
    long long cap;
    if (c->capacity_override > 0) {
        cap = c->capacity_override;
    } else {
        const double per_token = c->capacity_mode == MOE_CAPACITY_LAYOUT ? 1.0 : (double)c->k;
        const double v = std::ceil((double)c->capacity_factor * per_token * (double)c->T / (double)c->E);
        if (v > 2.0e9) return MOE_ERR_INVALID_ARG;
        cap = v < 1.0 ? 1 : (long long)v;
    }
    const long long pad = (cap + kRowTile - 1) / kRowTile * kRowTile;
    if (pad > 0x7fffffffLL) return MOE_ERR_INVALID_ARG;
    *C = (int)cap;
    *C_pad = (int)pad;
    return MOE_OK;
}

moe_status make_plan(const moe_config* c, Plan* p) {
    moe_status st = check_config(c);
    if (st != MOE_OK) return st;
    st = capacity_of(c, &p->C, &p->C_pad);
    if (st != MOE_OK) return st;
    p->elem = c->dtype == MOE_F32 ? 4 : 2;
    p->E_pad = (int)align_up((size_t)c->E, kGatePad);
    const size_t T = c->T, H = c->H, I = c->I, E = c->E, el = p->elem;
    const size_t rows = E * (size_t)p->C_pad;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, kAlign); return o; };
    p->off_wgt = take((size_t)p->E_pad * H * el);
    p->off_logits = take(T * E * 4);
    p->off_slot_token = take(E * (size_t)p->C * 4);
    p->off_slot_weight = take(E * (size_t)p->C * 4);
    p->off_counts = take((size_t)moe::route_chunks(c->T) * E * 4);
    // 16-bit storage: the two lists of live row tiles of the weight-streaming kernels; fp32: the list of live 64-row
    // tiles of the equal-span kernel and its partial tiles
    p->off_units = take((c->dtype == MOE_F32 ? moe::f32_units_ints(c->E, p->C) : moe::ffn_units_ints(c->E, p->C)) * 4);
    p->off_partials = take(c->dtype == MOE_F32 ? moe::f32_partials_bytes(c->E, p->C, c->H, c->I) : 0);
    p->ldh = c->I;                                       // (a pitch padded by one 128-byte line measured no different)
    p->off_h = take(rows * (size_t)p->ldh * el);
    p->off_y = take(rows * H * el);
    p->total = off;
    return MOE_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// MOE_FLAG_FFN_SINGLE_LAUNCH asks for both FFN tasks in one persistent launch; only shapes that the
// weight-streaming kernel takes for both tasks can run that way.  `gather`: the first task reads token rows
// through the routing table (moe_forward) instead of packed rows (moe_expert_ffn).
moe_status check_single_launch(const moe_config* c, const Plan& p, bool gather) {
    if (!(c->flags & MOE_FLAG_FFN_SINGLE_LAUNCH)) return MOE_OK;
    const bool ok = moe::stream_gemm_shape_ok(c->dtype, c->I, c->H, c->H, c->I, p.ldh, gather ? c->T : p.C_pad) &&
                    moe::stream_gemm_shape_ok(c->dtype, c->H, c->I, p.ldh, c->H, c->H, p.C_pad);
    return ok ? MOE_OK : MOE_ERR_UNSUPPORTED;
}

moe_status hip_status(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

char* ws_at(void* ws, size_t off) { return (char*)ws + off; }

// ---- stage launchers (arguments already validated) ---------------------------------

moe_status run_gate(const moe_config* c, const Plan& p, void* ws, const void* x, const void* Wg,
                    const float* gate_bias, float* logits, int32_t* topk_expert, float* topk_weight,
                    bool* route_counts_written, hipStream_t s) {
    // route_counts_written != nullptr: the caller goes on to the slot assignment; the fused gate then writes
    // the per-chunk expert counts into the workspace and says so
    if (route_counts_written) *route_counts_written = false;
    if (moe::gate_fused_eligible(c->T, c->H, c->E, c->k, c->dtype)) {
        int32_t* counts = route_counts_written ? (int32_t*)ws_at(ws, p.off_counts) : nullptr;
        if (route_counts_written) *route_counts_written = true;
        return hip_status(moe::launch_gate_fused(x, Wg, gate_bias, c->T, c->H, c->E, c->k, c->dtype, logits,
                                                 topk_expert, topk_weight, counts, s));
    }
    void* wgt = ws_at(ws, p.off_wgt);
    hipError_t e = moe::launch_transpose_pad(Wg, wgt, c->H, c->E, p.E_pad, c->dtype, s);
    if (e != hipSuccess) return MOE_ERR_HIP;
    moe::GemmArgs g{};
    g.A = x; g.a_group_stride = 0; g.lda = c->H;
    g.a_row_index = nullptr; g.a_index_stride = 0; g.a_rows_total = c->T;
    g.B = wgt; g.b_group_stride = 0; g.ldb = c->H;
    g.C = logits; g.c_group_stride = 0; g.ldc = c->E;
    g.bias = gate_bias; g.bias_group_stride = 0;
    g.rows_dev = nullptr; g.rows_fixed = c->T; g.rows_cap = c->T;
    g.groups = 1; g.max_rows = c->T;
    g.N = c->E; g.K = c->H;
    g.act = MOE_ACT_IDENTITY; g.dtype = c->dtype; g.b_is_nk = true; g.c_f32 = true;
    e = moe::launch_grouped_gemm(g, s);
    if (e != hipSuccess) return MOE_ERR_HIP;
    return hip_status(moe::launch_topk(logits, c->T, c->E, c->k, topk_expert, topk_weight, s));
}

// counts: scratch of route_chunks(T) * E ints; units: the FFN kernels' scratch block to fill, or nullptr
moe_status run_dispatch(const moe_config* c, const Plan& p, int32_t* counts, int32_t* units, const void* x,
                        const int32_t* topk_expert, const float* topk_weight, int32_t* slot,
                        int32_t* expert_demand, int32_t* slot_token, float* slot_weight, void* xe,
                        bool counts_ready, hipStream_t s) {
    // the fused gate counts per chunk of 64 tokens, which is a chunk of the pair order only under token-major priority
    const bool choice_major = c->drop_policy == MOE_DROP_CHOICE_MAJOR;
    hipError_t e = moe::launch_route(topk_expert, topk_weight, c->T, c->E, c->k, p.C, choice_major,
                                     counts, counts_ready && !choice_major, slot, expert_demand,
                                     slot_token, slot_weight, units, c->dtype == MOE_F32, s);
    if (e != hipSuccess) return MOE_ERR_HIP;
    if (!xe) return MOE_OK;
    return hip_status(moe::launch_pack(x, topk_expert, slot, c->T, c->H, c->k, c->E, p.C, p.C_pad, c->dtype, xe, s));
}

// The two GEMMs of the expert FFN as grouped-GEMM arguments.
// xe: packed rows [E, C_pad, H]; or, with slot_token given, the token matrix x[T, H] whose rows the
// first GEMM gathers through slot_token[E, C] (no packed copy).
void ffn_gemms(const moe_config* c, const Plan& p, void* ws, const void* xe, const int32_t* slot_token,
               const int32_t* expert_demand, const void* W1, const void* b1, const void* W2, const void* b2, void* y,
               moe::GemmArgs* g1_out, moe::GemmArgs* g2_out) {
    void* h = ws_at(ws, p.off_h);
    const long long H = c->H, I = c->I;
    moe::GemmArgs g{};
    g.rows_dev = expert_demand; g.rows_fixed = 0; g.rows_cap = p.C;
    g.groups = c->E; g.max_rows = p.C;
    g.dtype = c->dtype; g.b_is_nk = false; g.c_f32 = false;
    // both tasks walk the same live (expert, row tile) units
    g.units = (int32_t*)ws_at(ws, p.off_units);
    if (c->dtype == MOE_F32) g.partials = (float*)ws_at(ws, p.off_partials);
    // task t1: h = phi1(xe W1 + b1)
    moe::GemmArgs g1 = g;
    g1.A = xe; g1.a_group_stride = (long long)p.C_pad * H; g1.lda = c->H;
    g1.a_row_index = slot_token; g1.a_index_stride = p.C;
    g1.a_rows_total = slot_token ? c->T : p.C_pad;
    g1.B = W1; g1.b_group_stride = H * I; g1.ldb = c->I;
    g1.C = h; g1.c_group_stride = (long long)p.C_pad * p.ldh; g1.ldc = p.ldh;
    g1.bias = b1; g1.bias_group_stride = I;
    g1.N = c->I; g1.K = c->H; g1.act = c->act;
    // task t2: y = h W2 + b2
    moe::GemmArgs g2 = g;
    g2.A = h; g2.a_group_stride = (long long)p.C_pad * p.ldh; g2.lda = p.ldh;
    g2.a_row_index = nullptr; g2.a_index_stride = 0;
    g2.a_rows_total = p.C_pad;
    g2.B = W2; g2.b_group_stride = I * H; g2.ldb = c->H;
    g2.C = y; g2.c_group_stride = (long long)p.C_pad * H; g2.ldc = c->H;
    g2.bias = b2; g2.bias_group_stride = H;
    g2.N = c->H; g2.K = c->I; g2.act = MOE_ACT_IDENTITY;
    *g1_out = g1;
    *g2_out = g2;
}

moe_status run_ffn(const moe_config* c, const Plan& p, void* ws, const void* xe, const int32_t* slot_token,
                   const int32_t* expert_demand, const void* W1, const void* b1, const void* W2,
                   const void* b2, void* y, bool units_ready, hipEvent_t between, hipStream_t s) {
    moe::GemmArgs g1, g2;
    ffn_gemms(c, p, ws, xe, slot_token, expert_demand, W1, b1, W2, b2, y, &g1, &g2);
    hipError_t e = hipSuccess;
    if (!units_ready) {
        e = c->dtype == MOE_F32 ? moe::launch_f32_units(expert_demand, p.C, c->E, p.C, g1.units, s)
                                : moe::launch_ffn_units(expert_demand, p.C, c->E, p.C, g1.units, s);
        if (e != hipSuccess) return MOE_ERR_HIP;
    }
    // Optional: one persistent launch for both tasks, a t2 tile starting when the t1 tiles it reads are stored
    // (the tile-level dependency of the paper's processors, Alg. 2).  No faster than two launches on one
    // MI355X at the paper's shapes, so it is opt-in (MOE_FLAG_FFN_SINGLE_LAUNCH; shapes checked by the caller).
    if (c->flags & MOE_FLAG_FFN_SINGLE_LAUNCH) {
        if (!moe::ffn_fused_eligible(g1, g2)) return MOE_ERR_UNSUPPORTED;
        e = moe::launch_ffn_stream_fused(g1, g2, (c->flags & MOE_FLAG_DEBUG_DEPENDENCY_NEVER_MET) != 0, s);
        if (e == hipSuccess && between) e = hipEventRecord(between, s);
        return hip_status(e);
    }
    e = moe::launch_grouped_gemm(g1, s);
    if (e != hipSuccess) return MOE_ERR_HIP;
    if (between && hipEventRecord(between, s) != hipSuccess) return MOE_ERR_HIP;
    return hip_status(moe::launch_grouped_gemm(g2, s));
}

moe_status run_combine(const moe_config* c, const Plan& p, const void* y, const int32_t* topk_expert,
                       const float* topk_weight, const int32_t* slot, void* out, hipStream_t s) {
    return hip_status(moe::launch_combine(y, topk_expert, topk_weight, slot, c->T, c->H, c->k, c->E, p.C,
                                          p.C_pad, c->dtype, out, s));
}

bool bad_required(std::initializer_list<const void*> ptrs) {
    for (const void* q : ptrs)
        if (!q || misaligned(q)) return true;
    return false;
}
bool bad_optional(std::initializer_list<const void*> ptrs) {
    for (const void* q : ptrs)
        if (q && misaligned(q)) return true;
    return false;
}

// The whole layer on one stream.  `ev` (optional, MOE_FORWARD_EVENTS events) are recorded on the stream at the
// stage boundaries: before the gate, after the gate, after the routing launches, after the first FFN launch,
// after the second (the same point as the first under the single-launch flag), after the combine.
moe_status forward_impl(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x,
                        const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                        const void* W2, const void* b2, void* out, float* gate_logits,
                        int32_t* topk_expert, float* topk_weight, int32_t* slot, int32_t* expert_demand,
                        const hipEvent_t* ev, hipStream_t s) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({workspace, x, Wg, W1, W2, out, topk_expert, topk_weight, slot, expert_demand}) ||
        bad_optional({gate_bias, b1, b2, gate_logits}))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    st = check_single_launch(cfg, p, true);
    if (st != MOE_OK) return st;
    const bool one_launch = (cfg->flags & MOE_FLAG_LAYER_SINGLE_LAUNCH) != 0;
    if (one_launch && (cfg->drop_policy != MOE_DROP_TOKEN_MAJOR ||
                       !moe::layer_fused_eligible(cfg->T, cfg->H, cfg->I, p.ldh, cfg->E, cfg->k, p.C_pad, cfg->dtype)))
        return MOE_ERR_UNSUPPORTED;
    auto mark = [&](int i) { return !ev || hipEventRecord(ev[i], s) == hipSuccess; };
    float* logits = gate_logits ? gate_logits : (float*)ws_at(workspace, p.off_logits);
    int32_t* slot_token = (int32_t*)ws_at(workspace, p.off_slot_token);
    float* slot_weight = (float*)ws_at(workspace, p.off_slot_weight);
    void* y = ws_at(workspace, p.off_y);
    bool counts_ready = false;
    if (!mark(0)) return MOE_ERR_HIP;
    if (one_launch) {
        // Alg. 1 as one persistent kernel: the same stages from one launch, device-wide barriers in between
        moe::GemmArgs g1, g2;
        ffn_gemms(cfg, p, workspace, x, slot_token, expert_demand, W1, b1, W2, b2, y, &g1, &g2);
        if (moe::launch_layer_fused(x, Wg, gate_bias, cfg->T, cfg->H, cfg->E, cfg->k, p.C, p.C_pad, cfg->dtype, logits, topk_expert,
                                    topk_weight, (int32_t*)ws_at(workspace, p.off_counts), slot, expert_demand, slot_token,
                                    slot_weight, g1, g2, out, s) != hipSuccess)
            return MOE_ERR_HIP;
        for (int i = 1; i < MOE_FORWARD_EVENTS; ++i)
            if (!mark(i)) return MOE_ERR_HIP;
        return MOE_OK;
    }
    st = run_gate(cfg, p, workspace, x, Wg, gate_bias, logits, topk_expert, topk_weight, &counts_ready, s);
    if (st != MOE_OK) return st;
    if (!mark(1)) return MOE_ERR_HIP;
    // Dispatch builds the routing table only; the first FFN GEMM gathers its rows from x through
    // slot_token, so the packed copy xe is never materialised on this path.
    // the scatter launch also lists the live FFN units
    st = run_dispatch(cfg, p, (int32_t*)ws_at(workspace, p.off_counts), (int32_t*)ws_at(workspace, p.off_units), x, topk_expert,
                      topk_weight, slot, expert_demand, slot_token, slot_weight, nullptr, counts_ready, s);
    if (st != MOE_OK) return st;
    if (!mark(2)) return MOE_ERR_HIP;
    st = run_ffn(cfg, p, workspace, x, slot_token, expert_demand, W1, b1, W2, b2, y, true, ev ? ev[3] : nullptr, s);
    if (st != MOE_OK) return st;
    if (!mark(4)) return MOE_ERR_HIP;
    st = run_combine(cfg, p, y, topk_expert, topk_weight, slot, out, s);
    if (st != MOE_OK) return st;
    return mark(5) ? MOE_OK : MOE_ERR_HIP;
}

// ---- backward pass: workspace carving and launch order -------------------------------------------------------
struct BwdPlan {
    Plan p;
    int ldL, T_pad;
    int wg_slices, wg_slice_k;                           // dWg = x^T dL as wg_slices partial products over wg_slice_k tokens each
    size_t off_wg_part;
    size_t off_counts, off_units, off_slot_token, off_slot_weight, off_slot, off_demand, off_dl, off_dL, off_wgt, off_xe,
        off_gy, off_a, off_h, off_dh, off_y, off_hT, off_xeT, off_xT, off_wrows, off_wunits1, off_wunits2, total;
};

moe_status make_bwd_plan(const moe_config* c, BwdPlan* b) {
    moe_status st = make_plan(c, &b->p);
    if (st != MOE_OK) return st;
    if (c->k > 64) return MOE_ERR_UNSUPPORTED;          // the gate's Jacobian kernel keeps a token's choices in one wavefront
    if (c->flags != 0) return MOE_ERR_UNSUPPORTED;
    const Plan& p = b->p;
    const size_t T = c->T, H = c->H, I = c->I, E = c->E, k = c->k, el = p.elem;
    const size_t rows = E * (size_t)p.C_pad;
    b->ldL = (int)align_up(E, 8);
    // dWg has only (H / 128) x (E / 128) output tiles for a contraction over all T tokens: the tokens are cut into up to
    // 16 slices of at least 1024, each slice one "group" of the grouped GEMM, and the partial products added in slice order
    b->wg_slices = (int)(T / 1024 < 1 ? 1 : (T / 1024 > 16 ? 16 : T / 1024));
    b->wg_slice_k = (int)align_up((T + b->wg_slices - 1) / b->wg_slices, 64);
    b->T_pad = b->wg_slices * b->wg_slice_k;             // >= T: x^T rows and dL are zero beyond T
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, kAlign); return o; };
    b->off_counts = take((size_t)moe::route_chunks(c->T) * E * 4);
    b->off_units = take(moe::ffn_units_ints(c->E, p.C) * 4);
    b->off_slot_token = take(E * (size_t)p.C * 4);
    b->off_slot_weight = take(E * (size_t)p.C * 4);
    b->off_slot = take(T * k * 4);
    b->off_demand = take(E * 4);
    b->off_dl = take(T * k * 4);
    b->off_dL = take((size_t)b->T_pad * b->ldL * el);
    b->off_wg_part = take(b->wg_slices > 1 ? (size_t)b->wg_slices * H * E * 4 : 0);
    b->off_wgt = take((size_t)p.E_pad * H * el);
    b->off_xe = take(rows * H * el);
    b->off_gy = take(rows * H * el);
    b->off_a = take(rows * I * el);
    b->off_h = take(rows * I * el);
    b->off_dh = take(rows * I * el);
    b->off_y = take(rows * H * el);
    b->off_hT = take(rows * I * el);
    b->off_xeT = take(rows * H * el);
    b->off_xT = take(H * (size_t)b->T_pad * el);
    // the weight-gradient GEMMs as streaming-kernel launches: their "experts" have H (dW1) or I (dW2) rows each
    b->off_wrows = take(2 * E * 4);
    b->off_wunits1 = take(moe::ffn_units_ints(c->E, c->H) * 4);
    b->off_wunits2 = take(moe::ffn_units_ints(c->E, c->I) * 4);
    b->total = off;
    return MOE_OK;
}

moe_status run_backward(const moe_config* c, const BwdPlan& b, void* ws, const void* x, const void* Wg, const void* W1,
                        const void* b1, const void* W2, const void* b2, const int32_t* topk_expert, const float* topk_weight,
                        const void* dout, float* dx, float* dWg, float* dgate_bias, float* dW1, float* db1, float* dW2,
                        float* db2, hipStream_t s) {
    const Plan& p = b.p;
    const int T = c->T, H = c->H, I = c->I, E = c->E, k = c->k, C = p.C, C_pad = p.C_pad, dt = c->dtype;
    int32_t* counts = (int32_t*)ws_at(ws, b.off_counts);
    int32_t* units = dt != MOE_F32 ? (int32_t*)ws_at(ws, b.off_units) : nullptr;
    int32_t* slot_token = (int32_t*)ws_at(ws, b.off_slot_token);
    float* slot_weight = (float*)ws_at(ws, b.off_slot_weight);
    int32_t* slot = (int32_t*)ws_at(ws, b.off_slot);
    int32_t* demand = (int32_t*)ws_at(ws, b.off_demand);
    float* dl = (float*)ws_at(ws, b.off_dl);
    void *dL = ws_at(ws, b.off_dL), *wgt = ws_at(ws, b.off_wgt), *xe = ws_at(ws, b.off_xe), *gy = ws_at(ws, b.off_gy);
    void *a = ws_at(ws, b.off_a), *h = ws_at(ws, b.off_h), *dh = ws_at(ws, b.off_dh), *y = ws_at(ws, b.off_y);
    void *hT = ws_at(ws, b.off_hT), *xeT = ws_at(ws, b.off_xeT), *xT = ws_at(ws, b.off_xT);
#define MOE_TRY(call) do { if ((call) != hipSuccess) return MOE_ERR_HIP; } while (0)
    // the routing tables again, from the selection the forward pass made (slots are a function of it)
    MOE_TRY(moe::launch_route(topk_expert, topk_weight, T, E, k, C, c->drop_policy == MOE_DROP_CHOICE_MAJOR, counts, false, slot,
                              demand, slot_token, slot_weight, units, false, s));
    MOE_TRY(moe::launch_transpose_pad(Wg, wgt, H, E, p.E_pad, dt, s));
    MOE_TRY(moe::launch_bwd_gather(x, dout, slot_token, slot_weight, H, E, C, C_pad, dt, xe, gy, s));
    // grouped GEMMs over the experts' live rows
    moe::GemmArgs g{};
    g.rows_dev = demand; g.rows_fixed = 0; g.rows_cap = C; g.groups = E; g.max_rows = C;
    g.dtype = dt; g.act = MOE_ACT_IDENTITY; g.a_rows_total = C_pad;
    const long long rH = (long long)C_pad * H, rI = (long long)C_pad * I, HI = (long long)H * I;
    // forward again, keeping the pre-activation: a = xe W1 + b1, h = phi(a), y = h W2 + b2
    moe::GemmArgs f1 = g;
    f1.A = xe; f1.a_group_stride = rH; f1.lda = H; f1.B = W1; f1.b_group_stride = HI; f1.ldb = I;
    f1.C = a; f1.c_group_stride = rI; f1.ldc = I; f1.bias = b1; f1.bias_group_stride = I; f1.N = I; f1.K = H; f1.units = units;
    MOE_TRY(moe::launch_grouped_gemm(f1, s));
    MOE_TRY(moe::launch_bwd_act(a, nullptr, demand, E, C, C_pad, I, c->act, dt, false, h, s));
    moe::GemmArgs f2 = g;
    f2.A = h; f2.a_group_stride = rI; f2.lda = I; f2.B = W2; f2.b_group_stride = HI; f2.ldb = H;
    f2.C = y; f2.c_group_stride = rH; f2.ldc = H; f2.bias = b2; f2.bias_group_stride = H; f2.N = H; f2.K = I; f2.units = units;
    MOE_TRY(moe::launch_grouped_gemm(f2, s));
    // gate: dL/dw from <dout, y>, then the softmax Jacobian
    MOE_TRY(moe::launch_bwd_gate(dout, y, topk_expert, topk_weight, slot, T, b.T_pad, H, k, E, C, C_pad, b.ldL, dt, dl, dL, s));
    // dh = gy W2^T (W2[e] read as [N = I][K = H]); da = dh * phi'(a); dxe = da W1^T (W1[e] as [N = H][K = I])
    moe::GemmArgs d1 = g;
    d1.A = gy; d1.a_group_stride = rH; d1.lda = H; d1.B = W2; d1.b_group_stride = HI; d1.ldb = H; d1.b_is_nk = true;
    d1.C = dh; d1.c_group_stride = rI; d1.ldc = I; d1.N = I; d1.K = H;
    MOE_TRY(moe::launch_grouped_gemm(d1, s));
    MOE_TRY(moe::launch_bwd_act(a, dh, demand, E, C, C_pad, I, c->act, dt, true, dh, s));
    moe::GemmArgs d2 = g;
    d2.A = dh; d2.a_group_stride = rI; d2.lda = I; d2.B = W1; d2.b_group_stride = HI; d2.ldb = I; d2.b_is_nk = true;
    d2.C = y; d2.c_group_stride = rH; d2.ldc = H; d2.N = H; d2.K = I;       // dxe takes y's place
    MOE_TRY(moe::launch_grouped_gemm(d2, s));
    // weight gradients as row-major GEMMs over all C_pad rows (rows beyond the live ones are zero in gy and da):
    // dW2[e] = h[e]^T gy[e], dW1[e] = xe[e]^T da[e]
    MOE_TRY(moe::launch_bwd_transpose(h, hT, E, C_pad, I, C_pad, dt, s));
    MOE_TRY(moe::launch_bwd_transpose(xe, xeT, E, C_pad, H, C_pad, dt, s));
    // 16-bit storage: row counts and lists of row tiles, so that the persistent weight-streaming kernel takes them (each
    // GEMM writes E H I floats from a contraction over only C_pad rows: its stores must overlap the next tile's loads)
    int32_t* wrows = (int32_t*)ws_at(ws, b.off_wrows);
    int32_t *wunits1 = nullptr, *wunits2 = nullptr;
    if (dt != MOE_F32) {
        wunits1 = (int32_t*)ws_at(ws, b.off_wunits1);
        wunits2 = (int32_t*)ws_at(ws, b.off_wunits2);
        MOE_TRY(moe::launch_bwd_fill_rows(wrows, E, H, I, s));
        MOE_TRY(moe::launch_ffn_units(wrows, H, E, H, wunits1, s));
        MOE_TRY(moe::launch_ffn_units(wrows + E, I, E, I, wunits2, s));
    }
    moe::GemmArgs w{};
    w.rows_dev = nullptr; w.groups = E; w.dtype = dt; w.act = MOE_ACT_IDENTITY; w.c_f32 = true; w.K = C_pad; w.lda = C_pad;
    moe::GemmArgs w2 = w;
    if (wunits2) { w2.rows_dev = wrows + E; w2.units = wunits2; }
    w2.A = hT; w2.a_group_stride = rI; w2.a_rows_total = I; w2.rows_fixed = I; w2.rows_cap = I; w2.max_rows = I;
    w2.B = gy; w2.b_group_stride = rH; w2.ldb = H; w2.C = dW2; w2.c_group_stride = HI; w2.ldc = H; w2.N = H;
    MOE_TRY(moe::launch_grouped_gemm(w2, s));
    moe::GemmArgs w1 = w;
    if (wunits1) { w1.rows_dev = wrows; w1.units = wunits1; }
    w1.A = xeT; w1.a_group_stride = rH; w1.a_rows_total = H; w1.rows_fixed = H; w1.rows_cap = H; w1.max_rows = H;
    w1.B = dh; w1.b_group_stride = rI; w1.ldb = I; w1.C = dW1; w1.c_group_stride = HI; w1.ldc = I; w1.N = I;
    MOE_TRY(moe::launch_grouped_gemm(w1, s));
    MOE_TRY(moe::launch_bwd_colsum(gy, demand, E, C, C_pad, H, dt, db2, s));
    MOE_TRY(moe::launch_bwd_colsum(dh, demand, E, C, C_pad, I, dt, db1, s));
    // gate weights: dWg = x^T dL, dgate_bias = column sums of dl
    MOE_TRY(moe::launch_bwd_transpose(x, xT, 1, T, H, b.T_pad, dt, s));
    moe::GemmArgs wg{};
    wg.rows_dev = nullptr; wg.groups = 1; wg.dtype = dt; wg.act = MOE_ACT_IDENTITY; wg.c_f32 = true;
    wg.A = xT; wg.lda = b.T_pad; wg.a_rows_total = H; wg.rows_fixed = H; wg.rows_cap = H; wg.max_rows = H;
    wg.B = dL; wg.ldb = b.ldL; wg.C = dWg; wg.ldc = E; wg.N = E; wg.K = T;
    if (b.wg_slices > 1) {
        float* part = (float*)ws_at(ws, b.off_wg_part);
        wg.groups = b.wg_slices; wg.K = b.wg_slice_k;
        wg.a_group_stride = b.wg_slice_k;                // slice g of every row of x^T
        wg.b_group_stride = (long long)b.wg_slice_k * b.ldL;
        wg.C = part; wg.c_group_stride = (long long)H * E;
        MOE_TRY(moe::launch_grouped_gemm(wg, s));
        MOE_TRY(moe::launch_bwd_sum_slices(part, b.wg_slices, (long long)H * E, dWg, s));
    } else {
        MOE_TRY(moe::launch_grouped_gemm(wg, s));
    }
    MOE_TRY(moe::launch_bwd_gate_bias(topk_expert, dl, T, k, E, dgate_bias, s));
    // dx: the kept choices' rows of dxe plus the gate path
    MOE_TRY(moe::launch_bwd_dx(y, wgt, topk_expert, slot, dl, T, H, k, E, C, C_pad, dt, dx, s));
#undef MOE_TRY
    return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported configuration";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_HIP: return "HIP launch error";
        case MOE_ERR_FFN_DEPENDENCY_TIMEOUT: return "single-launch FFN: a wait for first-task tiles gave up (results invalid)";
        case MOE_ERR_FFN_PLACEMENT: return "single-launch FFN: workgroups of one class ran on different XCDs (results may be stale)";
        case MOE_ERR_STATIC_SCRATCH_TOO_SMALL: return "configuration needs more than the fixed scratch of the no-allocation entry point";
    }
    return "unknown status";
}

int32_t moe_row_tile(void) { return kRowTile; }

moe_status moe_init(void) {
    hipError_t e = moe::prepare_gate_fused();
    if (e == hipSuccess) e = moe::prepare_grouped_gemm();
    if (e == hipSuccess) e = moe::prepare_grouped_gemm_stream();
    if (e == hipSuccess) e = moe::prepare_layer_fused();
    if (e == hipSuccess) e = moe::prepare_gemm_f32();
    void* scratch_here = nullptr;
    if (e == hipSuccess) e = static_scratch(&scratch_here);
    if (e != hipSuccess) return MOE_ERR_HIP;
    (void)moe::device_cu_count();
    return MOE_OK;
}

int32_t moe_ffn_schedule(int32_t large_list, int32_t n_units_large, int32_t n_units_small, int32_t nrow_large,
                         int32_t ncol, int32_t xcd, int32_t wg, int32_t wgs, int32_t* list_index, int32_t* col_tile,
                         int32_t max_tasks) {
    if (n_units_large < 0 || n_units_small < 0 || nrow_large < 0 || ncol <= 0 || xcd < 0 || xcd >= moe::kXcds ||
        wgs <= 0 || wg < 0 || wg >= wgs || max_tasks < 0 || (max_tasks > 0 && (!list_index || !col_tile)))
        return -1;
    int unit0, unit_step, ux_l, ux;
    moe::ffn_xcd_share(true, n_units_large, nrow_large, xcd, unit0, unit_step, ux_l);
    int w = wg, handicap = 0;
    if (large_list) {
        ux = ux_l;
    } else {
        moe::ffn_xcd_share(false, n_units_small, 1, xcd, unit0, unit_step, ux);
        w = moe::ffn_small_list_rotation(wg, wgs, ux_l, ncol);
        handicap = moe::ffn_small_list_handicap(wgs, ux_l, ncol);
    }
    if ((long long)ux * ncol > 0x7fffffffLL - 2ll * wgs) return -1;
    const int n = moe::ffn_slot_count(w, wgs, handicap, ux * ncol);
    const int first = moe::ffn_first_slot(w, wgs, handicap);
    for (int j = 0; j < n && j < max_tasks; ++j)
        moe::ffn_task_at(moe::ffn_slot_position(first + j * wgs, wgs, handicap), ncol, unit0, unit_step, list_index[j], col_tile[j]);
    return n;
}

int32_t moe_f32_ffn_schedule(const int32_t* rows, int32_t groups, int32_t capacity, int32_t N, int32_t K, int32_t workgroups,
                             int64_t* first_iteration, int64_t* fix_tile, int32_t* unit_id, int32_t* unit_cum, int32_t max_units) {
    if (!rows || groups <= 0 || capacity <= 0 || N <= 0 || K <= 0 || workgroups <= 0 || !first_iteration || !fix_tile || !unit_id ||
        !unit_cum || (long long)groups * moe::f32_units_nrow(capacity) > max_units)
        return -1;
    const int n = moe::f32_build_units_host(rows, capacity, groups, capacity, unit_id, unit_cum);
    const moe::F32Work k(unit_id, unit_cum, n, (N + moe::kF32TileCols - 1) / moe::kF32TileCols, (K + moe::kF32TileK - 1) / moe::kF32TileK);
    for (int w = 0; w <= workgroups; ++w) first_iteration[w] = k.boundary(w, workgroups);
    for (int w = 0; w < workgroups; ++w) fix_tile[w] = k.tile_to_fix(first_iteration[w], first_iteration[w + 1]);
    return n;
}

moe_status moe_ffn_status(const moe_config* cfg, const void* workspace, size_t workspace_bytes, void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (!workspace || misaligned(workspace)) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (cfg->dtype == MOE_F32) return MOE_OK;            // the unit lists (and their fault words) belong to the 16-bit kernels
    long long w0 = 0, w1 = 0;
    moe::ffn_units_fault_words(cfg->E, p.C, &w0, &w1);
    const int32_t* units = (const int32_t*)((const char*)workspace + p.off_units);
    int32_t f0 = 0, f1 = 0;
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(&f0, units + w0, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(&f1, units + w1, sizeof(int32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return MOE_ERR_HIP;
    const int32_t f = f0 | f1;
    if ((f & 1) && (cfg->flags & MOE_FLAG_LAYER_SINGLE_LAUNCH)) {
        // a device-wide barrier of the single-launch layer may have been left half-way: start the next launch clean
        if (moe::reset_layer_sync(s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return MOE_ERR_HIP;
    }
    if (f & 1) return MOE_ERR_FFN_DEPENDENCY_TIMEOUT;
    if (f & 2) return MOE_ERR_FFN_PLACEMENT;
    return MOE_OK;
}

moe_status moe_layer_stage_ms(double* host_ms, int32_t n, void* stream) {
    if (!host_ms || n < 0 || n > MOE_LAYER_STAGES) return MOE_ERR_INVALID_ARG;
    return moe::layer_stage_ms(host_ms, n, (hipStream_t)stream) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

moe_status moe_capacity(const moe_config* cfg, int32_t* C, int32_t* C_pad) {
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    int c = 0, cp = 0;
    st = capacity_of(cfg, &c, &cp);
    if (st != MOE_OK) return st;
    if (C) *C = c;
    if (C_pad) *C_pad = cp;
    return MOE_OK;
}

moe_status moe_workspace_bytes(const moe_config* cfg, size_t* bytes) {
    if (!bytes) return MOE_ERR_INVALID_ARG;
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    *bytes = p.total;
    return MOE_OK;
}

moe_status moe_forward(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x,
                       const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                       const void* W2, const void* b2, void* out, float* gate_logits,
                       int32_t* topk_expert, float* topk_weight, int32_t* slot, int32_t* expert_demand,
                       void* stream) {
    return forward_impl(cfg, workspace, workspace_bytes, x, Wg, gate_bias, W1, b1, W2, b2, out, gate_logits, topk_expert,
                        topk_weight, slot, expert_demand, nullptr, (hipStream_t)stream);
}

moe_status moe_forward_timed(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x,
                             const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                             const void* W2, const void* b2, void* out, float* gate_logits,
                             int32_t* topk_expert, float* topk_weight, int32_t* slot, int32_t* expert_demand,
                             void* const* events, void* stream) {
    if (!events) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < MOE_FORWARD_EVENTS; ++i)
        if (!events[i]) return MOE_ERR_INVALID_ARG;
    return forward_impl(cfg, workspace, workspace_bytes, x, Wg, gate_bias, W1, b1, W2, b2, out, gate_logits, topk_expert,
                        topk_weight, slot, expert_demand, (const hipEvent_t*)events, (hipStream_t)stream);
}

moe_status moe_gate(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x,
                    const void* Wg, const float* gate_bias, float* gate_logits, int32_t* topk_expert,
                    float* topk_weight, void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({workspace, x, Wg, gate_logits, topk_expert, topk_weight}) || bad_optional({gate_bias}))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    return run_gate(cfg, p, workspace, x, Wg, gate_bias, gate_logits, topk_expert, topk_weight, nullptr, (hipStream_t)stream);
}

moe_status moe_route(const moe_config* cfg, const float* gate_logits, int32_t* topk_expert,
                     float* topk_weight, void* stream) {
    moe_status st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (bad_required({gate_logits, topk_expert, topk_weight})) return MOE_ERR_INVALID_ARG;
    return hip_status(moe::launch_topk(gate_logits, cfg->T, cfg->E, cfg->k, topk_expert, topk_weight, (hipStream_t)stream));
}

moe_status moe_dispatch(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x,
                        const int32_t* topk_expert, const float* topk_weight, int32_t* slot,
                        int32_t* expert_demand, int32_t* slot_token, float* slot_weight, void* xe,
                        void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({workspace, topk_expert, topk_weight, slot, expert_demand, slot_token, slot_weight}) ||
        bad_optional({x, xe}) || (xe && !x))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    return run_dispatch(cfg, p, (int32_t*)ws_at(workspace, p.off_counts), nullptr, x, topk_expert, topk_weight, slot,
                        expert_demand, slot_token, slot_weight, xe, false, (hipStream_t)stream);
}

moe_status moe_dispatch_noalloc(const moe_config* cfg, const void* x, const int32_t* topk_expert,
                                const float* topk_weight, int32_t* slot, int32_t* expert_demand, int32_t* slot_token,
                                float* slot_weight, void* xe, void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({topk_expert, topk_weight, slot, expert_demand, slot_token, slot_weight}) || bad_optional({x, xe}) ||
        (xe && !x))
        return MOE_ERR_INVALID_ARG;
    // the only scratch of the routing kernels: per-chunk expert counts (every entry is written before it is read,
    // so nothing of an earlier call has to be cleared)
    const size_t need = (size_t)moe::route_chunks(cfg->T) * (size_t)cfg->E * sizeof(int32_t);
    if (need > kStaticScratchBytes) return MOE_ERR_STATIC_SCRATCH_TOO_SMALL;
    void* counts = nullptr;
    if (static_scratch(&counts) != hipSuccess) return MOE_ERR_HIP;
    return run_dispatch(cfg, p, (int32_t*)counts, nullptr, x, topk_expert, topk_weight, slot, expert_demand, slot_token,
                        slot_weight, xe, false, (hipStream_t)stream);
}

moe_status moe_expert_ffn(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* xe,
                          const int32_t* expert_demand, const void* W1, const void* b1, const void* W2,
                          const void* b2, void* y, void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({workspace, xe, expert_demand, W1, W2, y}) || bad_optional({b1, b2})) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    st = check_single_launch(cfg, p, false);
    if (st != MOE_OK) return st;
    return run_ffn(cfg, p, workspace, xe, nullptr, expert_demand, W1, b1, W2, b2, y, false, nullptr, (hipStream_t)stream);
}

moe_status moe_backward_workspace_bytes(const moe_config* cfg, size_t* bytes) {
    if (!bytes) return MOE_ERR_INVALID_ARG;
    BwdPlan b;
    moe_status st = make_bwd_plan(cfg, &b);
    if (st != MOE_OK) return st;
    *bytes = b.total;
    return MOE_OK;
}

moe_status moe_backward(const moe_config* cfg, void* workspace, size_t workspace_bytes, const void* x, const void* Wg,
                        const void* W1, const void* b1, const void* W2, const void* b2, const int32_t* topk_expert,
                        const float* topk_weight, const void* dout, float* dx, float* dWg, float* dgate_bias, float* dW1,
                        float* db1, float* dW2, float* db2, void* stream) {
    BwdPlan b;
    moe_status st = make_bwd_plan(cfg, &b);
    if (st != MOE_OK) return st;
    if (bad_required({workspace, x, Wg, W1, W2, topk_expert, topk_weight, dout, dx, dWg, dgate_bias, dW1, db1, dW2, db2}) ||
        bad_optional({b1, b2}))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < b.total) return MOE_ERR_WORKSPACE_TOO_SMALL;
    return run_backward(cfg, b, workspace, x, Wg, W1, b1, W2, b2, topk_expert, topk_weight, dout, dx, dWg, dgate_bias, dW1, db1,
                        dW2, db2, (hipStream_t)stream);
}

moe_status moe_combine(const moe_config* cfg, const void* y, const int32_t* topk_expert,
                       const float* topk_weight, const int32_t* slot, void* out, void* stream) {
    Plan p;
    moe_status st = make_plan(cfg, &p);
    if (st != MOE_OK) return st;
    if (bad_required({y, topk_expert, topk_weight, slot, out})) return MOE_ERR_INVALID_ARG;
    return run_combine(cfg, p, y, topk_expert, topk_weight, slot, out, (hipStream_t)stream);
}

}  // extern "C"
