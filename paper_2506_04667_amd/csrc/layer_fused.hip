// The whole layer in ONE launch (Alg. 1 on one GPU: FusedGate, Dispatch, the processors' GEMM tasks, combine):
// a persistent kernel, one workgroup per CU, that walks the same stages as the six launches of the default path
// -- the same device functions, so the same bits -- separated by device-wide barriers where a stage reads what
// workgroups on other XCDs wrote:
//
//   gate tiles (64 tokens each)                      -> logits, top-k, combine weights, per-chunk expert counts
//   ---- barrier ----
//   scan (one wavefront per expert) + table clearing -> chunk bases, expert_demand
//   ---- barrier ----
//   scatter (one wavefront per chunk) + unit lists   -> slot, routing table, lists of live (expert, row tile) units
//   ---- barrier ----
//   first-GEMM tasks, then second-GEMM tasks         -> h, y; a second-GEMM task waits for its unit's first-GEMM
//                                                       tiles by completion counter (no barrier in between)
//   ---- barrier ----
//   combine (one wavefront per token at a time)      -> out
//
// The paper's kernel needs its scheduler and subscriber because tasks arrive from peers at unknown times; on one
// GPU the stage boundaries are the only global dependencies, so four barriers replace them.  A barrier is an
// arrival counter and a generation word in device memory: every thread makes its stores visible device-wide
// (agent-scope release: the XCD's L2 is written back), the workgroup's first thread arrives and polls the
// generation, and everybody then drops stale lines (agent-scope acquire).  The polls are bounded; a give-up sets
// the fault word that moe_ffn_status reports.  All workgroups must be resident at once (one per CU, never more
// workgroups than CUs; 160 KB of LDS each keeps a second one off a CU), and launches of this kernel must not
// overlap on one GPU: they share the barrier words.
#include "combine_body.h"
#include "gate_fused_body.h"
#include "gemm_stream_body.h"
#include "route_body.h"

// Barrier state of the single-launch layer: { arrivals, generation }.  A fixed array in device memory, zero when
// the code object is loaded; every barrier leaves the arrival count at zero again.  In host code this name is only
// a handle for hipGetSymbolAddress.  Words 16.. hold workgroup 0's wall-clock stamps of the last launch (kLayerStamps
// of 64 bits each), which moe_layer_stage_ms turns into stage times.
static __device__ __align__(256) int32_t layer_sync[64];

namespace moe {
namespace {

constexpr int L_THREADS = 512, L_WAVES = L_THREADS / 64;
constexpr int L_GATE_BN = 128;                          // experts covered by the gate tile of this kernel
constexpr int kLayerStamps = 11, kLayerStampWord = 16;  // stamps of workgroup 0: start, before/after each barrier, ...

// Workgroup 0 notes the constant-rate wall clock at the stage boundaries it passes.
__device__ __forceinline__ void stamp(int32_t* sync, int i) {
    if (blockIdx.x == 0 && threadIdx.x == 0) ((long long*)(sync + kLayerStampWord))[i] = (long long)wall_clock64();
}

struct LayerArgs {
    const unsigned char* x; const unsigned char* Wg; const float* gate_bias;
    int T, H, E, k, C, C_pad;
    float* logits; int32_t* topk_expert; float* topk_weight;
    int32_t* counts;                                    // [chunks][E] scratch of the slot assignment
    int32_t* slot; int32_t* expert_demand; int32_t* slot_token; float* slot_weight;
    StreamArgs ffn;                                     // both GEMMs; lists = the unit-list scratch block
    void* out;
    int32_t* sync;                                      // { arrivals, generation }
};

// Device-wide barrier for a grid whose workgroups are all resident.  Every thread calls it.
// The workgroup barrier orders every thread's stores before thread 0 (they have reached the XCD's L2 by then: the
// vector L1 writes through), so thread 0's agent-scope release, which writes that L2 back, covers them all: one
// write-back per workgroup instead of one per wavefront.  Likewise thread 0's agent-scope acquire drops the stale
// lines of the CU's L1 and of the L2 before the second workgroup barrier lets the other wavefronts read.
__device__ __forceinline__ void grid_barrier(int32_t* sync, int nblocks, int spin_limit, int32_t* fault) {
    __syncthreads();
    if (threadIdx.x == 0) {
        // read the generation, then arrive: it cannot advance before this workgroup has arrived
        const int gen = __hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__hip_atomic_fetch_add(sync, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == nblocks - 1) {
            __hip_atomic_store(sync, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(sync + 1, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            int spins = 0;
            while (__hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gen) {
                if (++spins > spin_limit) {
                    __hip_atomic_fetch_or(fault, kFaultWaitGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

template <class S, int ACT>
__global__ __launch_bounds__(L_THREADS) void moe_layer_kernel(LayerArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int nb = gridDim.x, bid = blockIdx.x;
    const int wave_in_wg = threadIdx.x >> 6;
    const int gwave = bid * L_WAVES + wave_in_wg, waves = nb * L_WAVES;
    int32_t* const fault = a.ffn.lists + ffn_units_small_offset(a.ffn.groups, a.ffn.max_rows);
    const int n_chunks = (a.T + G_BM - 1) / G_BM;       // a gate tile is one chunk of the slot assignment

    stamp(a.sync, 0);
    // ---- gate: logits, top-k, combine weights, per-chunk expert counts
    for (int tile = bid; tile < n_chunks; tile += nb) {
        gate_fused_tile<S, L_GATE_BN>(a.x, a.Wg, a.gate_bias, a.T, a.H, a.E, a.k, a.logits, a.topk_expert, a.topk_weight, a.counts, tile);
        __syncthreads();                                // the tile's LDS is free again
    }
    stamp(a.sync, 1);
    grid_barrier(a.sync, nb, a.ffn.spin_limit, fault);
    stamp(a.sync, 2);

    // ---- slot assignment, part 1: chunk bases per expert; the routing table emptied
    route_clear_tables(a.slot_token, a.slot_weight, (long long)a.E * a.C, (long long)bid * L_THREADS + threadIdx.x, (long long)nb * L_THREADS);
    for (int e = gwave; e < a.E; e += waves) route_scan_expert(a.counts, n_chunks, a.E, e, a.expert_demand);
    stamp(a.sync, 3);
    grid_barrier(a.sync, nb, a.ffn.spin_limit, fault);
    stamp(a.sync, 4);

    // ---- slot assignment, part 2: slots and the routing table; the last workgroup also lists the live FFN units
    {
        int32_t* const run = (int32_t*)smem + wave_in_wg * a.E;        // one array of E ints per wavefront
        for (int c = gwave; c < n_chunks; c += waves)
            route_scatter_chunk(a.topk_expert, a.topk_weight, (long long)a.T * a.k, G_BM * a.k, a.T, false, a.E, a.k, a.C, a.counts, a.slot,
                                a.slot_token, a.slot_weight, c, run);
        if (bid == nb - 1) {
            __syncthreads();
            build_ffn_units(a.expert_demand, a.C, a.E, a.C, a.ffn.lists, (int*)smem, L_THREADS);
        }
    }
    stamp(a.sync, 5);
    grid_barrier(a.sync, nb, a.ffn.spin_limit, fault);
    stamp(a.sync, 6);

    // ---- expert FFNs: all first-GEMM tasks of this workgroup, then its second-GEMM tasks, each of which waits for
    // its unit's first-GEMM tiles (tile-level dependency by completion counter, as in the single-launch FFN)
    {
        const int xcd = bid % kXcds, wg = bid / kXcds, wgs = nb / kXcds;
        if (threadIdx.x == 0) check_xcd_placement(a.ffn, xcd);
        stream_gemm<S, ACT, 0, true, false>(a.ffn, xcd, wg, wgs);
        __syncthreads();
        stamp(a.sync, 7);
        stream_gemm<S, 3, 1, false, true>(a.ffn, xcd, wg, wgs);
    }
    stamp(a.sync, 8);
    grid_barrier(a.sync, nb, a.ffn.spin_limit, fault);
    stamp(a.sync, 9);

    // ---- combine
    combine_tokens<S>(a.ffn.ph[1].C, a.topk_expert, a.topk_weight, a.slot, a.T, a.H, a.k, a.E, a.C, a.C_pad, a.out, gwave, waves);
    __syncthreads();
    stamp(a.sync, 10);
}

// Device address of the barrier words on the current device, looked up once per device with that device current.
hipError_t layer_sync_ptr(int32_t** out) {
    static std::atomic<int32_t*> ptr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int32_t* p = ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(layer_sync));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

template <class S, int ACT>
hipError_t prepare_layer_t() {
    static DeviceFlags limit_raised = {};
    return raise_lds_limit(reinterpret_cast<const void*>(moe_layer_kernel<S, ACT>), LDS_BYTES, limit_raised);
}

template <class S, int ACT>
hipError_t launch_layer_t(const LayerArgs& a, long long grid, hipStream_t stream) {
    if (hipError_t e = prepare_layer_t<S, ACT>(); e != hipSuccess) return e;
    hipLaunchKernelGGL((moe_layer_kernel<S, ACT>), dim3((unsigned)grid), dim3(L_THREADS), LDS_BYTES, stream, a);
    return hipGetLastError();
}

template <class S>
hipError_t launch_layer_s(const LayerArgs& a, int act, long long grid, hipStream_t stream) {
    switch (act) {
        case 0: return launch_layer_t<S, 0>(a, grid, stream);
        case 1: return launch_layer_t<S, 1>(a, grid, stream);
        case 2: return launch_layer_t<S, 2>(a, grid, stream);
        default: return launch_layer_t<S, 3>(a, grid, stream);
    }
}

template <class S>
hipError_t prepare_layer_s() {
    hipError_t e = prepare_layer_t<S, 0>();
    if (e == hipSuccess) e = prepare_layer_t<S, 1>();
    if (e == hipSuccess) e = prepare_layer_t<S, 2>();
    if (e == hipSuccess) e = prepare_layer_t<S, 3>();
    return e;
}

}  // namespace

hipError_t prepare_layer_fused() {
    int32_t* p = nullptr;
    hipError_t e = layer_sync_ptr(&p);
    if (e == hipSuccess) e = prepare_layer_s<BF16>();
    if (e == hipSuccess) e = prepare_layer_s<F16>();
    return e;
}

hipError_t reset_layer_sync(hipStream_t stream) {
    int32_t* p = nullptr;
    if (hipError_t e = layer_sync_ptr(&p); e != hipSuccess) return e;
    return hipMemsetAsync(p, 0, 2 * sizeof(int32_t), stream);
}

hipError_t layer_stage_ms(double* ms, int n, hipStream_t stream) {
    int32_t* p = nullptr;
    if (hipError_t e = layer_sync_ptr(&p); e != hipSuccess) return e;
    long long t[kLayerStamps];
    if (hipError_t e = hipMemcpyAsync(t, p + kLayerStampWord, sizeof(t), hipMemcpyDeviceToHost, stream); e != hipSuccess) return e;
    if (hipError_t e = hipStreamSynchronize(stream); e != hipSuccess) return e;
    int dev = 0, khz = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (hipError_t e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev); e != hipSuccess) return e;
    if (khz <= 0) return hipErrorInvalidValue;
    for (int i = 0; i < n && i < kLayerStamps - 1; ++i) ms[i] = (double)(t[i + 1] - t[i]) / (double)khz;
    return hipSuccess;
}

bool layer_fused_eligible(int T, int H, int I, int ldh, int E, int k, int C_pad, int dtype) {
    static_assert(G_THREADS == L_THREADS && THREADS == L_THREADS, "every stage of the layer runs with the same workgroup size");
    static_assert(GateCfg<BF16, L_GATE_BN>::LDS_BYTES <= LDS_BYTES, "the gate tile fits in the FFN kernel's LDS");
    return dtype != 0 && E <= L_GATE_BN && gate_fused_eligible(T, H, E, k, dtype) &&
           stream_gemm_shape_ok(dtype, I, H, H, I, ldh, T) && stream_gemm_shape_ok(dtype, H, I, ldh, H, H, C_pad) &&
           (long long)L_WAVES * E * 4 + 64 * 4 <= LDS_BYTES;
}

hipError_t launch_layer_fused(const void* x, const void* Wg, const float* gate_bias, int T, int H, int E, int k, int C, int C_pad,
                              int dtype, float* logits, int32_t* topk_expert, float* topk_weight, int32_t* counts, int32_t* slot,
                              int32_t* expert_demand, int32_t* slot_token, float* slot_weight, const GemmArgs& g1, const GemmArgs& g2,
                              void* out, hipStream_t stream) {
    LayerArgs a{};
    a.x = (const unsigned char*)x; a.Wg = (const unsigned char*)Wg; a.gate_bias = gate_bias;
    a.T = T; a.H = H; a.E = E; a.k = k; a.C = C; a.C_pad = C_pad;
    a.logits = logits; a.topk_expert = topk_expert; a.topk_weight = topk_weight; a.counts = counts;
    a.slot = slot; a.expert_demand = expert_demand; a.slot_token = slot_token; a.slot_weight = slot_weight;
    a.out = out;
    a.ffn.ph[0] = to_phase(g1);
    a.ffn.ph[1] = to_phase(g2);
    a.ffn.rows_dev = g1.rows_dev; a.ffn.rows_cap = g1.rows_cap; a.ffn.max_rows = g1.max_rows;
    a.ffn.lists = const_cast<int32_t*>(g1.units);
    a.ffn.groups = g1.groups;
    a.ffn.wait_target = ((g1.N + BN - 1) / BN) * (THREADS / 64);
    a.ffn.spin_limit = kSpinLimit;
    if (hipError_t e = layer_sync_ptr(&a.sync); e != hipSuccess) return e;
    // one persistent workgroup per CU, the same number on every XCD
    const long long grid = device_cu_count() / kXcds * kXcds;
    if (grid < kXcds) return hipErrorInvalidValue;
    return dtype == 1 ? launch_layer_s<BF16>(a, g1.act, grid, stream) : launch_layer_s<F16>(a, g1.act, grid, stream);
}

}  // namespace moe
