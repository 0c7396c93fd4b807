#!/usr/bin/env python3
"""Benchmark of the MoE layer forward on one MI355X.

A step is one pass of the whole hot path (gate -> dispatch -> expert FFNs ->
combine) through ``moe_forward`` over one batch of seeded synthetic input that is
already resident in HBM.  Prints ONE JSON line (see the keys below).  The default
workload is the configuration the headline metric is quoted on: T = 16384 tokens,
H = I = 2048, E = 128 local experts, top-2, capacity factor 1.0, bf16 storage with
fp32 accumulation.

Extra objects on the line:
  roofline       the dominant kernel (the first expert-FFN launch, x W1 + activation)
                 against its binding roof; its duration is measured INSIDE moe_forward
                 with HIP events on the launch stream (moe_forward_timed records them
                 at the stage boundaries), over as many steps as the timed region, right
                 after it;
  roofline_other the same launch priced against the other roof (MFMA peak / HBM);
  roofline_gemm2 the second FFN launch (h W2) the same way;
  forward_stage_ms  every stage of the whole-layer call from the same events;
  staged_stage_ms   the staged entry points called one by one (the staged dispatch
                 also packs xe, which moe_forward does not);
  steady_ms      the layer time once the chip has been busy for 256 steps, measured
                 after the official timed loop (`value` is the official loop alone);
  measured_peaks a read-stream, a copy and a register-resident MFMA loop run in this
                 process: what the chip sustains, next to the published peaks;
  cpu_baseline   the CPU oracle, as it stands, timed on this machine's host cores on a
                 bounded sample (a slice of the tokens, scaled to the full batch).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {  # MI355X published peaks
    "hbm_gbs": 8000.0,
    "mfma_tflops": {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3},
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the paper's protocol (Sec. 4: 32 warm-up passes, then the mean of 32)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--steady-after", type=int, default=256,
                    help="steps run after the timed region before steady_ms is measured (0 = skip)")
    ap.add_argument("--no-probes", action="store_true", help="skip the stream / MFMA yardstick kernels")
    ap.add_argument("--workload", default="paper_bf16_e128")
    ap.add_argument("--cpu-baseline-tokens", type=int, default=16384,
                    help="tokens in the oracle's timed sample (0 = skip the cpu_baseline leg)")
    ap.add_argument("--tokens", type=int, default=0, help="override T of the workload (sweeps; not the headline run)")
    ap.add_argument("--experts", type=int, default=0, help="override E of the workload")
    ap.add_argument("--hidden", type=int, default=0, help="override H of the workload")
    ap.add_argument("--inter", type=int, default=0, help="override I of the workload")
    ap.add_argument("--topk", type=int, default=0, help="override k of the workload")
    ap.add_argument("--act", default="", help="override the activation (relu, gelu_tanh, gelu_erf, identity)")
    ap.add_argument("--with-bias", action="store_true", help="give the experts bias vectors b1, b2")
    ap.add_argument("--capacity-factor", type=float, default=0.0, help="override the capacity factor of the workload")
    ap.add_argument("--capacity-mode", default="", help="per_choice (C = ceil(cf k T / E), default) or layout (no factor k)")
    ap.add_argument("--drop-policy", default="", help="token_major (default) or choice_major")
    ap.add_argument("--single-launch-ffn", action="store_true",
                    help="both FFN GEMMs in one persistent launch (MOE_FLAG_FFN_SINGLE_LAUNCH)")
    ap.add_argument("--lib", default="", help="load this build of the library instead of the product (layout studies; see build.py --define)")
    ap.add_argument("--backward", action="store_true",
                    help="also time moe_backward (gradients under the forward's routing); reported as backward_ms, not part of value")
    ap.add_argument("--single-launch-layer", action="store_true",
                    help="the whole layer from one persistent launch (MOE_FLAG_LAYER_SINGLE_LAUNCH)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a captured HIP graph in the timed loop (the same kernels, one launch call)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy kernel (moe_probe_stream with a destination: the "
                         "reference for hardware traffic counters)")
    return ap.parse_args()


def read_traffic(workload, dtype):
    """HBM bytes per launch of the dominant kernel, from the committed counter summary (or None)."""
    path = os.path.join(ROOT, "profiles", "ffn_gemm_stream_%s_%s_traffic.txt" % (dtype, workload))
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the layer on ONE GPU; --gpus %d is not supported "
              "(no collectives are part of this build)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_04667_amd import binding as moe
    from paper_2506_04667_amd.inputs import WORKLOADS, make_inputs, scaled

    w = WORKLOADS[args.workload]
    over = {}
    if args.tokens > 0: over["T"] = args.tokens
    if args.experts > 0: over["E"] = args.experts
    if args.hidden > 0: over["H"] = args.hidden
    if args.inter > 0: over["I"] = args.inter
    if args.topk > 0: over["k"] = args.topk
    if args.act: over["act"] = args.act
    if args.with_bias: over["with_bias"] = True
    if args.capacity_factor > 0: over["capacity_factor"] = args.capacity_factor
    if args.capacity_mode: over["capacity_mode"] = args.capacity_mode
    if args.drop_policy: over["drop_policy"] = args.drop_policy
    if args.single_launch_ffn: over["flags"] = 1
    if args.single_launch_layer: over["flags"] = 4
    if over:
        w = scaled(w, name=w.name + "+" + ",".join("%s=%s" % kv for kv in sorted(over.items())), **over)
    if args.lib:
        moe._LIB = moe.load(args.lib)
    moe.load()
    torch.cuda.set_device(0)
    t0 = time.time()
    cpu = make_inputs(w)
    dev = {n: (None if v is None else v.to("cuda")) for n, v in cpu.items()}
    gen_s = time.time() - t0

    cfg = moe.config_of(w)
    b = moe.Buffers(cfg).alloc_staged()

    def step():
        moe.moe_forward(cfg, b.workspace, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["b1"], dev["W2"],
                        dev["b2"], b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot, b.expert_demand)

    moe.moe_init()
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        moe.moe_probe_stream(src, dst, sink)
        torch.cuda.synchronize()
        del src, dst

    run_step = step
    if args.graph:
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        run_step = graph.replay

    def timed(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            run_step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    # ---- the official protocol: W untimed steps, then exactly K timed ones
    for _ in range(args.warmup):
        run_step()
    ms_per_step = timed(args.steps)

    # ---- the same K steps again with events at the stage boundaries inside moe_forward
    NE = moe.FORWARD_EVENTS
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(NE)] for _ in range(args.steps)]
    handles = [moe.event_handles(e) for e in ev]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for h in handles:
        moe.moe_forward_timed(cfg, b.workspace, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["b1"], dev["W2"],
                              dev["b2"], b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot, b.expert_demand, h)
    torch.cuda.synchronize()
    ms_with_events = (time.perf_counter() - t0) * 1e3 / args.steps
    names = ["gate", "route", "ffn_gemm1", "ffn_gemm2", "combine"]
    fwd_ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in ev) / args.steps for i, n in enumerate(names)}
    fwd_ms["layer"] = sum(e[0].elapsed_time(e[NE - 1]) for e in ev) / args.steps
    layer_stage_ms = None
    if getattr(w, "flags", 0) & 4:                                 # the one launch's own stage clocks (last step, workgroup 0)
        layer_stage_ms = {n: round(v, 4) for n, v in moe.moe_layer_stage_ms().items()}

    # ---- per-stage times of the staged entry points (the same kernels, called one by one)
    stage_calls = [
        ("gate", lambda: moe.moe_gate(cfg, b.workspace, dev["x"], dev["Wg"], dev["gate_bias"], b.gate_logits,
                                      b.topk_expert, b.topk_weight)),
        ("dispatch", lambda: moe.moe_dispatch(cfg, b.workspace, dev["x"], b.topk_expert, b.topk_weight, b.slot,
                                              b.expert_demand, b.slot_token, b.slot_weight, b.xe)),
        ("expert_ffn", lambda: moe.moe_expert_ffn(cfg, b.workspace, b.xe, b.expert_demand, dev["W1"], dev["b1"],
                                                  dev["W2"], dev["b2"], b.y)),
        ("combine", lambda: moe.moe_combine(cfg, b.y, b.topk_expert, b.topk_weight, b.slot, b.out)),
    ]
    stage_ms = {n: 0.0 for n, _ in stage_calls}
    events = []
    for _ in range(args.steps):
        for n, call in stage_calls:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            call()
            e1.record()
            events.append((n, e0, e1))
    torch.cuda.synchronize()
    for n, e0, e1 in events:
        stage_ms[n] += e0.elapsed_time(e1) / args.steps

    # ---- steady state: the layer once the chip has been busy for a while (not part of `value`)
    steady_ms = None
    if args.steady_after > 0:
        for _ in range(args.steady_after):
            run_step()
        steady_ms = timed(max(args.steps, 32))

    # ---- backward pass (optional; the metric is the forward latency)
    backward = None
    if args.backward:
        f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
        grads = [f32(w.T, w.H), f32(w.H, w.E), f32(w.E), f32(w.E, w.H, w.I), f32(w.E, w.I), f32(w.E, w.I, w.H), f32(w.E, w.H)]
        bws = torch.empty(moe.moe_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        dout = torch.randn((w.T, w.H), device="cuda").to(dev["x"].dtype)

        def bstep():
            moe.moe_backward(cfg, bws, dev["x"], dev["Wg"], dev["W1"], dev["b1"], dev["W2"], dev["b2"], b.topk_expert,
                             b.topk_weight, dout, *grads)
        for _ in range(3):
            bstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nb = max(4, args.steps // 4)
        for _ in range(nb):
            bstep()
        torch.cuda.synchronize()
        bms = (time.perf_counter() - t0) * 1e3 / nb
        kept = int((b.slot >= 0).sum())
        backward = {"backward_ms": round(bms, 4), "steps": nb, "workspace_bytes": bws.numel(),
                    # recomputed forward (4 R H I) + data gradients (4 R H I) + weight gradients (4 R H I on the live rows)
                    "gemm_tflops_on_live_rows": round(12.0 * kept * w.H * w.I / (bms * 1e-3) / 1e12, 1)}
        del grads, bws, dout

    # ---- yardsticks measured in this run: streaming read, copy, MFMA loop
    measured = None
    if not args.no_probes:
        def ev_time(fn, reps):
            fn()
            pairs = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                pairs.append((e0, e1))
            torch.cuda.synchronize()
            t = sorted(a.elapsed_time(c) for a, c in pairs)
            return t[len(t) // 2]                                  # median ms
        src = dev["W1"].view(torch.uint8).reshape(-1)
        src = src[: min(src.numel(), 1 << 30) // 16 * 16]
        dst = torch.empty_like(src)
        rd = ev_time(lambda: moe.moe_probe_stream(src, None, sink), 20)
        cp = ev_time(lambda: moe.moe_probe_stream(src, dst, sink), 20)
        del dst
        iters = 20000 if w.dtype != "f32" else 3000
        flops = [0.0]
        def mf():
            flops[0] = moe.moe_probe_mfma(w.dtype, iters, sink)
        mm = ev_time(mf, 5)
        # L2 -> LDS fill rate per CU by the two routes (2 MiB per XCD, resident in its L2 after the first lap)
        region, fsteps = 2 << 20, 512
        moved = [0.0]
        def fill(mode):
            def f():
                moved[0] = moe.moe_probe_lds_fill(mode, src, region, fsteps, sink)
            return f
        fills = {}
        for mode, name in ((0, "direct_copy"), (1, "load_then_ds_write"), (2, "load_only")):
            ms = ev_time(fill(mode), 5)
            fills[name] = round(moved[0] / (ms * 1e-3) / 1e9, 1)
        measured = {"stream_read_gbs": round(src.numel() / (rd * 1e-3) / 1e9, 1),
                    "stream_copy_gbs_read_plus_write": round(2 * src.numel() / (cp * 1e-3) / 1e9, 1),
                    "mfma_loop_tflops": round(flops[0] / (mm * 1e-3) / 1e12, 1), "mfma_dtype": w.dtype,
                    "l2_to_lds_fill_gbs": fills,
                    "bytes": src.numel(), "kernels": "moe_probe_stream / moe_probe_mfma / moe_probe_lds_fill (csrc/probes.hip)"}

    slot = b.slot.cpu()
    demand = b.expert_demand.cpu()
    R = int((slot >= 0).sum())
    dropped = int((slot < 0).sum())
    el = 4 if w.dtype == "f32" else 2
    H, I, E, T, k = w.H, w.I, w.E, w.T, w.k

    # dominant kernel: the expert-FFN GEMM, two launches per step (x W1 + activation, then h W2); durations are
    # those measured inside moe_forward
    ffn_ms = fwd_ms["ffn_gemm1"] + fwd_ms["ffn_gemm2"]
    live = int((demand > 0).sum())                                 # experts nobody picked cost no weight traffic
    traffic = read_traffic(w.name, w.dtype)
    kname = "ffn_gemm_stream_kernel" if w.dtype != "f32" else "grouped_gemm_kernel, or ffn_f32_stream_kernel with its fix-up pass"

    def roofs(launch_ms, K, N, which):
        flops = 2.0 * R * K * N
        nbytes = (live * K * N + R * K + R * N) * el             # weights once + A rows read + C rows written
        gbs = nbytes / (launch_ms * 1e-3) / 1e9
        tf = flops / (launch_ms * 1e-3) / 1e12
        hbm = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
               "frac": round(gbs / PEAK["hbm_gbs"], 4), "traffic": traffic,
               "traffic_source": None if traffic is None else "committed rocprofv3 --pmc summary under profiles/ (not a counter of this run)",
               "kernel": "%s (%s, inside moe_forward)" % (kname, which), "launch_ms": round(launch_ms, 4),
               "algorithmic_bytes_per_launch": nbytes}
        if measured:
            hbm["measured_stream_read_peak"] = measured["stream_read_gbs"]
            hbm["frac_of_measured"] = round(gbs / measured["stream_read_gbs"], 4)
        mfma = {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK["mfma_tflops"][w.dtype], "unit": "TFLOP/s",
                "frac": round(tf / PEAK["mfma_tflops"][w.dtype], 4), "traffic": traffic,
                "kernel": "%s (%s, inside moe_forward)" % (kname, which), "launch_ms": round(launch_ms, 4),
                "algorithmic_flops_per_launch": flops}
        if measured:
            mfma["measured_mfma_loop_peak"] = measured["mfma_loop_tflops"]
            mfma["frac_of_measured"] = round(tf / measured["mfma_loop_tflops"], 4)
        binding_is_hbm = nbytes / (PEAK["hbm_gbs"] * 1e9) >= flops / (PEAK["mfma_tflops"][w.dtype] * 1e12)
        return (hbm, mfma) if binding_is_hbm else (mfma, hbm)

    flags = getattr(w, "flags", 0)
    if flags & 4:                                                  # one launch does the whole layer: the events see only its ends
        roofline, other = roofs(fwd_ms["layer"] / 2.0, H, I, "whole layer in one launch: half its duration, an upper "
                                "bound on one FFN GEMM's time")
        roofline2 = None
    elif flags & 1:                                                # one launch does both GEMMs: price them together
        roofline, other = roofs(ffn_ms / 2.0, H, I, "both FFN GEMMs in one launch: half its duration")
        roofline2 = None
    else:
        roofline, other = roofs(fwd_ms["ffn_gemm1"], H, I, "first FFN launch: x W1 + activation")
        roofline2, _ = roofs(fwd_ms["ffn_gemm2"], I, H, "second FFN launch: h W2")

    # achieved HBM rate of the bandwidth-bound stages: algorithmic bytes / stage time
    C = b.C
    stage_bytes = {
        "gate": T * H * el + H * E * el + T * E * 4 + T * k * 8,
        # the staged dispatch call packs xe as well (moe_forward gathers inside the first GEMM instead)
        "dispatch": T * k * 4 + (T * k + 2 * E * C + E) * 4 + T * H * el + R * H * el,
        "combine": R * H * el + T * k * 12 + T * H * el,
    }
    stage_gbs = {n: round(v / (stage_ms[n] * 1e-3) / 1e9, 1) for n, v in stage_bytes.items()}
    # the same for the stages as they run inside moe_forward (no packing there: routing tables only)
    fwd_bytes = {"gate": stage_bytes["gate"], "route": T * k * 4 + (T * k + 2 * E * C + E) * 4, "combine": stage_bytes["combine"]}
    fwd_gbs = {n: round(v / (max(fwd_ms[n], 1e-6) * 1e-3) / 1e9, 1) for n, v in fwd_bytes.items()}

    cpu_baseline = None
    if args.cpu_baseline_tokens > 0:
        from oracle import load_oracle
        oracle = load_oracle()
        Ts = min(args.cpu_baseline_tokens, T)
        ws = scaled(w, T=Ts)
        xs = cpu["x"][:Ts].contiguous()
        gb = None if cpu["gate_bias"] is None else cpu["gate_bias"].numpy()
        t0 = time.perf_counter()
        oracle.forward(xs, cpu["Wg"], gb, cpu["W1"], cpu["b1"], cpu["W2"], cpu["b2"], Ts, H, I, E, k,
                       ws.capacity_factor, w.act, w.dtype, capacity_override=moe.moe_capacity(cfg)[0])
        sec = time.perf_counter() - t0
        cpu_baseline = {"value": round(sec * 1e3 * T / Ts, 1), "unit": "ms", "cores": oracle.get_threads(),
                        "kind": "oracle",
                        "sample": "oracle_forward on the first %d of %d tokens with the full weights "
                                  "(%.1f s measured), scaled by T/%d" % (Ts, T, sec, Ts)}

    line = {
        "metric": "MoE fwd latency (ms) + expert-FFN TFLOPS & % MFMA peak, T=16K E=128 k=2",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic", "launch": "hip_graph_replay" if args.graph else "stream",
        "config": {"workload": w.name, "T": T, "H": H, "I": I, "E": E, "k": k,
                   "capacity_factor": w.capacity_factor, "act": w.act, "capacity": b.C,
                   "capacity_mode": w.capacity_mode, "drop_policy": w.drop_policy},
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "kept_rows": R, "dropped_pairs": dropped,
        "expert_demand": {"min": int(demand.min()), "median": int(demand.median()), "max": int(demand.max()),
                          "empty": E - live},
        "ms_per_step_with_events": round(ms_with_events, 4),
        "steady_ms": None if steady_ms is None else round(steady_ms, 4),
        "forward_stage_ms": {n: round(v, 4) for n, v in fwd_ms.items()},
        "single_launch_layer_stage_ms": layer_stage_ms,
        "forward_stage_hbm_gbs": fwd_gbs,
        "staged_stage_ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "staged_stage_hbm_gbs": stage_gbs,
        "ffn_tflops": round(4.0 * R * H * I / (ffn_ms * 1e-3) / 1e12, 1),
        "ffn_mfma_frac": round(4.0 * R * H * I / (ffn_ms * 1e-3) / 1e12 / PEAK["mfma_tflops"][w.dtype], 4),
        "roofline": roofline,
        "roofline_other": other,
        "roofline_gemm2": roofline2,
        "measured_peaks": measured,
        "backward": backward,
        "cpu_baseline": cpu_baseline,
        "input_gen_s": round(gen_s, 1),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
