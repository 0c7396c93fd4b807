#!/usr/bin/env python3
"""Benchmark of the MoE layer forward on one MI355X.

A step is one pass of the whole hot path (gate -> dispatch -> expert FFNs ->
combine) through ``moe_forward`` over one batch of seeded synthetic input that is
already resident in HBM.  Prints ONE JSON line (see the keys below).  The default
workload is the configuration the headline metric is quoted on: T = 16384 tokens,
H = I = 2048, E = 128 local experts, top-2, capacity factor 1.0, bf16 storage with
fp32 accumulation.

Extra objects on the line:
  roofline      the dominant kernel (the grouped FFN GEMM; two launches per step)
                against its binding roof, from HIP-event timings of the staged
                expert-FFN call over the same number of steps;
  roofline_mfma the same launches priced against the dense MFMA peak;
  cpu_baseline  the CPU oracle, as it stands, timed on this machine's host cores on a
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

MEASURED_STREAM_GBS = 6100.0

PEAK = {  # MI355X published peaks
    "hbm_gbs": 8000.0,
    "mfma_tflops": {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3},
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    # the first ~100 steps after an idle period run about 3 % slower than the steady state (the chip's power
    # management settles), so the default warm-up is longer than that
    ap.add_argument("--warmup", type=int, default=256)
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
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a captured HIP graph in the timed loop (the same kernels, one launch call)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference for hardware counters)")
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
    if over:
        w = scaled(w, name=w.name + "+" + ",".join("%s=%s" % kv for kv in sorted(over.items())), **over)
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

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    run_step = step
    if args.graph:
        step()                                                   # kernel attributes are set on first use, outside capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        run_step = graph.replay
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-stage times: the same kernels through the staged entry points, HIP events on the launch stream
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

    slot = b.slot.cpu()
    demand = b.expert_demand.cpu()
    R = int((slot >= 0).sum())
    dropped = int((slot < 0).sum())
    el = 4 if w.dtype == "f32" else 2
    H, I, E, T, k = w.H, w.I, w.E, w.T, w.k

    # dominant kernel: grouped FFN GEMM, two launches per step (x W1 then h W2)
    ffn_ms = stage_ms["expert_ffn"]
    launch_ms = ffn_ms / 2.0
    flops_per_launch = 2.0 * R * H * I
    live = int((demand > 0).sum())                                 # experts nobody picked cost no weight traffic
    bytes_per_launch = (live * H * I + R * H + R * I) * el         # weights once + A rows + C rows; the sum is the same for both launches
    hbm_time = bytes_per_launch / (PEAK["hbm_gbs"] * 1e9)
    mfma_time = flops_per_launch / (PEAK["mfma_tflops"][w.dtype] * 1e12)
    traffic = read_traffic(w.name, w.dtype)
    kernel_name = ("ffn_gemm_stream_kernel" if w.dtype != "f32" else "grouped_gemm_kernel") + " (expert FFN, 2 launches/step)"
    ach_gbs = bytes_per_launch / (launch_ms * 1e-3) / 1e9
    ach_tf = flops_per_launch / (launch_ms * 1e-3) / 1e12
    roof_hbm = {"bound": "hbm", "achieved": round(ach_gbs, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                "frac": round(ach_gbs / PEAK["hbm_gbs"], 4), "traffic": traffic,
                "kernel": kernel_name, "launch_ms": round(launch_ms, 4),
                "algorithmic_bytes_per_launch": bytes_per_launch,
                # context: the best streaming-read rate a plain copy kernel reaches on this chip (measured, GB/s)
                "measured_stream_peak": MEASURED_STREAM_GBS, "frac_of_measured": round(ach_gbs / MEASURED_STREAM_GBS, 4)}
    roof_mfma = {"bound": "mfma", "achieved": round(ach_tf, 1), "peak": PEAK["mfma_tflops"][w.dtype],
                 "unit": "TFLOP/s", "frac": round(ach_tf / PEAK["mfma_tflops"][w.dtype], 4), "traffic": traffic,
                 "kernel": kernel_name, "launch_ms": round(launch_ms, 4),
                 "algorithmic_flops_per_launch": flops_per_launch}
    binding_is_hbm = hbm_time >= mfma_time
    roofline = roof_hbm if binding_is_hbm else roof_mfma
    other = roof_mfma if binding_is_hbm else roof_hbm

    # achieved HBM rate of the bandwidth-bound stages: algorithmic bytes / stage time
    C = b.C
    stage_bytes = {
        "gate": T * H * el + H * E * el + T * E * 4 + T * k * 8,
        # the staged dispatch call packs xe as well (moe_forward gathers inside the first GEMM instead)
        "dispatch": T * k * 4 + (T * k + 2 * E * C + E) * 4 + T * H * el + R * H * el,
        "combine": R * H * el + T * k * 12 + T * H * el,
    }
    stage_gbs = {n: round(v / (stage_ms[n] * 1e-3) / 1e9, 1) for n, v in stage_bytes.items()}

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
        "stage_ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "stage_hbm_gbs": stage_gbs,
        "ffn_tflops": round(4.0 * R * H * I / (ffn_ms * 1e-3) / 1e12, 1),
        "ffn_mfma_frac": round(4.0 * R * H * I / (ffn_ms * 1e-3) / 1e12 / PEAK["mfma_tflops"][w.dtype], 4),
        "roofline": roofline,
        "roofline_other": other,
        "cpu_baseline": cpu_baseline,
        "input_gen_s": round(gen_s, 1),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
