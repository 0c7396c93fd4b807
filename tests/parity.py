"""Parity protocol shared by the GPU tests: HIP path (through the C ABI) vs the CPU oracle.

Three separate checks, because near-tied top-k choices may legitimately differ
when the logits differ in their last bits:
  (i)   GPU gate logits vs oracle gate logits, within the floating-point bar;
  (ii)  oracle routing *fed the GPU's logits* vs GPU routing: expert ids, slots,
        demand bit-exact; combine weights within 1e-5;
  (iii) GPU `out` vs oracle FFN + combine run under that routing, within the bar.
The floating-point bar: |gpu - ref| <= tol * |ref| + tol * rms(ref), tol = 1e-5 for
fp32 storage and 2e-2 for bf16/fp16 storage with fp32 accumulation.
"""
import numpy as np
import torch

from paper_2506_04667_amd import binding as moe

TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}


def to_np64(t):
    return t.detach().to("cpu").double().numpy()


def rms(a):
    return float(np.sqrt(np.mean(np.square(a, dtype=np.float64)))) if a.size else 0.0


def assert_close(got, ref, tol, what):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), what + ": non-finite values"
    bound = tol * np.abs(ref) + tol * rms(ref)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d elements outside tol %.1e; worst at %s: got %r ref %r (rms %.3e, max err/rms %.3e)"
                             % (what, bad.sum(), bad.size, tol, i, got[i], ref[i], rms(ref), err.max() / max(rms(ref), 1e-300)))
    return float(err.max() / max(rms(ref), 1e-300))


def to_device(inputs):
    return {n: (None if v is None else v.to("cuda")) for n, v in inputs.items()}


def gpu_forward(w, dev_inputs, staged=False):
    """Run the layer through the C ABI.  Returns (buffers, dict of host copies)."""
    cfg = moe.config_of(w)
    b = moe.Buffers(cfg)
    d = dev_inputs
    if not staged:
        moe.moe_forward(cfg, b.workspace, d["x"], d["Wg"], d["gate_bias"], d["W1"], d["b1"], d["W2"], d["b2"],
                        b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot, b.expert_demand)
    else:
        b.alloc_staged()
        moe.moe_gate(cfg, b.workspace, d["x"], d["Wg"], d["gate_bias"], b.gate_logits, b.topk_expert, b.topk_weight)
        moe.moe_dispatch(cfg, b.workspace, d["x"], b.topk_expert, b.topk_weight, b.slot, b.expert_demand,
                         b.slot_token, b.slot_weight, b.xe)
        moe.moe_expert_ffn(cfg, b.workspace, b.xe, b.expert_demand, d["W1"], d["b1"], d["W2"], d["b2"], b.y)
        moe.moe_combine(cfg, b.y, b.topk_expert, b.topk_weight, b.slot, b.out)
    torch.cuda.synchronize()
    host = {
        "gate_logits": b.gate_logits.cpu().numpy(),
        "topk_expert": b.topk_expert.cpu().numpy(),
        "topk_weight": b.topk_weight.cpu().numpy(),
        "slot": b.slot.cpu().numpy(),
        "expert_demand": b.expert_demand.cpu().numpy(),
    }
    return b, host


def check_routing(oracle, w, host, C, slot_token=None, slot_weight=None):
    """(ii): the oracle's routing of the GPU's logits must equal the GPU's routing."""
    choice_major = getattr(w, "drop_policy", "token_major") == "choice_major"
    te, tw = oracle.topk(host["gate_logits"], w.k)
    np.testing.assert_array_equal(host["topk_expert"], te, err_msg="topk_expert")
    np.testing.assert_allclose(host["topk_weight"], tw, rtol=1e-5, atol=1e-7, err_msg="topk_weight")
    # slots from the GPU's own (expert, weight) tables: bit-exact integer work
    slot, demand, st, sw = oracle.slots(host["topk_expert"], host["topk_weight"], w.E, C, choice_major=choice_major)
    np.testing.assert_array_equal(host["slot"], slot, err_msg="slot")
    np.testing.assert_array_equal(host["expert_demand"], demand, err_msg="expert_demand")
    if slot_token is not None:
        np.testing.assert_array_equal(slot_token, st, err_msg="slot_token")
        np.testing.assert_array_equal(slot_weight, sw, err_msg="slot_weight")
    return slot, demand


def check_layer(oracle, w, cpu_inputs, buffers, host, tokens=None, check_logits=True):
    """(i) + (ii) + (iii).  `tokens`: sample of token ids for (iii) (None = all)."""
    tol = TOL[w.dtype]
    i = cpu_inputs
    report = {}
    if check_logits:
        ref_logits = oracle.gate_logits(i["x"], i["Wg"], None if i["gate_bias"] is None else i["gate_bias"].numpy(),
                                        w.T, w.H, w.E, w.dtype)
        report["logits_err"] = assert_close(host["gate_logits"], ref_logits, tol, "gate_logits")
    C = buffers.C
    if getattr(w, "capacity_mode", "per_choice") == "layout" and not w.capacity_override:
        assert C == oracle.capacity_layout(w.T, w.E, w.capacity_factor)
    else:
        assert C == oracle.capacity(w.T, w.E, w.k, w.capacity_factor, w.capacity_override)
    check_routing(oracle, w, host, C)
    ref_out = oracle.ffn_combine(i["x"], i["W1"], i["b1"], i["W2"], i["b2"], host["topk_expert"],
                                 host["topk_weight"], host["slot"], w.T, w.H, w.I, w.E, w.act, w.dtype,
                                 tokens=tokens)
    got = to_np64(buffers.out)
    if tokens is not None:
        got = got[np.asarray(tokens)]
    report["out_err"] = assert_close(got, ref_out, tol, "out")
    report["kept"] = int((host["slot"] >= 0).sum())
    report["dropped"] = int((host["slot"] < 0).sum())
    return report
