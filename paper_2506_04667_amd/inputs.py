"""Seeded synthetic inputs for the MoE layer forward.

This module serves both the HIP path's callers and the CPU oracle's callers and
holds none of the method's arithmetic: it only draws tensors.  The shapes are the
paper's evaluation shapes (Sec. 4 set-up: embedding 2048, FFN intermediate 2048,
top-2, capacity factor 1.0, up to 16K tokens and 128 experts) plus two small
cases the oracle finishes in seconds.

Recipe: every tensor is drawn on the host from numpy's Philox generator keyed by
(seed, tensor id), as float32 standard normals, scaled, then rounded (to nearest
even) to the storage dtype.  The same bytes go to the GPU and to the oracle.
Expert weights are drawn one expert at a time so that the paper-scale cases stay
within a few GiB of host memory.
"""
import math
from dataclasses import dataclass, replace

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


@dataclass(frozen=True)
class MoEWorkload:
    name: str
    T: int
    H: int
    I: int
    E: int
    k: int
    capacity_factor: float
    act: str            # "relu" | "gelu_tanh" | "gelu_erf" | "identity"
    dtype: str          # "f32" | "bf16" | "f16"
    seed: int
    x_scale_by_fan_in: bool = False   # tiny case: x ~ N(0,1)/sqrt(H); else x ~ N(0,1)
    zipf_s: float = 0.0               # > 0: gate_bias[e] = -s * ln(rank_e), rank a seeded permutation
    with_bias: bool = False           # draw b1, b2 (all paper configs: False)
    capacity_override: int = 0
    drop_policy: str = "token_major"  # or "choice_major": who keeps a slot on overflow
    capacity_mode: str = "per_choice" # or "layout": capacity factor scales k T / E, or T / E
    flags: int = 0                    # moe_config.flags (launch options of the HIP library; the oracle ignores them)


WORKLOADS = {
    # the five configurations of the benchmark definition, in order
    "tiny_f32": MoEWorkload("tiny_f32", 128, 64, 128, 4, 1, 2.0, "relu", "f32", 0, x_scale_by_fan_in=True),
    "small_f32": MoEWorkload("small_f32", 2048, 1024, 4096, 16, 2, 1.25, "gelu_tanh", "f32", 2),
    "paper_f32_e64": MoEWorkload("paper_f32_e64", 16384, 2048, 2048, 64, 2, 1.0, "gelu_erf", "f32", 3),
    "paper_bf16_e128": MoEWorkload("paper_bf16_e128", 16384, 2048, 2048, 128, 2, 1.0, "gelu_erf", "bf16", 4),
    "skew_f16_e128": MoEWorkload("skew_f16_e128", 16384, 2048, 2048, 128, 2, 1.25, "gelu_erf", "f16", 5, zipf_s=1.2),
}

_TENSOR_ID = {"x": 1, "Wg": 2, "W1": 3, "W2": 4, "b1": 5, "b2": 6, "perm": 7}


def _rng(seed, tensor, sub=0):
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | _TENSOR_ID[tensor], sub]))


def _normal(seed, tensor, shape, scale, dtype, sub=0):
    a = _rng(seed, tensor, sub).standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(scale)
    return torch.from_numpy(a).to(TORCH_DTYPE[dtype])


def scaled(w: MoEWorkload, **kw) -> MoEWorkload:
    """A copy of a workload with some fields replaced (for reduced-size test cases)."""
    return replace(w, **kw)


def make_inputs(w: MoEWorkload, device="cpu"):
    """Draw the layer's inputs.  Returns a dict of tensors in the storage dtype
    (``gate_bias`` in float32, or None; ``b1``/``b2`` None unless ``with_bias``).
    With a non-CPU ``device`` each tensor is moved there as it is drawn."""
    dev = torch.device(device)
    T, H, I, E = w.T, w.H, w.I, w.E
    x_scale = 1.0 / math.sqrt(H) if w.x_scale_by_fan_in else 1.0
    out = {}
    out["x"] = _normal(w.seed, "x", (T, H), x_scale, w.dtype).to(dev)
    out["Wg"] = _normal(w.seed, "Wg", (H, E), 1.0 / math.sqrt(H), w.dtype).to(dev)
    W1 = torch.empty((E, H, I), dtype=TORCH_DTYPE[w.dtype], device=dev)
    W2 = torch.empty((E, I, H), dtype=TORCH_DTYPE[w.dtype], device=dev)
    for e in range(E):
        W1[e].copy_(_normal(w.seed, "W1", (H, I), 1.0 / math.sqrt(H), w.dtype, sub=e))
        W2[e].copy_(_normal(w.seed, "W2", (I, H), 1.0 / math.sqrt(I), w.dtype, sub=e))
    out["W1"], out["W2"] = W1, W2
    if w.with_bias:
        out["b1"] = _normal(w.seed, "b1", (E, I), 0.5, w.dtype).to(dev)
        out["b2"] = _normal(w.seed, "b2", (E, H), 0.5, w.dtype).to(dev)
    else:
        out["b1"] = out["b2"] = None
    if w.zipf_s > 0.0:
        rank = _rng(w.seed, "perm").permutation(E) + 1          # rank_e in 1..E
        gb = (-w.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)
        out["gate_bias"] = torch.from_numpy(gb).to(dev)
    else:
        out["gate_bias"] = None
    return out
