"""Thin ctypes binding of the C ABI in ``include/moe.h``.

Argument marshalling only: torch tensors supply device pointers and the current
HIP stream; every step of the layer runs in the library's kernels.  There is no
fallback: if the built library is missing, ``load()`` raises.
"""
import ctypes
import os

import torch

from .build import LIB_PATH

MOE_OK = 0
DTYPE = {"f32": 0, "bf16": 1, "f16": 2}
ACT = {"relu": 0, "gelu_tanh": 1, "gelu_erf": 2, "identity": 3}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}

EXPORTS = ["moe_status_string", "moe_init", "moe_row_tile", "moe_capacity", "moe_workspace_bytes", "moe_forward",
           "moe_gate", "moe_route", "moe_dispatch", "moe_expert_ffn", "moe_combine", "moe_ffn_status", "moe_ffn_schedule",
           "moe_forward_timed", "moe_probe_stream", "moe_probe_mfma", "moe_dispatch_noalloc",
           "moe_backward_workspace_bytes", "moe_backward", "moe_layer_stage_ms", "moe_f32_ffn_schedule", "moe_probe_lds_fill"]
LAYER_STAGES = ("gate", "barrier1", "clear_scan", "barrier2", "scatter_units", "barrier3", "ffn_gemm1", "ffn_gemm2", "barrier4",
                "combine")
STATIC_SCRATCH_BYTES = 4 << 20
FORWARD_EVENTS = 6
FLAG_FFN_SINGLE_LAUNCH = 1
FLAG_DEBUG_DEPENDENCY_NEVER_MET = 2
FLAG_LAYER_SINGLE_LAUNCH = 4


class MoeConfig(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("I", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("capacity_factor", ctypes.c_float),
                ("capacity_override", ctypes.c_int32), ("dtype", ctypes.c_int32), ("act", ctypes.c_int32),
                ("drop_policy", ctypes.c_int32), ("capacity_mode", ctypes.c_int32), ("flags", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("moe: %s (%d)" % (text, code))
        self.code = code


_LIB = None


def load(path=None):
    """Load the built HIP library.  Raises if it has not been built."""
    global _LIB
    if _LIB is not None and path is None:
        return _LIB
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError("HIP library %s is missing: run __graft_entry__.build() (or "
                           "python -m paper_2506_04667_amd.build) first; there is no fallback path" % p)
    lib = ctypes.CDLL(p)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    cfgp = ctypes.POINTER(MoeConfig)
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [ctypes.c_int]
    lib.moe_init.restype = ctypes.c_int
    lib.moe_init.argtypes = []
    lib.moe_ffn_status.restype = ctypes.c_int
    lib.moe_ffn_status.argtypes = [cfgp, vp, ctypes.c_size_t, vp]
    lib.moe_ffn_schedule.restype = ctypes.c_int32
    lib.moe_ffn_schedule.argtypes = [ctypes.c_int32] * 8 + [i32p, i32p, ctypes.c_int32]
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib.moe_f32_ffn_schedule.restype = ctypes.c_int32
    lib.moe_f32_ffn_schedule.argtypes = [i32p] + [ctypes.c_int32] * 5 + [i64p, i64p, i32p, i32p, ctypes.c_int32]
    lib.moe_layer_stage_ms.restype = ctypes.c_int
    lib.moe_layer_stage_ms.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, vp]
    lib.moe_row_tile.restype = ctypes.c_int32
    lib.moe_row_tile.argtypes = []
    lib.moe_capacity.restype = ctypes.c_int
    lib.moe_capacity.argtypes = [cfgp, i32p, i32p]
    lib.moe_workspace_bytes.restype = ctypes.c_int
    lib.moe_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.moe_forward.restype = ctypes.c_int
    lib.moe_forward.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 14
    lib.moe_forward_timed.restype = ctypes.c_int
    lib.moe_forward_timed.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 13 + [ctypes.POINTER(vp), vp]
    lib.moe_probe_lds_fill.restype = ctypes.c_int
    lib.moe_probe_lds_fill.argtypes = [ctypes.c_int32, vp, ctypes.c_size_t, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.moe_probe_stream.restype = ctypes.c_int
    lib.moe_probe_stream.argtypes = [vp, vp, ctypes.c_size_t, vp, vp]
    lib.moe_probe_mfma.restype = ctypes.c_int
    lib.moe_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.moe_gate.restype = ctypes.c_int
    lib.moe_gate.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 7
    lib.moe_route.restype = ctypes.c_int
    lib.moe_route.argtypes = [cfgp] + [vp] * 4
    lib.moe_dispatch.restype = ctypes.c_int
    lib.moe_dispatch.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 9
    lib.moe_dispatch_noalloc.restype = ctypes.c_int
    lib.moe_dispatch_noalloc.argtypes = [cfgp] + [vp] * 9
    lib.moe_backward_workspace_bytes.restype = ctypes.c_int
    lib.moe_backward_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.moe_backward.restype = ctypes.c_int
    lib.moe_backward.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 17
    lib.moe_expert_ffn.restype = ctypes.c_int
    lib.moe_expert_ffn.argtypes = [cfgp, vp, ctypes.c_size_t] + [vp] * 8
    lib.moe_combine.restype = ctypes.c_int
    lib.moe_combine.argtypes = [cfgp] + [vp] * 6
    if path is None:
        _LIB = lib
    return lib


DROP_POLICY = {"token_major": 0, "choice_major": 1}
CAPACITY_MODE = {"per_choice": 0, "layout": 1}


def make_config(T, H, I, E, k, capacity_factor, act, dtype, capacity_override=0, drop_policy="token_major",
                capacity_mode="per_choice", flags=0):
    return MoeConfig(T, H, I, E, k, float(capacity_factor), int(capacity_override), DTYPE[dtype], ACT[act],
                     DROP_POLICY[drop_policy], CAPACITY_MODE[capacity_mode], int(flags))


def config_of(w):
    """moe_config of a workload description (anything with T, H, I, E, k, capacity_factor, act, dtype)."""
    return make_config(w.T, w.H, w.I, w.E, w.k, w.capacity_factor, w.act, w.dtype,
                       getattr(w, "capacity_override", 0), getattr(w, "drop_policy", "token_major"),
                       getattr(w, "capacity_mode", "per_choice"), getattr(w, "flags", 0))


def _p(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    assert t.is_cuda and t.is_contiguous(), "device pointers only: pass contiguous tensors on the GPU"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(code):
    if code != MOE_OK:
        raise MoeError(code, load().moe_status_string(code).decode())


def moe_status_string(code):
    return load().moe_status_string(code).decode()


def moe_init():
    _check(load().moe_init())


def moe_row_tile():
    return load().moe_row_tile()


def moe_ffn_schedule(large_list, n_units_large, n_units_small, nrow_large, ncol, xcd, wg, wgs, max_tasks=4096):
    """(list index, column tile) of each task of one workgroup, in the order it runs them (host arithmetic)."""
    li = (ctypes.c_int32 * max_tasks)()
    ct = (ctypes.c_int32 * max_tasks)()
    n = load().moe_ffn_schedule(int(large_list), n_units_large, n_units_small, nrow_large, ncol, xcd, wg, wgs, li, ct, max_tasks)
    if n < 0 or n > max_tasks:
        raise MoeError(-1, "moe_ffn_schedule: invalid arguments or more than max_tasks tasks")
    return [(li[i], ct[i]) for i in range(n)]


def moe_ffn_status(cfg, workspace, stream=None):
    """Status code of the last single-launch FFN on this workspace (synchronises the stream)."""
    return load().moe_ffn_status(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _stream(stream))


def moe_f32_ffn_schedule(rows, capacity, N, K, workgroups):
    """Host replay of the fp32 equal-share FFN dealing: (unit ids, weight prefix sums, first iteration per workgroup
    [workgroups + 1], tile to fix per workgroup [-1 = none])."""
    groups = len(rows)
    cap = groups * (-(-capacity // 256))
    r = (ctypes.c_int32 * groups)(*[int(v) for v in rows])
    first = (ctypes.c_int64 * (workgroups + 1))()
    fix = (ctypes.c_int64 * workgroups)()
    ids = (ctypes.c_int32 * max(cap, 1))()
    cum = (ctypes.c_int32 * (cap + 1))()
    n = load().moe_f32_ffn_schedule(r, groups, capacity, N, K, workgroups, first, fix, ids, cum, cap)
    if n < 0:
        raise MoeError(-1, "moe_f32_ffn_schedule")
    return list(ids[:n]), list(cum[:n + 1]), list(first), list(fix)


def moe_layer_stage_ms(stream=None):
    """Stage times (ms, by name) of the last single-launch layer, as seen by its workgroup 0 (synchronises the stream)."""
    ms = (ctypes.c_double * len(LAYER_STAGES))()
    _check(load().moe_layer_stage_ms(ms, len(LAYER_STAGES), _stream(stream)))
    return dict(zip(LAYER_STAGES, ms))


def moe_capacity(cfg):
    C, Cp = ctypes.c_int32(), ctypes.c_int32()
    _check(load().moe_capacity(ctypes.byref(cfg), ctypes.byref(C), ctypes.byref(Cp)))
    return C.value, Cp.value


def moe_workspace_bytes(cfg):
    n = ctypes.c_size_t()
    _check(load().moe_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return n.value


def _ws_bytes(ws):
    return ws.numel() * ws.element_size()


def moe_forward(cfg, workspace, x, Wg, gate_bias, W1, b1, W2, b2, out, gate_logits, topk_expert,
                topk_weight, slot, expert_demand, stream=None):
    _check(load().moe_forward(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(x), _p(Wg),
                              _p(gate_bias), _p(W1), _p(b1), _p(W2), _p(b2), _p(out), _p(gate_logits),
                              _p(topk_expert), _p(topk_weight), _p(slot), _p(expert_demand), _stream(stream)))


def event_handles(events):
    """The hipEvent_t handles of torch events (created with enable_timing=True).  torch creates the handle at the
    first record(), so each event is recorded once here."""
    arr = (ctypes.c_void_p * len(events))()
    for i, e in enumerate(events):
        if not e.cuda_event:
            e.record()
        arr[i] = e.cuda_event
    return arr


def moe_forward_timed(cfg, workspace, x, Wg, gate_bias, W1, b1, W2, b2, out, gate_logits, topk_expert,
                      topk_weight, slot, expert_demand, handles, stream=None):
    """moe_forward with the FORWARD_EVENTS events of ``handles`` (from event_handles) recorded at its stage boundaries."""
    _check(load().moe_forward_timed(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(x), _p(Wg),
                                    _p(gate_bias), _p(W1), _p(b1), _p(W2), _p(b2), _p(out), _p(gate_logits),
                                    _p(topk_expert), _p(topk_weight), _p(slot), _p(expert_demand), handles,
                                    _stream(stream)))


def moe_probe_stream(src, dst, sink, stream=None):
    _check(load().moe_probe_stream(_p(src), _p(dst), src.numel() * src.element_size(), _p(sink), _stream(stream)))


def moe_probe_mfma(dtype, iters, sink, stream=None):
    """Launch the MFMA loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double()
    _check(load().moe_probe_mfma(DTYPE[dtype], int(iters), _p(sink), ctypes.byref(flops), _stream(stream)))
    return flops.value


def moe_probe_lds_fill(mode, src, region_bytes, steps, sink, stream=None):
    """Launch the LDS-fill yardstick (mode 0 direct copies, 1 loads + ds_write, 2 loads alone); returns the bytes moved."""
    moved = ctypes.c_double()
    _check(load().moe_probe_lds_fill(int(mode), _p(src), int(region_bytes), int(steps), _p(sink), ctypes.byref(moved), _stream(stream)))
    return moved.value


def moe_gate(cfg, workspace, x, Wg, gate_bias, gate_logits, topk_expert, topk_weight, stream=None):
    _check(load().moe_gate(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(x), _p(Wg),
                           _p(gate_bias), _p(gate_logits), _p(topk_expert), _p(topk_weight), _stream(stream)))


def moe_route(cfg, gate_logits, topk_expert, topk_weight, stream=None):
    _check(load().moe_route(ctypes.byref(cfg), _p(gate_logits), _p(topk_expert), _p(topk_weight), _stream(stream)))


def moe_dispatch(cfg, workspace, x, topk_expert, topk_weight, slot, expert_demand, slot_token, slot_weight,
                 xe, stream=None):
    _check(load().moe_dispatch(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(x), _p(topk_expert),
                               _p(topk_weight), _p(slot), _p(expert_demand), _p(slot_token), _p(slot_weight),
                               _p(xe), _stream(stream)))


def moe_dispatch_noalloc(cfg, x, topk_expert, topk_weight, slot, expert_demand, slot_token, slot_weight, xe, stream=None):
    _check(load().moe_dispatch_noalloc(ctypes.byref(cfg), _p(x), _p(topk_expert), _p(topk_weight), _p(slot),
                                       _p(expert_demand), _p(slot_token), _p(slot_weight), _p(xe), _stream(stream)))


def moe_backward_workspace_bytes(cfg):
    n = ctypes.c_size_t()
    _check(load().moe_backward_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return n.value


def moe_backward(cfg, workspace, x, Wg, W1, b1, W2, b2, topk_expert, topk_weight, dout, dx, dWg, dgate_bias, dW1, db1,
                 dW2, db2, stream=None):
    _check(load().moe_backward(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(x), _p(Wg), _p(W1), _p(b1),
                               _p(W2), _p(b2), _p(topk_expert), _p(topk_weight), _p(dout), _p(dx), _p(dWg),
                               _p(dgate_bias), _p(dW1), _p(db1), _p(dW2), _p(db2), _stream(stream)))


def moe_expert_ffn(cfg, workspace, xe, expert_demand, W1, b1, W2, b2, y, stream=None):
    _check(load().moe_expert_ffn(ctypes.byref(cfg), _p(workspace), _ws_bytes(workspace), _p(xe),
                                 _p(expert_demand), _p(W1), _p(b1), _p(W2), _p(b2), _p(y), _stream(stream)))


def moe_combine(cfg, y, topk_expert, topk_weight, slot, out, stream=None):
    _check(load().moe_combine(ctypes.byref(cfg), _p(y), _p(topk_expert), _p(topk_weight), _p(slot), _p(out),
                              _stream(stream)))


class Buffers:
    """Device buffers for one configuration: outputs of the layer, the staged
    calls' intermediates and the workspace.  Allocation is plumbing, done by torch."""

    def __init__(self, cfg, device="cuda"):
        self.cfg = cfg
        T, H, E, k = cfg.T, cfg.H, cfg.E, cfg.k
        td = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}[cfg.dtype]
        self.C, self.C_pad = moe_capacity(cfg)
        dev = torch.device(device)
        self.workspace = torch.empty(moe_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
        self.out = torch.empty((T, H), dtype=td, device=dev)
        self.gate_logits = torch.empty((T, E), dtype=torch.float32, device=dev)
        self.topk_expert = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.topk_weight = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.slot = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.expert_demand = torch.empty((E,), dtype=torch.int32, device=dev)
        self._td, self._dev = td, dev
        self.slot_token = self.slot_weight = self.xe = self.y = None

    def alloc_staged(self):
        cfg, dev = self.cfg, self._dev
        self.slot_token = torch.empty((cfg.E, self.C), dtype=torch.int32, device=dev)
        self.slot_weight = torch.empty((cfg.E, self.C), dtype=torch.float32, device=dev)
        self.xe = torch.zeros((cfg.E, self.C_pad, cfg.H), dtype=self._td, device=dev)
        self.y = torch.zeros((cfg.E, self.C_pad, cfg.H), dtype=self._td, device=dev)
        return self
