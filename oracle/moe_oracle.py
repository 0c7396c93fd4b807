"""ctypes front end of the C++ CPU oracle (``moe_oracle.cpp``).

Test infrastructure only.  Inputs are host arrays: numpy arrays, or CPU torch
tensors (needed for bf16, which numpy cannot hold).  Outputs are numpy arrays.
The steps O1..O7 and the readings of the paper are stated in ``moe_oracle.h``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

DTYPE = {"f32": 0, "bf16": 1, "f16": 2}
ACT = {"relu": 0, "gelu_tanh": 1, "gelu_erf": 2, "identity": 3}


def oracle_lib_path():
    return os.path.join(_HERE, "libmoe_oracle.so")


def build_oracle(force=True):
    """Compile the oracle with the host compiler (no HIP involved)."""
    out = oracle_lib_path()
    src = os.path.join(_HERE, "moe_oracle.cpp")
    if not force and os.path.exists(out) and os.path.getmtime(out) >= max(
            os.path.getmtime(src), os.path.getmtime(os.path.join(_HERE, "moe_oracle.h"))):
        return out
    cmd = ["g++", "-std=c++17", "-O3", "-march=native", "-ffp-contract=off", "-fopenmp",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", out, src]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return out


def _ptr(a):
    if a is None:
        return None
    if hasattr(a, "data_ptr"):  # CPU torch tensor
        assert a.device.type == "cpu" and a.is_contiguous()
        return ctypes.c_void_p(a.data_ptr())
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


class Oracle:
    def __init__(self, path=None):
        self.lib = ctypes.CDLL(path or oracle_lib_path())
        L = self.lib
        vp, i32, f32, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_double
        i64 = ctypes.c_int64
        L.oracle_set_threads.restype = ctypes.c_int
        L.oracle_set_threads.argtypes = [ctypes.c_int]
        L.oracle_get_threads.restype = ctypes.c_int
        L.oracle_capacity.restype = i32
        L.oracle_capacity.argtypes = [i32, i32, i32, f32, i32]
        L.oracle_capacity_layout.restype = i32
        L.oracle_capacity_layout.argtypes = [i32, i32, f32]
        L.oracle_align_up.restype = i32
        L.oracle_align_up.argtypes = [i32, i32]
        L.oracle_symmetric_layout_bytes.restype = f64
        L.oracle_symmetric_layout_bytes.argtypes = [i64] * 5
        L.oracle_activation.restype = f64
        L.oracle_activation.argtypes = [f64, i32]
        L.oracle_load_elem.restype = f64
        L.oracle_load_elem.argtypes = [vp, i64, i32]
        L.oracle_store_elem.restype = None
        L.oracle_store_elem.argtypes = [vp, i64, i32, f64]
        L.oracle_gate_logits.restype = None
        L.oracle_gate_logits.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
        L.oracle_topk.restype = None
        L.oracle_topk.argtypes = [vp, i32, i32, i32, vp, vp]
        L.oracle_slots.restype = None
        L.oracle_slots.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        L.oracle_slots_choice_major.restype = None
        L.oracle_slots_choice_major.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        L.oracle_ffn_rows.restype = None
        L.oracle_ffn_rows.argtypes = [vp] * 7 + [i32] * 5 + [vp]
        L.oracle_ffn_combine.restype = None
        L.oracle_ffn_combine.argtypes = [vp] * 8 + [i32] * 7 + [vp, i32, vp, vp]
        L.oracle_backward.restype = None
        L.oracle_backward.argtypes = [vp] * 10 + [i32] * 7 + [vp] * 7
        L.oracle_activation_grad.restype = f64
        L.oracle_activation_grad.argtypes = [f64, i32]
        L.oracle_forward.restype = i32
        L.oracle_forward.argtypes = [vp] * 7 + [i32] * 5 + [f32, i32, i32, i32] + [vp] * 9

    # -- knobs ---------------------------------------------------------------------
    def set_threads(self, n):
        return self.lib.oracle_set_threads(int(n))

    def get_threads(self):
        return self.lib.oracle_get_threads()

    # -- scalar helpers --------------------------------------------------------------
    def capacity(self, T, E, k, cf, override=0):
        return self.lib.oracle_capacity(T, E, k, cf, override)

    def capacity_layout(self, T, E, cf):
        return self.lib.oracle_capacity_layout(T, E, cf)

    def align_up(self, C, bM):
        return self.lib.oracle_align_up(C, bM)

    def symmetric_layout_bytes(self, S, E, H, bM=128, elem_bytes=4):
        return self.lib.oracle_symmetric_layout_bytes(S, E, H, bM, elem_bytes)

    def activation(self, v, act):
        return self.lib.oracle_activation(float(v), ACT[act])

    def load_elem(self, a, idx, dtype):
        return self.lib.oracle_load_elem(_ptr(a), idx, DTYPE[dtype])

    def round_to_dtype(self, values, dtype):
        """Round float64 values to the storage dtype; returns them widened back to float64."""
        v = np.ascontiguousarray(np.asarray(values, dtype=np.float64)).ravel()
        buf = np.zeros(v.size, dtype=np.float32 if dtype == "f32" else np.uint16)
        for i in range(v.size):
            self.lib.oracle_store_elem(_ptr(buf), i, DTYPE[dtype], float(v[i]))
        out = np.array([self.lib.oracle_load_elem(_ptr(buf), i, DTYPE[dtype]) for i in range(v.size)])
        return out.reshape(np.shape(values)), buf.reshape(np.shape(values))

    # -- stages ---------------------------------------------------------------------
    def gate_logits(self, x, Wg, gate_bias, T, H, E, dtype):
        logits = np.empty((T, E), dtype=np.float32)
        gb = None if gate_bias is None else _f32(gate_bias)
        self.lib.oracle_gate_logits(_ptr(x), _ptr(Wg), _ptr(gb), T, H, E, DTYPE[dtype], _ptr(logits))
        return logits

    def topk(self, logits, k):
        logits = _f32(logits)
        T, E = logits.shape
        te = np.empty((T, k), dtype=np.int32)
        tw = np.empty((T, k), dtype=np.float32)
        self.lib.oracle_topk(_ptr(logits), T, E, k, _ptr(te), _ptr(tw))
        return te, tw

    def slots(self, topk_expert, topk_weight, E, C, choice_major=False):
        te, tw = _i32(topk_expert), _f32(topk_weight)
        T, k = te.shape
        slot = np.empty((T, k), dtype=np.int32)
        demand = np.empty((E,), dtype=np.int32)
        slot_token = np.empty((E, C), dtype=np.int32)
        slot_weight = np.empty((E, C), dtype=np.float32)
        fn = self.lib.oracle_slots_choice_major if choice_major else self.lib.oracle_slots
        fn(_ptr(te), _ptr(tw), T, E, k, C, _ptr(slot), _ptr(demand), _ptr(slot_token), _ptr(slot_weight))
        return slot, demand, slot_token, slot_weight

    def ffn_rows(self, x, W1, b1, W2, b2, pair_token, pair_expert, H, I, act, dtype):
        pt, pe = _i32(pair_token), _i32(pair_expert)
        y = np.empty((pt.size, H), dtype=np.float64)
        self.lib.oracle_ffn_rows(_ptr(x), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(pt), _ptr(pe),
                                 pt.size, H, I, ACT[act], DTYPE[dtype], _ptr(y))
        return y

    def ffn_combine(self, x, W1, b1, W2, b2, topk_expert, topk_weight, slot, T, H, I, E, act,
                    dtype, tokens=None):
        te, tw, sl = _i32(topk_expert), _f32(topk_weight), _i32(slot)
        k = te.shape[1]
        tok = None if tokens is None else _i32(tokens)
        n = T if tok is None else tok.size
        out = np.empty((n, H), dtype=np.float64)
        self.lib.oracle_ffn_combine(_ptr(x), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(te),
                                    _ptr(tw), _ptr(sl), T, H, I, E, k, ACT[act], DTYPE[dtype],
                                    _ptr(tok), n, _ptr(out), None)
        return out

    def activation_grad(self, v, act):
        return self.lib.oracle_activation_grad(float(v), ACT[act])

    def backward(self, x, Wg, gate_bias, W1, b1, W2, b2, topk_expert, slot, dout, T, H, I, E, act, dtype):
        """Gradients under the given routing; dout is [T, H] float64.  Returns a dict of float64 arrays."""
        te, sl = _i32(topk_expert), _i32(slot)
        k = te.shape[1]
        do = np.ascontiguousarray(np.asarray(dout, dtype=np.float64))
        gb = None if gate_bias is None else _f32(gate_bias)
        g = {"dx": np.empty((T, H)), "dWg": np.empty((H, E)), "dgate_bias": np.empty((E,)),
             "dW1": np.empty((E, H, I)), "db1": np.empty((E, I)), "dW2": np.empty((E, I, H)), "db2": np.empty((E, H))}
        self.lib.oracle_backward(_ptr(x), _ptr(Wg), _ptr(gb), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(te), _ptr(sl),
                                 _ptr(do), T, H, I, E, k, ACT[act], DTYPE[dtype], _ptr(g["dx"]), _ptr(g["dWg"]),
                                 _ptr(g["dgate_bias"]), _ptr(g["dW1"]), _ptr(g["db1"]), _ptr(g["dW2"]), _ptr(g["db2"]))
        return g

    def forward(self, x, Wg, gate_bias, W1, b1, W2, b2, T, H, I, E, k, cf, act, dtype,
                capacity_override=0, compute_out=True):
        C = self.capacity(T, E, k, cf, capacity_override)
        assert C > 0
        r = {
            "C": C,
            "gate_logits": np.empty((T, E), dtype=np.float32),
            "topk_expert": np.empty((T, k), dtype=np.int32),
            "topk_weight": np.empty((T, k), dtype=np.float32),
            "slot": np.empty((T, k), dtype=np.int32),
            "expert_demand": np.empty((E,), dtype=np.int32),
            "slot_token": np.empty((E, C), dtype=np.int32),
            "slot_weight": np.empty((E, C), dtype=np.float32),
            "out": np.empty((T, H), dtype=np.float64) if compute_out else None,
        }
        gb = None if gate_bias is None else _f32(gate_bias)
        got = self.lib.oracle_forward(
            _ptr(x), _ptr(Wg), _ptr(gb), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2),
            T, H, I, E, k, cf, capacity_override, ACT[act], DTYPE[dtype],
            _ptr(r["gate_logits"]), _ptr(r["topk_expert"]), _ptr(r["topk_weight"]), _ptr(r["slot"]),
            _ptr(r["expert_demand"]), _ptr(r["slot_token"]), _ptr(r["slot_weight"]),
            _ptr(r["out"]), None)
        assert got == C
        return r


_ORACLE = None


def load_oracle():
    """Load the oracle, compiling it first if no built library is present."""
    global _ORACLE
    if _ORACLE is None:
        if not os.path.exists(oracle_lib_path()):
            build_oracle()
        _ORACLE = Oracle()
    return _ORACLE
