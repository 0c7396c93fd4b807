"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every
symbol the header declares, and its host logic (capacity arithmetic, workspace
sizing, argument validation) agrees with the oracle and the documented error
behaviour.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2506_04667_amd import binding as moe
from paper_2506_04667_amd.build import LIB_PATH, build_hip
from paper_2506_04667_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB_PATH):
        build_hip()
    return moe.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert set(names) == set(moe.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_config_struct_matches_header():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} moe_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|float)\s+(\w+);", body)
    assert [f for _, f in fields] == [f for f, _ in moe.MoeConfig._fields_]
    assert ctypes.sizeof(moe.MoeConfig) == 4 * len(fields)


def test_capacity_matches_oracle_and_alignment(lib, oracle):
    assert moe.moe_row_tile() == 128
    for w in WORKLOADS.values():
        C, C_pad = moe.moe_capacity(moe.config_of(w))
        assert C == oracle.capacity(w.T, w.E, w.k, w.capacity_factor)
        assert C_pad == oracle.align_up(C, moe.moe_row_tile())
    for (T, E, k, cf, ov) in [(10, 3, 1, 1.0, 0), (1, 64, 1, 0.5, 0), (16384, 128, 2, 1.0, 128), (1000, 7, 3, 1.37, 0)]:
        C, C_pad = moe.moe_capacity(moe.make_config(T, 64, 64, E, k, cf, "relu", "f32", ov))
        assert C == oracle.capacity(T, E, k, cf, ov) and C_pad % 128 == 0 and 0 <= C_pad - C < 128
        # the layout reading drops the factor k; an override wins over either mode
        C, C_pad = moe.moe_capacity(moe.make_config(T, 64, 64, E, k, cf, "relu", "f32", ov, capacity_mode="layout"))
        assert C == (ov if ov else oracle.capacity_layout(T, E, cf)) and C_pad == oracle.align_up(C, 128)


def test_workspace_covers_the_per_expert_buffers(lib):
    for w in WORKLOADS.values():
        cfg = moe.config_of(w)
        C, C_pad = moe.moe_capacity(cfg)
        el = 4 if w.dtype == "f32" else 2
        need = w.E * C_pad * (w.H + w.I) * el + w.T * w.E * 4   # h and y per expert, logits
        got = moe.moe_workspace_bytes(cfg)
        assert need <= got <= need * 1.05 + (1 << 22)


@pytest.mark.parametrize("kw,code", [
    (dict(T=0), -1), (dict(E=0), -1), (dict(k=0), -1), (dict(k=5, E=4), -1), (dict(H=-8), -1),
    (dict(capacity_factor=0.0), -1), (dict(capacity_factor=float("nan")), -1), (dict(capacity_override=-1), -1),
    (dict(H=60), -2), (dict(I=100), -2), (dict(E=9000, k=1), -2), (dict(dtype=3), -2), (dict(act=9), -2),
    (dict(drop_policy=2), -2), (dict(drop_policy=-1), -2), (dict(capacity_mode=2), -2), (dict(capacity_mode=-1), -2),
])
def test_invalid_configs_are_rejected(lib, kw, code):
    base = dict(T=128, H=64, I=128, E=4, k=1, capacity_factor=2.0, capacity_override=0, dtype=0, act=0)
    base.update(kw)
    cfg = moe.MoeConfig(**base)
    n = ctypes.c_size_t()
    assert lib.moe_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)) == code
    assert lib.moe_capacity(ctypes.byref(cfg), None, None) == code
    # the compute entry points validate before they touch the device
    assert lib.moe_forward(ctypes.byref(cfg), None, 0, *([None] * 14)) == code
    assert isinstance(moe.moe_status_string(code), str) and moe.moe_status_string(code) != "ok"


def test_null_and_misaligned_pointers_are_rejected(lib):
    cfg = moe.make_config(128, 64, 128, 4, 1, 2.0, "relu", "f32")
    assert lib.moe_forward(ctypes.byref(cfg), None, 0, *([None] * 14)) == -1
    assert lib.moe_workspace_bytes(ctypes.byref(cfg), None) == -1
    assert lib.moe_workspace_bytes(None, None) == -1
    ok = ctypes.c_void_p(4096)
    bad = ctypes.c_void_p(4100)                                   # not 16-byte aligned
    args = [ok] * 14
    args[0] = bad
    assert lib.moe_forward(ctypes.byref(cfg), ok, 1 << 40, *args) == -1
    assert lib.moe_route(ctypes.byref(cfg), bad, ok, ok, None) == -1
    assert lib.moe_combine(ctypes.byref(cfg), ok, ok, ok, None, ok, None) == -1
    # workspace too small is reported before anything is enqueued
    args = [ok] * 14
    assert lib.moe_forward(ctypes.byref(cfg), ok, 16, *args) == -3


def test_status_strings(lib):
    assert moe.moe_status_string(0) == "ok"
    assert len({moe.moe_status_string(c) for c in (0, -1, -2, -3, -4)}) == 5


def test_binding_fails_loudly_without_the_library(tmp_path):
    with pytest.raises(RuntimeError, match="missing"):
        moe.load(str(tmp_path / "libmoe_hip.so"))
