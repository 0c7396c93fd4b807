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
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


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
        if w.dtype == "f32":                                    # two partial 256 x 256 tiles per workgroup of the equal-share FFN kernel
            units = w.E * -(-C // 256)
            wgs = max(units * -(-w.I // 256) * -(-w.H // 32), units * -(-w.H // 256) * -(-w.I // 32))
            need += min(256, wgs) * 2 * 256 * 256 * 4
        got = moe.moe_workspace_bytes(cfg)
        assert need <= got <= need * 1.05 + (1 << 22)


@pytest.mark.parametrize("kw,code", [
    (dict(T=0), -1), (dict(E=0), -1), (dict(k=0), -1), (dict(k=5, E=4), -1), (dict(H=-8), -1),
    (dict(capacity_factor=0.0), -1), (dict(capacity_factor=float("nan")), -1), (dict(capacity_override=-1), -1),
    (dict(H=60), -2), (dict(I=100), -2), (dict(E=9000, k=1), -2), (dict(dtype=3), -2), (dict(act=9), -2),
    (dict(drop_policy=2), -2), (dict(drop_policy=-1), -2), (dict(capacity_mode=2), -2), (dict(capacity_mode=-1), -2),
    (dict(flags=8), -1), (dict(flags=2), -1), (dict(flags=5), -1),   # unknown bit; the test aid without the single launch; the layer flag with another
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


def test_backward_entry_points_validate_on_the_host(lib):
    ok = ctypes.c_void_p(4096)
    cfg = moe.make_config(128, 64, 128, 4, 1, 2.0, "relu", "f32")
    n = ctypes.c_size_t()
    assert lib.moe_backward_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)) == 0 and n.value > 0
    assert lib.moe_backward_workspace_bytes(ctypes.byref(cfg), None) == -1
    assert lib.moe_backward(ctypes.byref(cfg), ok, 16, *([ok] * 17)) == -3          # workspace too small
    args = [ok] * 17
    args[9] = None                                                                 # dx missing
    assert lib.moe_backward(ctypes.byref(cfg), ok, 1 << 40, *args) == -1
    many = moe.make_config(128, 64, 128, 128, 65, 2.0, "relu", "f32")               # k > 64
    assert lib.moe_backward_workspace_bytes(ctypes.byref(many), ctypes.byref(n)) == -2
    flagged = moe.make_config(512, 256, 256, 4, 2, 1.0, "relu", "bf16", flags=1)
    assert lib.moe_backward_workspace_bytes(ctypes.byref(flagged), ctypes.byref(n)) == -2


def test_layer_stage_clock_arguments_are_checked_on_the_host(lib):
    ms = (ctypes.c_double * 10)()
    assert lib.moe_layer_stage_ms(None, 10, None) == -1
    assert lib.moe_layer_stage_ms(ms, 11, None) == -1
    assert lib.moe_layer_stage_ms(ms, -1, None) == -1
    assert len(moe.LAYER_STAGES) == 10


def test_yardstick_arguments_are_checked_on_the_host(lib):
    ok = ctypes.c_void_p(4096)
    moved = ctypes.c_double()
    assert lib.moe_probe_lds_fill(3, ok, 1 << 21, 8, ok, ctypes.byref(moved), None) == -1     # unknown mode
    assert lib.moe_probe_lds_fill(0, ok, 1 << 21, 7, ok, ctypes.byref(moved), None) == -1     # odd step count
    assert lib.moe_probe_lds_fill(0, ok, 1000, 8, ok, ctypes.byref(moved), None) == -1        # region not a multiple of 64 KiB
    assert lib.moe_probe_lds_fill(0, None, 1 << 21, 8, ok, ctypes.byref(moved), None) == -1
    assert lib.moe_probe_stream(ok, None, 8, ok, None) == -1                                   # fewer than 16 bytes
    assert lib.moe_probe_mfma(7, 10, ok, None, None) == -1                                     # unknown dtype


def test_status_strings(lib):
    assert moe.moe_status_string(0) == "ok"
    assert len({moe.moe_status_string(c) for c in (0, -1, -2, -3, -4, -5, -6, -7)}) == 8


def test_single_launch_flag_needs_a_shape_the_streaming_kernel_takes(lib):
    ok = ctypes.c_void_p(4096)
    for kw, code in [(dict(dtype=0), -2),                          # fp32 storage
                     (dict(I=200), -2), (dict(H=128), -2),         # I not a multiple of 64; H below 256
                     (dict(), -3)]:                                # eligible: the next check (workspace size) is reached
        base = dict(T=512, H=256, I=256, E=4, k=2, capacity_factor=1.0, capacity_override=0, dtype=1, act=2, flags=1)
        base.update(kw)
        cfg = moe.MoeConfig(**base)
        assert lib.moe_forward(ctypes.byref(cfg), ok, 1 << 40 if code != -3 else 16, *([ok] * 14)) == code, kw


# ---- dealing of the FFN tasks and the single-launch dependency protocol, replayed on the host -------------

def _programs(n_l, n_s, nrow_l, ncol0, ncol1, wgs, t2_first=False):
    """Per workgroup (xcd, wg): the operations of the single-launch FFN kernel in program order.
    ("store", phase, list, index, column tile) | ("wait", list, index)."""
    progs = {}
    for xcd in range(8):
        for wg in range(wgs):
            ops = []
            bodies = [(ph, large) for ph in ((1, 0) if t2_first else (0, 1)) for large in (1, 0)]
            for ph, large in bodies:
                ncol = ncol1 if ph else ncol0
                tasks = moe.moe_ffn_schedule(large, n_l, n_s, nrow_l, ncol, xcd, wg, wgs)
                if not tasks:
                    continue
                if ph == 0:                                         # first-GEMM tasks never wait
                    ops += [("store", 0, large, li, ct) for li, ct in tasks]
                else:                                               # waits run two tasks ahead of the stores
                    ops += [("wait", large, li) for li, _ in tasks[:2]]
                    for j, (li, ct) in enumerate(tasks):
                        if j + 2 < len(tasks):
                            ops.append(("wait", large, tasks[j + 2][0]))
                        ops.append(("store", 1, large, li, ct))
            progs[(xcd, wg)] = ops
    return progs


def _replay(progs, ncol0, order_seed):
    """Run the programs under an arbitrary interleaving; returns (stalled, stores in order)."""
    import random
    rng = random.Random(order_seed)
    pc = {w: 0 for w in progs}
    done = {}
    log = []
    live = [w for w in progs if progs[w]]
    while live:
        rng.shuffle(live)
        progress = False
        for w in list(live):
            steps = rng.randint(1, 4)
            while steps and pc[w] < len(progs[w]):
                op = progs[w][pc[w]]
                if op[0] == "wait" and done.get((op[1], op[2]), 0) < ncol0:
                    break
                if op[0] == "store":
                    log.append(op[1:])
                    if op[1] == 0:
                        done[(op[2], op[3])] = done.get((op[2], op[3]), 0) + 1
                pc[w] += 1
                steps -= 1
                progress = True
            if pc[w] == len(progs[w]):
                live.remove(w)
        if not progress:
            return True, log
    return False, log


@pytest.mark.parametrize("wgs", [1, 2, 5, 32])
def test_ffn_tasks_are_dealt_exactly_once_and_single_launch_waits_end(lib, wgs):
    # the shapes a reviewer's replay of the earlier schedule stalled on are among these: 4 one-tile units per
    # XCD with 8 + 8 column tiles and 32 workgroups; fewer first-GEMM than second-GEMM column tiles
    cases = [(0, 32, 0, 8, 8), (16, 0, 1, 8, 8), (128, 0, 1, 8, 8), (0, 32, 0, 1, 8), (0, 32, 0, 2, 8), (0, 32, 0, 16, 8),
             (40, 7, 3, 3, 5), (1, 1, 2, 1, 1), (5, 33, 1, 8, 2), (0, 0, 0, 4, 4), (14, 53, 2, 8, 8), (9, 3, 4, 2, 16)]
    for n_l, n_s, nrow_l, ncol0, ncol1 in cases:
        progs = _programs(n_l, n_s, nrow_l, ncol0, ncol1, wgs)
        for seed in (0, 1):
            stalled, log = _replay(progs, ncol0, seed)
            assert not stalled, (n_l, n_s, nrow_l, ncol0, ncol1, wgs)
            want = sorted([(ph, large, li, ct) for ph, ncol in ((0, ncol0), (1, ncol1))
                           for large, n in ((1, n_l), (0, n_s)) for li in range(n) for ct in range(ncol)])
            assert sorted(log) == want                              # every (phase, unit, column tile) exactly once
            first_t2 = {}
            last_t1 = {}
            for pos, (ph, large, li, ct) in enumerate(log):
                if ph == 0:
                    last_t1[(large, li)] = pos
                else:
                    first_t2.setdefault((large, li), pos)
            assert all(first_t2[u] > last_t1[u] for u in first_t2)  # no second-GEMM tile before its unit's first-GEMM tiles
    # the replay does notice a protocol that cannot make progress: second-GEMM tasks walked first
    stalled, _ = _replay(_programs(0, 32, 0, 8, 8, wgs, t2_first=True), 8, 0)
    assert stalled


def test_ffn_schedule_balances_the_xcds(lib):
    # every XCD gets the same number of units to within one, whatever the counts
    for n_l, n_s, nrow_l in [(14, 53, 2), (128, 0, 1), (3, 5, 7), (0, 1, 0)]:
        per_xcd = []
        for xcd in range(8):
            per_xcd.append(sum(len(moe.moe_ffn_schedule(large, n_l, n_s, nrow_l, 1, xcd, wg, 4)) for large in (1, 0) for wg in range(4)))
        assert sum(per_xcd) == n_l + n_s and max(per_xcd) - min(per_xcd) <= 2
    assert lib.moe_ffn_schedule(1, 4, 4, 1, 0, 0, 0, 1, None, None, 0) == -1


@pytest.mark.parametrize("case", [
    dict(rows=[257, 254, 265, 257, 247, 261, 275, 270, 245, 237, 246, 256, 221, 252, 237, 245], cap=320, N=4096, K=1024),   # config 2's shape
    dict(rows=[257, 254, 265, 257, 247, 261, 275, 270, 245, 237, 246, 256, 221, 252, 237, 245], cap=320, N=1024, K=4096),
    dict(rows=[0, 0, 0, 0, 0, 0, 150, 0, 0], cap=150, N=512, K=4096),                  # one live expert cut into many pieces
    dict(rows=[5, 0, 700, 1, 33, 64, 65, 999, 256, 512], cap=600, N=264, K=40),        # every weight; values above the capacity
    dict(rows=[0] * 7, cap=64, N=256, K=32),                                           # nothing live
    dict(rows=[3], cap=3, N=8, K=8),                                                   # a single iteration
])
@pytest.mark.parametrize("wgs", [1, 3, 8, 128, 256])
def test_f32_ffn_work_is_dealt_exactly_once_and_every_cut_tile_has_one_owner(lib, case, wgs):
    rows, cap, N, K = case["rows"], case["cap"], case["N"], case["K"]
    ids, cum, first, fix = moe.moe_f32_ffn_schedule(rows, cap, N, K, wgs)
    ncol, nk, nrow = -(-N // 256), -(-K // 32), -(-cap // 256)
    # the list: every live 256-row tile once, in order of expert, with the documented weights
    live = [min(r, cap) for r in rows]
    want = [g * nrow + rt for g, r in enumerate(live) for rt in range(-(-r // 256))]
    assert ids == want
    weight = []
    for r in live:
        for rt in range(-(-r // 256)):
            b = min(8, -(-r // 32) - 8 * rt)                  # live 32-row MFMA tiles of the unit
            weight.append(min(12, 3 * -(-b // 2)))
    assert [cum[u + 1] - cum[u] for u in range(len(ids))] == weight and cum[0] == 0
    # the ranges: consecutive, covering every iteration once
    total = len(ids) * ncol * nk
    assert first[0] == 0 and first[-1] == total and all(a <= b for a, b in zip(first, first[1:]))
    # ... and of about equal cost: a range's cost differs from the equal share by less than two iterations of the heaviest unit
    cost_of = lambda L: cum[L // (ncol * nk)] * ncol * nk + (L % (ncol * nk)) * weight[L // (ncol * nk)] if L < total else cum[-1] * ncol * nk
    if total:
        share = cum[-1] * ncol * nk / wgs
        for w in range(wgs):
            assert abs(cost_of(first[w + 1]) - cost_of(first[w]) - share) < 2 * 12 + 1
    # the second pass: a tile is cut if a range boundary falls strictly inside it; each cut tile is fixed by exactly one
    # workgroup, the one whose range holds the tile's first K-tile; whole tiles by nobody
    cut = {}
    for w in range(wgs):
        a, b = first[w], first[w + 1]
        L = a
        while L < b:
            t = L // nk
            end = min(b, (t + 1) * nk)
            if not (L == t * nk and end == (t + 1) * nk):
                cut.setdefault(t, []).append((w, L, end))
            L = end
    owners = {}
    for w, t in enumerate(fix):
        if t >= 0:
            assert t not in owners
            owners[t] = w
    assert set(owners) == set(cut)
    for t, pieces in cut.items():
        assert pieces[0][0] == owners[t] and pieces[0][1] == t * nk and pieces[-1][2] == (t + 1) * nk
        assert all(p[2] == q[1] for p, q in zip(pieces, pieces[1:]))       # the pieces tile the K range, in workgroup order
        assert [p[0] for p in pieces] == sorted(p[0] for p in pieces)


def test_binding_fails_loudly_without_the_library(tmp_path):
    with pytest.raises(RuntimeError, match="missing"):
        moe.load(str(tmp_path / "libmoe_hip.so"))
