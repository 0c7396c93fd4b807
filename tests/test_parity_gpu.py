"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs (protocol in tests/parity.py)."""
import numpy as np
import pytest
import torch

from paper_2506_04667_amd import binding as moe
from paper_2506_04667_amd.inputs import WORKLOADS, make_inputs, scaled

import parity

pytestmark = pytest.mark.gpu


def _run(oracle, w, staged=False, tokens=None, gate_bias=None):
    print("case", w, "staged", staged, flush=True)
    cpu = make_inputs(w)
    if gate_bias is not None:
        cpu["gate_bias"] = gate_bias
    dev = parity.to_device(cpu)
    b, host = parity.gpu_forward(w, dev, staged=staged)
    rep = parity.check_layer(oracle, w, cpu, b, host, tokens=tokens)
    print("  ", rep, flush=True)
    return cpu, dev, b, host, rep


# ------------------------------------------------------------ the benchmark's small configurations

def test_tiny_f32_full(oracle):
    cpu, dev, b, host, rep = _run(oracle, WORKLOADS["tiny_f32"])
    assert rep["dropped"] == 0


def test_tiny_f32_staged_matches_fused_call(oracle):
    w = WORKLOADS["tiny_f32"]
    cpu = make_inputs(w)
    dev = parity.to_device(cpu)
    b1, h1 = parity.gpu_forward(w, dev, staged=False)
    b2, h2 = parity.gpu_forward(w, dev, staged=True)
    for n in h1:
        np.testing.assert_array_equal(h1[n], h2[n], err_msg=n)
    assert torch.equal(b1.out, b2.out)


def test_small_f32_full(oracle):
    # capacity 320 is four standard deviations above the mean demand of 256: nothing is dropped here
    _run(oracle, WORKLOADS["small_f32"])


# ------------------------------------------------------------ reduced 16-bit cases: several tiles, ragged tails

@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_reduced_ragged_with_biases(oracle, dtype):
    # rows per expert ~ 190 +- (two row tiles, ragged); I = 840 and H = 328 leave ragged column and k tiles
    w = scaled(WORKLOADS["paper_bf16_e128"], name="reduced", T=757, H=328, I=840, E=8, k=2, capacity_factor=1.0,
               dtype=dtype, seed=11, with_bias=True, act="gelu_tanh")
    cpu, dev, b, host, rep = _run(oracle, w, staged=True)
    assert rep["dropped"] > 0
    # staged intermediates: routing tables and the packed buffer are bit-exact
    slot, demand = parity.check_routing(oracle, w, host, b.C, b.slot_token.cpu().numpy(), b.slot_weight.cpu().numpy())
    st = b.slot_token.cpu().numpy()
    xe = b.xe.cpu()
    x = cpu["x"]
    for e in range(w.E):
        n_e = min(int(demand[e]), b.C)
        assert torch.equal(xe[e, :n_e], x[torch.from_numpy(st[e, :n_e]).long()])
    # expert outputs row by row against the oracle's FFN
    pt = [int(st[e, s]) for e in range(w.E) for s in range(min(int(demand[e]), b.C))][::37]
    pe = [e for e in range(w.E) for s in range(min(int(demand[e]), b.C))][::37]
    ps = [s for e in range(w.E) for s in range(min(int(demand[e]), b.C))][::37]
    y_ref = oracle.ffn_rows(cpu["x"], cpu["W1"], cpu["b1"], cpu["W2"], cpu["b2"], pt, pe, w.H, w.I, w.act, w.dtype)
    y_gpu = parity.to_np64(b.y)[pe, ps]
    parity.assert_close(y_gpu, y_ref, parity.TOL[dtype], "y rows")


@pytest.mark.parametrize("act", ["relu", "gelu_erf", "identity"])
def test_activations_bf16(oracle, act):
    w = scaled(WORKLOADS["paper_bf16_e128"], name="acts", T=300, H=128, I=256, E=4, k=2, capacity_factor=2.0,
               seed=12, act=act)
    _run(oracle, w)


# ------------------------------------------------------------ shapes that take the weight-streaming FFN kernel

@pytest.mark.parametrize("case", [
    # several ragged row tiles per expert, fewer experts than XCDs, shortest K the kernel takes, ragged last column tile
    dict(T=900, H=192, I=448, E=3, k=2, capacity_factor=1.0, dtype="bf16", with_bias=True, act="gelu_erf"),
    # experts nobody picks between live ones; second column tile only 8 wide (I = 264); second GEMM on the generic kernel
    dict(T=2000, H=320, I=264, E=11, k=2, capacity_factor=1.25, dtype="f16", with_bias=True, act="relu", empty=(0, 4, 5, 10)),
    # more experts than XCDs, three row tiles each, both GEMMs streaming
    dict(T=3000, H=256, I=256, E=16, k=2, capacity_factor=1.5, dtype="f16", with_bias=False, act="gelu_tanh"),
    # one live expert out of nine: a single unit feeds one XCD only
    dict(T=300, H=256, I=512, E=9, k=1, capacity_factor=9.0, dtype="bf16", with_bias=True, act="identity",
         empty=(0, 1, 2, 3, 4, 5, 7, 8)),
    # capacities of at most 128 rows take the 128-row tile: ragged rows (C = 108), ragged last column tile
    dict(T=700, H=256, I=320, E=13, k=2, capacity_factor=1.0, dtype="bf16", with_bias=True, act="gelu_erf"),
    # ... with drops (C = 47), more units than XCDs, experts nobody picks
    dict(T=520, H=192, I=256, E=20, k=3, capacity_factor=0.6, dtype="f16", with_bias=False, act="relu", empty=(3, 19)),
    # ... exactly one full 128-row tile per expert
    dict(T=1024, H=512, I=512, E=16, k=2, capacity_factor=1.0, dtype="f16", with_bias=True, act="gelu_tanh"),
    # a handful of rows per expert (decode-like): C = 4 with drops; C = 2 with five tokens
    dict(T=64, H=256, I=512, E=16, k=2, capacity_factor=0.5, dtype="bf16", with_bias=True, act="gelu_erf"),
    dict(T=5, H=192, I=256, E=8, k=2, capacity_factor=1.0, dtype="f16", with_bias=False, act="relu"),
])
def test_streaming_ffn_shapes(oracle, case):
    case = dict(case)
    empty = case.pop("empty", ())
    w = scaled(WORKLOADS["paper_bf16_e128"], name="stream", seed=21, **case)
    gb = None
    if empty:
        gb = torch.zeros(w.E)
        gb[list(empty)] = -1.0e4
    cpu, dev, b, host, rep = _run(oracle, w, gate_bias=gb)
    for e in empty:
        assert host["expert_demand"][e] == 0
    # the staged path (packed rows) and the fused call (rows gathered through the routing table) agree bit for bit
    dev2 = dict(dev)
    b2, host2 = parity.gpu_forward(w, dev2, staged=True)
    assert torch.equal(b.out, b2.out)


# ------------------------------------------------------------ fp32 storage: the equal-span FFN kernel and its fix-up pass

# (the kernel takes a GEMM with fewer than 4 x 256 tiles of 256 x 256 at full capacity and at least 8 x 256 K-tiles of 32)
@pytest.mark.parametrize("case", [
    # one live expert of nine, long K: one or two live tiles for all the workgroups, so every tile is cut into many pieces
    dict(T=150, H=4096, I=512, E=9, k=1, capacity_factor=9.0, with_bias=True, act="gelu_erf", empty=(0, 1, 2, 3, 4, 5, 7, 8)),
    # short K (four K-tiles per tile): ranges of whole tiles with few cuts; 128 units
    dict(T=6000, H=128, I=1024, E=64, k=2, capacity_factor=1.5, with_bias=True, act="relu"),
    # two units per expert, the second one light; experts nobody picks; K not a multiple of the K-tile, ragged last column tile
    dict(T=2000, H=1000, I=776, E=11, k=2, capacity_factor=1.25, with_bias=True, act="gelu_tanh", empty=(0, 4, 5, 10)),
    # drops (C = 47: every unit has two live MFMA row tiles), more experts than XCDs, no bias
    dict(T=520, H=2048, I=512, E=20, k=3, capacity_factor=0.6, with_bias=False, act="identity", empty=(3, 19)),
    # a few rows per expert, very long K
    dict(T=5, H=8192, I=256, E=8, k=2, capacity_factor=1.0, with_bias=False, act="relu"),
    # skewed routing: units of every weight
    dict(T=4096, H=256, I=1024, E=32, k=2, capacity_factor=2.0, with_bias=True, act="gelu_erf", zipf_s=1.2),
])
def test_f32_equal_span_ffn_shapes(oracle, case):
    case = dict(case)
    empty = case.pop("empty", ())
    w = scaled(WORKLOADS["small_f32"], name="f32_span", seed=71, dtype="f32", **case)
    gb = None
    if empty:
        gb = torch.zeros(w.E)
        gb[list(empty)] = -1.0e4
    cpu, dev, b, host, rep = _run(oracle, w, gate_bias=gb)
    for e in empty:
        assert host["expert_demand"][e] == 0
    # the staged path (its own launch for the unit list, packed rows) and the fused call agree bit for bit, and so
    # does a second run: the pieces of a shared tile are added in a fixed order
    b2, host2 = parity.gpu_forward(w, dict(dev), staged=True)
    assert torch.equal(b.out, b2.out)
    b3, host3 = parity.gpu_forward(w, dict(dev))
    assert torch.equal(b.out, b3.out)


def test_many_experts_few_rows_each(oracle):
    # 2048 experts of at most 40 rows: the unit lists are built in several passes of the builder's workgroup, every
    # live unit is a 128-row tile, most experts get a handful of rows and some none; gate on the unfused path (E > 256)
    w = scaled(WORKLOADS["paper_bf16_e128"], name="many_experts", seed=29, T=5000, H=192, I=256, E=2048, k=2,
               capacity_factor=8.0, dtype="bf16", act="gelu_erf")
    cpu, dev, b, host, rep = _run(oracle, w)
    assert b.C == 40 and (host["expert_demand"] == 0).any() and rep["dropped"] == 0
    b2, host2 = parity.gpu_forward(w, dev, staged=True)
    assert torch.equal(b.out, b2.out)


def test_maximum_expert_count(oracle):
    # E = 8192, the largest count the configuration check admits: most experts get no token at all
    w = scaled(WORKLOADS["tiny_f32"], name="max_experts", seed=31, T=300, H=64, I=64, E=8192, k=3, capacity_factor=30.0,
               dtype="f32", act="gelu_tanh")
    cpu, dev, b, host, rep = _run(oracle, w)
    assert b.C == 4 and (host["expert_demand"] == 0).sum() > 7000
    # half as many experts on the weight-streaming FFN kernel (its weights are 400 M elements to draw)
    w16 = scaled(w, name="many_experts_bf16", dtype="bf16", E=4096, H=192, I=256, T=200, seed=32)
    _run(oracle, w16)


def test_single_launch_ffn_opt_in(oracle):
    # both FFN GEMMs in one persistent launch with tile-level dependencies (MOE_FLAG_FFN_SINGLE_LAUNCH): same
    # arithmetic in the same order as the two-launch path, so the outputs must agree bit for bit, and with the
    # oracle within the bar on every row
    cases = [scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn", seed=23, T=3000, H=256, I=256, E=16, k=2,
                    capacity_factor=1.5, dtype="f16", with_bias=True, act="gelu_erf"),
             scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn_few_units", seed=24, T=700, H=512, I=256, E=3, k=1,
                    capacity_factor=1.2, dtype="bf16", act="relu"),
             scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn_small_tile", seed=25, T=1200, H=256, I=512, E=24, k=2,
                    capacity_factor=1.0, dtype="bf16", with_bias=True, act="gelu_tanh"),       # C = 100: 128-row tiles
             # every workgroup's second task is a second-GEMM tile of the unit its own first task feeds (32 live
             # one-tile experts, 8 + 8 column tiles, 32 workgroups per XCD)
             scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn_one_round", seed=26, T=4096, E=32),
             # fewer first-GEMM than second-GEMM column tiles (1 against 8), and the reverse
             scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn_narrow_I", seed=27, T=4096, E=32, I=256, dtype="f16"),
             scaled(WORKLOADS["paper_bf16_e128"], name="fused_ffn_narrow_H", seed=28, T=2048, E=16, H=256, I=1024),
             WORKLOADS["paper_bf16_e128"]]
    for w in cases:
        print("case", w, flush=True)
        cpu = make_inputs(w)
        dev = parity.to_device(cpu)
        b0, host0 = parity.gpu_forward(w, dev)
        w1 = scaled(w, flags=moe.FLAG_FFN_SINGLE_LAUNCH)
        b1, host1 = parity.gpu_forward(w1, dev)
        assert moe.moe_ffn_status(moe.config_of(w1), b1.workspace) == 0
        b2, host2 = parity.gpu_forward(w1, dev)               # again: the completion counters are cleared per call
        assert moe.moe_ffn_status(moe.config_of(w1), b2.workspace) == 0
        assert torch.equal(b0.out, b1.out) and torch.equal(b0.out, b2.out)
        print("  ", parity.check_layer(oracle, w, cpu, b1, host1), flush=True)
        # the staged call takes the flag too (packed rows instead of gathered ones)
        b3, host3 = parity.gpu_forward(w1, dev, staged=True)
        assert moe.moe_ffn_status(moe.config_of(w1), b3.workspace) == 0
        assert torch.equal(b0.out, b3.out)


@pytest.mark.parametrize("case", [
    dict(T=1500, H=256, I=512, E=16, k=2, capacity_factor=1.0, dtype="bf16", with_bias=True, act="gelu_erf"),
    dict(T=700, H=256, I=256, E=8, k=1, capacity_factor=0.7, dtype="f16", with_bias=False, act="relu"),
    dict(T=323, H=256, I=320, E=24, k=3, capacity_factor=1.0, dtype="bf16", with_bias=True, act="gelu_tanh"),   # ragged last tile, C = 41
    dict(T=40000, H=256, I=256, E=64, k=2, capacity_factor=1.25, dtype="f16", with_bias=False, act="identity"),  # more gate tiles than workgroups
    "paper_bf16_e128", "skew_f16_e128",
])
def test_single_launch_layer_opt_in(oracle, case):
    # MOE_FLAG_LAYER_SINGLE_LAUNCH: the whole layer from one persistent kernel with device-wide barriers between
    # its stages.  The stages are the default path's device functions, so every output must equal the default
    # path's bit for bit; one case is also checked against the oracle on every row.
    w = WORKLOADS[case] if isinstance(case, str) else scaled(WORKLOADS["paper_bf16_e128"], name="one_launch", seed=61, **case)
    print("case", w, flush=True)
    cpu = make_inputs(w)
    dev = parity.to_device(cpu)
    b0, host0 = parity.gpu_forward(w, dev)
    w1 = scaled(w, flags=moe.FLAG_LAYER_SINGLE_LAUNCH)
    for rep in range(2):                                      # twice: the barrier words and counters start clean each time
        b1, host1 = parity.gpu_forward(w1, dev)
        assert moe.moe_ffn_status(moe.config_of(w1), b1.workspace) == 0
        for n in host0:
            np.testing.assert_array_equal(host0[n], host1[n], err_msg=n)
        assert torch.equal(b0.out, b1.out)
    stages = moe.moe_layer_stage_ms()                          # workgroup 0's clocks of the launch just checked
    assert all(0.0 <= v < 1e3 for v in stages.values()) and sum(stages.values()) > 0.0, stages
    if not isinstance(case, str) and w.T < 2000:
        print("  ", parity.check_layer(oracle, w, cpu, b1, host1), flush=True)


def test_single_launch_layer_rejects_what_it_cannot_run():
    for kw in (dict(dtype="f32"), dict(E=136), dict(I=200), dict(drop_policy="choice_major")):
        base = dict(T=512, H=256, I=256, E=8, k=2, capacity_factor=1.0, dtype="bf16", act="relu")
        base.update(kw)
        w = scaled(WORKLOADS["paper_bf16_e128"], name="reject", seed=62, flags=moe.FLAG_LAYER_SINGLE_LAUNCH, **base)
        cfg = moe.config_of(w)
        b = moe.Buffers(cfg)
        t = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
        with pytest.raises(moe.MoeError) as e:
            moe.moe_forward(cfg, b.workspace, t, t, None, t, None, t, None, b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot,
                            b.expert_demand)
        assert e.value.code == -2, kw


def test_single_launch_ffn_give_up_is_reported():
    # driven from the host: a completion target no counter reaches and 16 polls per wait, so every second-GEMM
    # task gives up at once; every kernel still exits normally, the call returns ok (it does not synchronise) and
    # the status query names the fault.  The next ordinary call on the same workspace is clean again.
    w = scaled(WORKLOADS["paper_bf16_e128"], name="give_up", seed=35, T=2000, H=256, I=512, E=16, k=2, capacity_factor=1.0)
    cpu = make_inputs(w)
    dev = parity.to_device(cpu)
    b_ref, _ = parity.gpu_forward(w, dev)
    cfg_bad = moe.config_of(scaled(w, flags=moe.FLAG_FFN_SINGLE_LAUNCH | moe.FLAG_DEBUG_DEPENDENCY_NEVER_MET))
    cfg_one = moe.config_of(scaled(w, flags=moe.FLAG_FFN_SINGLE_LAUNCH))
    cfg_two = moe.config_of(w)
    b = moe.Buffers(cfg_two)

    def run(cfg):
        moe.moe_forward(cfg, b.workspace, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["b1"], dev["W2"],
                        dev["b2"], b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot, b.expert_demand)

    run(cfg_bad)
    assert moe.moe_ffn_status(cfg_bad, b.workspace) == -5
    assert "gave up" in moe.moe_status_string(-5)
    run(cfg_one)
    assert moe.moe_ffn_status(cfg_one, b.workspace) == 0
    assert torch.equal(b.out, b_ref.out)
    run(cfg_two)
    assert moe.moe_ffn_status(cfg_two, b.workspace) == 0
    assert torch.equal(b.out, b_ref.out)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("act", ["relu", "gelu_tanh", "gelu_erf", "identity"])
def test_activation_over_its_whole_range(oracle, dtype, act):
    # phi_1 of the first FFN task (Eq. ffn) on a grid of pre-activations over [-10, 10], through the streaming
    # kernel's epilogue: row r of expert e is the unit vector of h = r, so x W1 reproduces row r of W1 exactly (one
    # non-zero product per sum); W2 is the identity, so y = phi(W1) rounded to storage.  The 16-bit erf-GELU is a
    # clamped polynomial: the grid covers the clamp at +-3 sqrt 2 and the tail below -5 that Gaussian
    # pre-activations never reach.
    E, H = 2, 256
    td = parity_dtype = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    n = E * H * H
    grid = torch.linspace(-10.0, 10.0, n, dtype=torch.float64)
    special = torch.tensor([4.2426406871, -4.2426406871, 4.25, -4.25, 4.2, -4.2, 0.0, -0.0, 1e-3, -1e-3, -5.0, -5.5, -6.0,
                            -7.0, -8.0, -9.0, -10.0, 10.0, 3.0, -3.0], dtype=torch.float64)
    grid[:special.numel()] = special
    W1 = grid.to(td).reshape(E, H, H).contiguous()
    v = W1.double().numpy()                                   # the pre-activations, exactly
    W2 = torch.eye(H, dtype=td).repeat(E, 1, 1).contiguous()
    xe = torch.eye(H, dtype=td).repeat(E, 1, 1).contiguous()  # [E, C_pad = 256, H]
    cfg = moe.make_config(H, H, H, E, 2, 1.0, act, dtype)     # C = k T / E = 256 rows per expert
    b = moe.Buffers(cfg).alloc_staged()
    assert b.C == H and b.C_pad == H
    demand = torch.full((E,), H, dtype=torch.int32, device="cuda")
    moe.moe_expert_ffn(cfg, b.workspace, xe.cuda(), demand, W1.cuda(), None, W2.cuda(), None, b.y)
    torch.cuda.synchronize()
    got = b.y.double().cpu().numpy()
    ref = np.vectorize(lambda t: oracle.activation(t, act))(v)
    # the layer's bar on the tensor as a whole ...
    parity.assert_close(got, ref, parity.TOL[dtype], "phi(v) over [-10, 10]")
    # ... and per element: two roundings to storage (h, then y) plus the documented bound of the polynomial,
    # 1.2e-5 |v|; this is what catches a wrong branch in the tails, where the tensor-wide bar is loose
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
    bound = 2.0 * ulp * np.abs(ref) + 1.3e-5 * np.abs(v) + 1e-7
    err = np.abs(got - ref)
    i = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), (act, dtype, v[i], got[i], ref[i])
    # the subnormal range of fp16 and the flush of tiny values must not produce anything but small numbers
    assert np.abs(got[v < -6.0]).max() <= 1.3e-4 if act != "identity" and act != "relu" else True


# ------------------------------------------------------------ shapes that take the fused gate kernel

@pytest.mark.parametrize("T,H,E,k,dtype,bias", [
    (1000, 192, 24, 3, "bf16", True),                         # ragged last token tile, E far below the tile width
    (64, 64, 256, 5, "f16", False),                           # one K-tile, widest expert tile
    (777, 128, 136, 4, "bf16", True),                         # wide tile with a ragged expert tail
    (130, 256, 8, 8, "f16", True),                            # k = E
    (4096, 1024, 128, 2, "bf16", False),                      # full-width tile, deep K
    (1000, 96, 12, 3, "f32", True),                           # fp32: narrowest tile (E <= 64), ragged everything
    (2048, 1024, 16, 2, "f32", False),                        # fp32, the small benchmark configuration's gate
    (500, 128, 64, 2, "f32", True),                           # fp32, E = 64 exactly
    (300, 64, 200, 5, "f32", False),                          # fp32, widest tile with a ragged expert tail
    (700, 2048, 128, 4, "f32", True),                         # fp32, deep K
])
def test_fused_gate_shapes(oracle, T, H, E, k, dtype, bias):
    w = scaled(WORKLOADS["paper_bf16_e128"], name="gate", T=T, H=H, I=8, E=E, k=k, dtype=dtype, seed=31)
    print("case", w, flush=True)
    cpu = make_inputs(w)
    gb = None
    if bias:
        gb = torch.from_numpy(np.random.default_rng(5).standard_normal(E).astype(np.float32))
    cfg = moe.config_of(w)
    b = moe.Buffers(cfg)
    moe.moe_gate(cfg, b.workspace, cpu["x"].cuda(), cpu["Wg"].cuda(), None if gb is None else gb.cuda(),
                 b.gate_logits, b.topk_expert, b.topk_weight)
    torch.cuda.synchronize()
    got = b.gate_logits.cpu().numpy()
    ref = oracle.gate_logits(cpu["x"], cpu["Wg"], None if gb is None else gb.numpy(), T, H, E, dtype)
    parity.assert_close(got, ref, parity.TOL[dtype], "gate_logits")
    te, tw = oracle.topk(got, k)
    np.testing.assert_array_equal(b.topk_expert.cpu().numpy(), te)
    np.testing.assert_allclose(b.topk_weight.cpu().numpy(), tw, rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("case", [
    dict(T=1000, H=256, I=256, E=24, k=3, capacity_factor=1.0, dtype="bf16", act="relu"),       # ragged last chunk of 64 tokens
    dict(T=700, H=128, I=264, E=136, k=4, capacity_factor=0.5, dtype="f16", act="gelu_tanh"),   # wide expert tile, many drops
    dict(T=63, H=64, I=64, E=8, k=8, capacity_factor=1.0, dtype="bf16", act="identity"),        # a single partial chunk, k = E
    dict(T=5000, H=256, I=512, E=256, k=2, capacity_factor=1.5, dtype="bf16", act="gelu_erf",
         with_bias=True),                                                                         # 256 experts, ~40 rows each: streaming FFN with one sparse row tile per expert
    dict(T=2500, H=192, I=256, E=40, k=1, capacity_factor=1.0, dtype="f16", act="relu"),        # top-1, C = 63
])
def test_fused_gate_feeds_the_routing_scan(oracle, case):
    # moe_forward: the fused gate kernel writes the per-chunk expert counts that the slot assignment starts from;
    # the staged calls count with the stand-alone kernel instead.  Both must give the oracle's routing.
    w = scaled(WORKLOADS["paper_bf16_e128"], name="gate_counts", seed=33, **case)
    cpu, dev, b, host, rep = _run(oracle, w)
    b2, host2 = parity.gpu_forward(w, dev, staged=True)
    for n in host:
        np.testing.assert_array_equal(host[n], host2[n], err_msg=n)
    assert torch.equal(b.out, b2.out)


@pytest.mark.parametrize("E,k,dtype", [(16, 4, "bf16"), (128, 2, "bf16"), (200, 7, "bf16"), (40, 3, "f32"), (256, 6, "f32")])
def test_fused_gate_exact_ties(oracle, E, k, dtype):
    # small-integer operands: every logit is an exact small integer, so whole groups of experts tie and the
    # logits themselves must match the oracle bit for bit
    rng = np.random.default_rng(E)
    T, H = 300, 128
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.from_numpy(rng.integers(0, 2, size=(T, H)).astype(np.float32)).to(td)
    Wg = torch.from_numpy(rng.integers(-1, 2, size=(H, E)).astype(np.float32)).to(td)
    Wg[:, 1] = Wg[:, 0]                                       # two experts tie on every token
    cfg = moe.make_config(T, H, 8, E, k, 1.0, "relu", dtype)
    b = moe.Buffers(cfg)
    moe.moe_gate(cfg, b.workspace, x.cuda(), Wg.cuda(), None, b.gate_logits, b.topk_expert, b.topk_weight)
    torch.cuda.synchronize()
    got = b.gate_logits.cpu().numpy()
    ref = oracle.gate_logits(x, Wg, None, T, H, E, dtype)
    np.testing.assert_array_equal(got, ref.astype(np.float32))
    te, tw = oracle.topk(got, k)
    np.testing.assert_array_equal(b.topk_expert.cpu().numpy(), te)
    np.testing.assert_allclose(b.topk_weight.cpu().numpy(), tw, rtol=1e-5, atol=1e-7)


# ------------------------------------------------------------ paper-scale configurations, every output row

@pytest.mark.parametrize("name", ["paper_bf16_e128", "skew_f16_e128", "paper_f32_e64", "paper_bf16_e128/layout"])
def test_paper_scale_every_row(oracle, name):
    # the full-size configurations in the launch configuration the benchmark times: logits, routing and all
    # T x H outputs against the oracle (its FFN + combine under the GPU's routing takes seconds on the host cores)
    w = WORKLOADS[name.split("/")[0]]
    if name.endswith("/layout"):                       # the layout reading of the capacity: C = 128, half the pairs dropped
        w = scaled(w, capacity_mode="layout")
    print("case", w, flush=True)
    cpu = make_inputs(w)
    dev = parity.to_device(cpu)
    b, host = parity.gpu_forward(w, dev)
    rep = parity.check_layer(oracle, w, cpu, b, host, tokens=None)
    print("  ", rep, flush=True)
    demand = host["expert_demand"]
    assert demand.sum() == w.T * w.k
    if name == "skew_f16_e128":
        assert (demand > b.C).any() and (demand < 8).any()
    else:
        assert rep["dropped"] > 0
    # properties that hold at any size: every kept pair's packed row is the token's row
    assert (host["slot"] < b.C).all()
    out = parity.to_np64(b.out)
    all_dropped = (host["slot"] < 0).all(axis=1)
    assert (out[all_dropped] == 0).all()
    # determinism: a second run is bit-identical
    b2, host2 = parity.gpu_forward(w, dev)
    assert torch.equal(b.out, b2.out)
    for n in host:
        np.testing.assert_array_equal(host[n], host2[n], err_msg=n)


# ------------------------------------------------------------ selection and slotting edge cases

def test_route_tie_heavy_logits(oracle):
    rng = np.random.default_rng(3)
    for T, E, k in [(257, 4, 1), (64, 7, 7), (1000, 130, 5), (33, 1, 1), (500, 64, 64), (129, 300, 3), (50, 600, 4)]:
        logits = rng.integers(-2, 3, size=(T, E)).astype(np.float32)
        logits[logits == 0] *= rng.choice([1.0, -1.0], size=int((logits == 0).sum())).astype(np.float32)
        cfg = moe.make_config(T, 8, 8, E, k, 1.0, "relu", "f32")
        gl = torch.from_numpy(logits).cuda()
        te = torch.empty((T, k), dtype=torch.int32, device="cuda")
        tw = torch.empty((T, k), dtype=torch.float32, device="cuda")
        moe.moe_route(cfg, gl, te, tw)
        torch.cuda.synchronize()
        te_ref, tw_ref = oracle.topk(logits, k)
        np.testing.assert_array_equal(te.cpu().numpy(), te_ref)
        np.testing.assert_allclose(tw.cpu().numpy(), tw_ref, rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("policy", ["token_major", "choice_major"])
@pytest.mark.parametrize("T,E,k,C", [(1, 1, 1, 0), (5, 3, 3, 2), (1000, 6, 2, 1), (4099, 37, 3, 0), (777, 128, 2, 7),
                                     (3000, 2, 2, 1000), (70000, 16, 4, 0)])
def test_dispatch_slots_bit_exact(oracle, T, E, k, C, policy):
    rng = np.random.default_rng(T + E)
    # skewed choices: some experts overflow, some stay empty
    logits = (rng.standard_normal((T, E)) + np.linspace(0, 4, E)).astype(np.float32)
    if E > 4:
        logits[:, 1] = -50.0                                  # an expert nobody picks (k < E)
    te, tw = oracle.topk(logits, k)
    cfg = moe.make_config(T, 8, 8, E, k, 1.0, "relu", "f32", capacity_override=C, drop_policy=policy)
    b = moe.Buffers(cfg).alloc_staged()
    te_d, tw_d = torch.from_numpy(te).cuda(), torch.from_numpy(tw).cuda()
    moe.moe_dispatch(cfg, b.workspace, None, te_d, tw_d, b.slot, b.expert_demand, b.slot_token, b.slot_weight, None)
    torch.cuda.synchronize()
    slot, demand, st, sw = oracle.slots(te, tw, E, b.C, choice_major=(policy == "choice_major"))
    np.testing.assert_array_equal(b.slot.cpu().numpy(), slot)
    np.testing.assert_array_equal(b.expert_demand.cpu().numpy(), demand)
    np.testing.assert_array_equal(b.slot_token.cpu().numpy(), st)
    np.testing.assert_array_equal(b.slot_weight.cpu().numpy(), sw)


def test_all_tokens_to_one_expert_and_empty_experts(oracle):
    w = scaled(WORKLOADS["paper_bf16_e128"], name="one_expert", T=400, H=64, I=64, E=8, k=1, capacity_factor=1.0,
               seed=13, dtype="f32", act="relu")
    gb = torch.zeros(8)
    gb[5] = 1000.0                                            # every token picks expert 5; C = 50 -> 350 drops
    cpu, dev, b, host, rep = _run(oracle, w, gate_bias=gb)
    assert rep["kept"] == 50 and rep["dropped"] == 350
    assert list(host["expert_demand"]) == [0, 0, 0, 0, 0, 400, 0, 0]


def test_k_equals_E_and_single_token(oracle):
    w = scaled(WORKLOADS["tiny_f32"], name="kE", T=65, H=64, I=72, E=5, k=5, capacity_factor=1.0, seed=14)
    _run(oracle, w)
    w = scaled(WORKLOADS["tiny_f32"], name="one_token", T=1, H=8, I=8, E=3, k=2, capacity_factor=1.0, seed=15)
    _run(oracle, w)
    w = scaled(WORKLOADS["tiny_f32"], name="E1", T=130, H=72, I=136, E=1, k=1, capacity_factor=0.5, seed=16, dtype="bf16")
    cpu, dev, b, host, rep = _run(oracle, w)
    assert rep["kept"] == 65


def test_capacity_override_paper_layout_reading(oracle):
    # the layout section's capacity reading (no factor k): C = ceil(T / E)
    w = scaled(WORKLOADS["tiny_f32"], name="override", T=512, H=64, I=128, E=8, k=2, capacity_factor=1.0, seed=17,
               capacity_override=64)
    cpu, dev, b, host, rep = _run(oracle, w)
    assert b.C == 64 and rep["dropped"] >= 512


@pytest.mark.parametrize("dtype,cf", [("bf16", 1.0), ("f32", 1.25)])
def test_layout_capacity_mode_end_to_end(oracle, dtype, cf):
    # the layout section's reading as a mode of the configuration: half the slots of the default at k = 2
    base = scaled(WORKLOADS["paper_bf16_e128"], name="layout_capacity", seed=47, T=3000, H=256, I=512, E=24, k=2,
                  capacity_factor=cf, dtype=dtype, act="gelu_erf")
    w = scaled(base, capacity_mode="layout")
    cpu = make_inputs(base)
    dev = parity.to_device(cpu)
    b, host = parity.gpu_forward(w, dev)
    assert b.C == oracle.capacity_layout(3000, 24, cf) == (125 if cf == 1.0 else 157)
    rep = parity.check_layer(oracle, w, cpu, b, host)
    print("  ", rep, flush=True)
    assert rep["dropped"] >= 6000 - 24 * b.C
    # the same layer through capacity_override gives the same bits
    ov = scaled(base, name="layout_capacity_override", capacity_override=b.C)
    b_ov, host_ov = parity.gpu_forward(ov, dev)
    assert np.array_equal(host_ov["slot"], host["slot"]) and torch.equal(b_ov.out, b.out)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_choice_major_drop_priority_end_to_end(oracle, dtype):
    # half the capacity the demand needs: many second choices lose their slots to later tokens' first choices
    base = scaled(WORKLOADS["paper_bf16_e128"], name="choice_major", seed=43, T=2100, H=256, I=256, E=16, k=2,
                  capacity_factor=0.6, dtype=dtype, act="gelu_tanh")
    w = scaled(base, drop_policy="choice_major")
    cpu = make_inputs(base)
    dev = parity.to_device(cpu)
    b, host = parity.gpu_forward(w, dev)
    rep = parity.check_layer(oracle, w, cpu, b, host)
    print("  ", rep, flush=True)
    assert rep["dropped"] > 0
    b_tok, host_tok = parity.gpu_forward(base, dev)            # the default priority keeps a different set
    assert (host_tok["slot"] != host["slot"]).any()
    dropped_first = (host["slot"][:, 0] < 0).sum(), (host_tok["slot"][:, 0] < 0).sum()
    assert dropped_first[0] <= dropped_first[1]                # first choices fare no worse when they go first
    b2, host2 = parity.gpu_forward(w, dev, staged=True)
    assert torch.equal(b.out, b2.out)


@pytest.mark.parametrize("dtype,flags,H", [("bf16", 0, 256), ("bf16", moe.FLAG_LAYER_SINGLE_LAUNCH, 256), ("f32", 0, 2048)])
def test_forward_replays_from_a_hip_graph(oracle, dtype, flags, H):
    # moe_forward allocates nothing, synchronises nothing and clears its scratch with kernels, so a caller may
    # capture it; every replay (with eager work and synchronisation in between, and new inputs in the same
    # buffers) must reproduce the eager result bit for bit.  Also for the whole layer as one launch (its barrier
    # words start and end every launch at zero) and for the fp32 FFN kernel with its second pass (H = 2048 makes
    # both GEMMs large enough for it).
    w = scaled(WORKLOADS["paper_bf16_e128"], name="graph", seed=41, T=1500, H=H, I=512, E=16, k=2,
               capacity_factor=1.0, with_bias=True, dtype=dtype, flags=flags)
    cpu = make_inputs(w)
    dev = parity.to_device(cpu)
    cfg = moe.config_of(w)
    b = moe.Buffers(cfg)

    def run():
        moe.moe_forward(cfg, b.workspace, dev["x"], dev["Wg"], dev["gate_bias"], dev["W1"], dev["b1"], dev["W2"],
                        dev["b2"], b.out, b.gate_logits, b.topk_expert, b.topk_weight, b.slot, b.expert_demand)

    run()                                                     # first call outside capture: kernel attributes get set
    torch.cuda.synchronize()
    eager = b.out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.current_stream().wait_stream(side)
    x0 = dev["x"].clone()
    for rep in range(4):
        if rep == 2:                                          # other inputs in the same buffer, then back
            dev["x"].copy_(x0.flip(0))
            run()
            torch.cuda.synchronize()
            eager_flipped = b.out.clone()
        b.out.zero_()
        b.workspace.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(b.out, eager_flipped if rep >= 2 else eager), rep
        _ = (dev["W1"][0, :8, :8].float() @ dev["W1"][0, :8, :8].float().t()).sum().item()   # unrelated eager work
    dev["x"].copy_(x0)
    host = {"gate_logits": b.gate_logits.cpu().numpy(), "topk_expert": b.topk_expert.cpu().numpy(),
            "topk_weight": b.topk_weight.cpu().numpy(), "slot": b.slot.cpu().numpy(),
            "expert_demand": b.expert_demand.cpu().numpy()}
    cpu_flipped = dict(cpu)
    cpu_flipped["x"] = cpu["x"].flip(0).contiguous()
    print("  ", parity.check_layer(oracle, w, cpu_flipped, b, host), flush=True)


def test_error_codes_on_device_calls():
    cfg = moe.make_config(128, 64, 128, 4, 1, 2.0, "relu", "f32")
    b = moe.Buffers(cfg)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    x = torch.zeros((128, 64), device="cuda")
    with pytest.raises(moe.MoeError) as e:
        moe.moe_gate(cfg, small, x, x, None, b.gate_logits, b.topk_expert, b.topk_weight)
    assert e.value.code == -3
    with pytest.raises(moe.MoeError) as e:
        moe.moe_gate(cfg, b.workspace, None, x, None, b.gate_logits, b.topk_expert, b.topk_weight)
    assert e.value.code == -1
