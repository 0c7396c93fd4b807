"""The entry point that allocates nothing (moe_dispatch_noalloc: the routing scan's scratch is a fixed device
array inside the library) against moe_dispatch with a caller workspace: identical results, bit for bit, on two
calls in a row of which the second is smaller, so that what the first left in the shared array must not matter."""
import gc

import numpy as np
import pytest
import torch

from paper_2506_04667_amd import binding as moe

pytestmark = pytest.mark.gpu


def _dispatch_both(T, H, E, k, C, policy, seed):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((T, E)) + np.linspace(0, 3, E)).astype(np.float32)   # some experts overflow
    order = np.argsort(-logits, axis=1, kind="stable")[:, :k].astype(np.int32)
    weight = rng.random((T, k), dtype=np.float32)
    x = torch.from_numpy(rng.standard_normal((T, H)).astype(np.float32)).to(torch.bfloat16).cuda()
    te, tw = torch.from_numpy(order).cuda(), torch.from_numpy(weight).cuda()
    cfg = moe.make_config(T, H, 64, E, k, 1.0, "relu", "bf16", capacity_override=C, drop_policy=policy)
    ref = moe.Buffers(cfg).alloc_staged()
    got = moe.Buffers(cfg).alloc_staged()
    moe.moe_dispatch(cfg, ref.workspace, x, te, tw, ref.slot, ref.expert_demand, ref.slot_token, ref.slot_weight, ref.xe)
    # no device memory is taken or given back by the call: the driver's free-memory figure does not move
    # (collect garbage of earlier tests first, so that nothing of theirs is freed in between)
    gc.collect()
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    moe.moe_dispatch_noalloc(cfg, x, te, tw, got.slot, got.expert_demand, got.slot_token, got.slot_weight, got.xe)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before
    for name in ("slot", "expert_demand", "slot_token", "slot_weight", "xe"):
        assert torch.equal(getattr(got, name), getattr(ref, name)), name
    return int((got.slot < 0).sum().item()), int(got.expert_demand.sum().item())


def test_noalloc_dispatch_matches_dispatch_on_two_calls_in_a_row():
    moe.moe_init()
    dropped, pairs = _dispatch_both(T=5000, H=128, E=48, k=3, C=200, policy="token_major", seed=1)
    assert pairs == 15000 and dropped > 0
    # a smaller input right after: fewer chunks and fewer experts than the counts the first call left behind
    dropped, pairs = _dispatch_both(T=333, H=64, E=5, k=2, C=90, policy="choice_major", seed=2)
    assert pairs == 666 and dropped > 0
    # and the benchmark's routing shape
    _dispatch_both(T=16384, H=64, E=128, k=2, C=256, policy="token_major", seed=3)


def test_noalloc_dispatch_rejects_what_its_scratch_cannot_hold():
    # ceil(T / 64) * E ints must fit in the fixed array: 1100 chunks x 1024 experts x 4 B > 4 MiB
    cfg = moe.make_config(70400, 64, 64, 1024, 1, 1.0, "relu", "bf16")
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoeError) as e:
        moe.moe_dispatch_noalloc(cfg, None, t, t, t, t, t, t, None)
    assert e.value.code == -7
    assert moe.STATIC_SCRATCH_BYTES == 4 << 20
