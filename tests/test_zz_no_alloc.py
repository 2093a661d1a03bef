"""The entry point that allocates nothing (rf_moe_routing_noalloc) against the entry point it is
a variant of (rf_moe_routing, caller's workspace): same kernels, so every probability and every
index must be identical.  Two calls in a row share the library's scratch array; the second works
on a smaller problem, so whatever the first left behind must not show."""
import sys

import pytest
import torch

from paper_2603_10026_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def rf():
    from paper_2603_10026_amd import binding
    binding.load_library()
    return binding


def _one(rf, seed, S, hd, E, topk):
    print(f"[case] moe_routing_noalloc S={S} hd={hd} E={E} topk={topk}", flush=True)
    sys.stdout.flush()
    x, w = I.moe_routing_inputs_device(seed, S, hd, E, 1.5, "bf16", DEV)
    p_ref, i_ref = rf.rf_moe_routing(x, w, topk)                      # caller's workspace
    prob = torch.full((S, topk), float("nan"), dtype=torch.float32, device=DEV)
    idx = torch.full((S, topk), -1, dtype=torch.int32, device=DEV)
    rf.rf_moe_routing_noalloc(x, w, topk, prob, idx)
    torch.cuda.synchronize()
    assert torch.equal(idx, i_ref)
    assert torch.equal(prob, p_ref)                                   # bit for bit: same arithmetic
    return x, w


def test_noalloc_matches_workspace_entry_point_twice(rf):
    assert rf.moe_routing_workspace_bytes(2048, 4096, 128) <= rf.MOE_ROUTING_NOALLOC_MAX_BYTES
    _one(rf, 31, 2048, 4096, 128, 8)       # the largest table shape: fills the scratch array
    _one(rf, 32, 300, 1024, 64, 4)         # smaller, ragged last row block, fewer slices and experts
    _one(rf, 33, 2048, 8192, 64, 8)


def test_noalloc_refuses_what_does_not_fit(rf):
    S = 1 << 16
    assert rf.moe_routing_workspace_bytes(S, 256, 64) > rf.MOE_ROUTING_NOALLOC_MAX_BYTES
    x = torch.zeros((S, 256), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((256, 64), dtype=torch.bfloat16, device=DEV)
    prob = torch.zeros((S, 4), dtype=torch.float32, device=DEV)
    idx = torch.zeros((S, 4), dtype=torch.int32, device=DEV)
    with pytest.raises(rf.RfError) as e:
        rf.rf_moe_routing_noalloc(x, w, 4, prob, idx)
    assert e.value.code == rf.RF_ERR_WORKSPACE
