"""The entry point that allocates nothing: moe_layer_forward_noalloc runs the layer in the library's static
device array and must give the bits moe_layer_forward gives with a caller workspace -- on two calls in a row,
the second with a smaller input (the array keeps what the first call left behind)."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def _layer(cfg):
    from paper_2405_18832_amd.device_layer import DeviceLayer
    layer = wl.make_layer(cfg)
    return DeviceLayer(cfg, layer.x, layer.w_gate, layer.b_gate, layer.expert, device="cuda:0")


def test_noalloc_matches_layer_forward(gpu_lib):
    moe = gpu_lib
    big = wl.MoEConfig("noalloc_big", T=96, d_model=256, d_ff=1024, E=16, k=2, dtype="bf16", renormalize=True,
                       seed=51, zipf_s=1.0, gate_std=0.3)
    small = wl.MoEConfig("noalloc_small", T=7, d_model=128, d_ff=256, E=5, k=1, dtype="bf16", renormalize=False,
                         seed=52, gate_std=0.3)
    moe.moe_init()
    assert moe.moe_noalloc_max_workspace() == 16 << 20
    for rep in range(2):                       # big, small, then again: every order of sizes back to back
        for cfg in (big, small):
            say(f"[case] moe_layer_forward_noalloc {cfg.name} (pass {rep})")
            L = _layer(cfg)
            assert moe.moe_workspace_bytes(L.shape) <= moe.moe_noalloc_max_workspace()
            for mask, H in ((None, -1), (None, 2), (torch.tensor([1, 0] * 8, dtype=torch.uint8)[:cfg.E].cuda(), -1)):
                L.out.fill_(float("nan"))
                L.forward(mask=mask, H=H)
                torch.cuda.synchronize()
                want = L.out.clone()
                got = torch.full_like(L.out, float("nan"))
                before = torch.cuda.memory_allocated()
                moe.moe_layer_forward_noalloc(L.shape, L.x, L.w_gate, L.b_gate, L.w1, L.w2, mask, H, got)
                torch.cuda.synchronize()
                assert torch.cuda.memory_allocated() == before
                assert torch.isfinite(got.float()).all()
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (cfg.name, rep, H)
            del L


def test_noalloc_rejects_what_does_not_fit(gpu_lib):
    moe = gpu_lib
    say("[case] moe_layer_forward_noalloc size limit")
    shape = moe.make_shape(T=4096, d_model=1024, d_ff=4096, E=128, k=1, dtype="bf16", renormalize=False)
    assert moe.moe_workspace_bytes(shape) > moe.moe_noalloc_max_workspace()
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(moe.MoEError) as err:
        moe.moe_layer_forward_noalloc(shape, dummy, dummy, None, dummy, dummy, None, -1, dummy)
    assert err.value.status == moe.MOE_ERR_WORKSPACE      # refused before any launch: the dummies are never touched
    torch.cuda.synchronize()
