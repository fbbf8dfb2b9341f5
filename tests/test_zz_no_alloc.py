"""moe_route_static (the entry point that allocates nothing: its scratch is a file-scope device
array) against moe_route, through the C ABI, bit for bit, on two calls in a row, the second with
a smaller input.  Collected last so that a failure here cannot hide another test."""
import ctypes

import numpy as np
import pytest
import torch

import moe_synth
import paper_2604_19241_amd as moe

KEYS = ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm")


def _same(a, b, what):
    for key in KEYS:
        x, y = getattr(a, key).cpu().numpy(), getattr(b, key).cpu().numpy()
        assert np.array_equal(x.view(np.int32), y.view(np.int32)), (what, key)


@pytest.mark.gpu
def test_route_static_matches_route_on_two_calls_in_a_row():
    torch.cuda.set_device(0)
    big = moe_synth.small_config(T=4096, d=256, E=128, k=8, I=64, name="static-big")
    small = moe_synth.small_config(T=777, d=256, E=64, k=6, I=64, e_start=16, e_count=32, name="static-small")
    calls = []
    for cfg in (big, small):
        shape = moe.make_shape(**cfg.shape_dict())
        assert moe.moe_workspace_bytes(shape)["route"] <= moe.ROUTE_STATIC_SCRATCH_BYTES
        logits = moe_synth.make_inputs(cfg, seed=5, with_dy=False, with_weights=False)["logits"].cuda()
        calls.append((shape, logits, moe.alloc_routing(shape, "cuda")))
    # the two calls back to back on one stream, nothing in between: the second, smaller problem
    # finds the first one's histogram in the scratch array
    for shape, logits, out in calls:
        moe.moe_route_static(shape, logits, out)
    torch.cuda.synchronize()
    for shape, logits, out in calls:
        want = moe.moe_route(shape, logits)
        torch.cuda.synchronize()
        _same(out, want, (shape.T, shape.E))
        assert int(want.offsets[-1]) > 0


@pytest.mark.gpu
def test_route_static_empty_input():
    torch.cuda.set_device(0)
    shape = moe.make_shape(T=0, d=64, E=8, k=2, I=64)
    out = moe.alloc_routing(shape, "cuda")
    moe.moe_route_static(shape, torch.empty((0, 8), dtype=torch.float32, device="cuda"), out)
    torch.cuda.synchronize()
    assert out.counts.cpu().tolist() == [0] * 8 and out.offsets.cpu().tolist() == [0] * 9


def test_route_static_rejects_problems_beyond_its_scratch():
    """Host-side check: no device is touched before the size test."""
    lib = moe.load_library()
    shape = moe.make_shape(T=16384, d=64, E=1024, k=16, I=64)   # 1024 chunks x 1024 experts x 4 B = 4 MiB + 256
    assert moe.moe_workspace_bytes(shape)["route"] > moe.ROUTE_STATIC_SCRATCH_BYTES
    r = moe.binding.MoERoutingC(*([8] * 6))   # non-null, aligned dummies: never dereferenced
    rc = lib.moe_route_static(ctypes.byref(shape), ctypes.c_void_p(8), ctypes.byref(r), None)
    assert rc == moe.binding.MOE_ERR_WORKSPACE
