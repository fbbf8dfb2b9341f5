"""GPU parity of moe_route: indices, counts and offsets bit-exact against the
oracle; gates to fp32 rounding."""
import numpy as np
import pytest
import torch

import moe_synth
import oracle
from helpers import gpu_routing_as_np, say

pytestmark = pytest.mark.gpu


def run_route(cfg, logits_np):
    import paper_2604_19241_amd as moe
    shape = moe.make_shape(**cfg.shape_dict())
    r = moe.moe_route(shape, torch.from_numpy(logits_np).cuda())
    torch.cuda.synchronize()
    return gpu_routing_as_np(r)


def check(cfg, logits_np, tag):
    say(f"[route] {tag} {cfg.shape_dict()}")
    want = oracle.route(cfg.shape_dict(), logits_np)
    got = run_route(cfg, logits_np)
    for key in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(got[key], want[key]), (tag, key)
    assert np.allclose(got["topk_w"], want["topk_w"], rtol=2e-6, atol=1e-7), tag
    return got


CASES = [
    dict(T=256, d=64, E=8, k=2, I=64),
    dict(T=1000, d=64, E=128, k=8, I=64),
    dict(T=777, d=64, E=256, k=8, I=64, e_start=32, e_count=32),
    dict(T=333, d=64, E=64, k=6, I=64),
    dict(T=129, d=64, E=512, k=10, I=64),
    dict(T=65, d=64, E=1024, k=16, I=64, e_start=1000, e_count=24),
    dict(T=50, d=64, E=5, k=5, I=64),
    dict(T=1, d=64, E=3, k=1, I=64),
    dict(T=2049, d=64, E=16, k=4, I=64, e_start=3, e_count=9),
]


@pytest.mark.parametrize("kw", CASES)
def test_route_matches_oracle(kw):
    cfg = moe_synth.small_config(**kw)
    rng = np.random.default_rng(kw["T"] + kw["E"])
    logits = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)
    check(cfg, logits, "random")


def test_route_ties_and_skew():
    cfg = moe_synth.small_config(T=600, d=64, E=48, k=4, I=64)
    rng = np.random.default_rng(7)
    logits = rng.integers(0, 3, (cfg.T, cfg.E)).astype(np.float32)   # many exact ties
    logits[0] = 1.0                                                   # all equal
    check(cfg, logits, "ties")
    bias = -3.0 * np.log(rng.permutation(cfg.E) + 1.0)
    logits = (rng.standard_normal((cfg.T, cfg.E)) * 0.3 + bias).astype(np.float32)
    got = check(cfg, logits, "skew")
    assert (got["counts"] == 0).any()
    one = np.zeros((cfg.T, cfg.E), np.float32)
    one[:, 17] = 5.0
    check(moe_synth.small_config(T=600, d=64, E=48, k=1, I=64), one, "one-expert")


def test_route_is_bitwise_repeatable():
    cfg = moe_synth.CONFIGS[4]
    inp = moe_synth.make_inputs(cfg, with_weights=False, with_dy=False)
    logits = inp["logits"].numpy()
    say(f"[route] repeat {cfg.name}")
    first = run_route(cfg, logits)
    for _ in range(9):
        again = run_route(cfg, logits)
        for key in first:
            assert np.array_equal(first[key], again[key]), key


@pytest.mark.parametrize("cid", [2, 3, 4])
def test_route_full_size_configs(cid):
    cfg = moe_synth.CONFIGS[cid]
    inp = moe_synth.make_inputs(cfg, with_weights=False, with_dy=False)
    got = check(cfg, inp["logits"].numpy(), cfg.name)
    say(f"[route] {cfg.name} histogram {moe_synth.histogram_summary(got['counts'])}")


def test_route_empty_batch():
    import paper_2604_19241_amd as moe
    shape = moe.make_shape(T=0, d=64, E=8, k=2, I=64)
    r = moe.moe_route(shape, torch.empty((0, 8), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    assert r.counts.cpu().tolist() == [0] * 8
    assert r.offsets.cpu().tolist() == [0] * 9


@pytest.mark.parametrize("kw", [
    dict(T=300, d=64, E=128, k=8, I=64),
    dict(T=65, d=64, E=1024, k=16, I=64),
    dict(T=129, d=64, E=5, k=5, I=64),
    dict(T=40, d=64, E=7, k=1, I=64),
])
def test_route_backward_matches_oracle(kw):
    """dlogits from the gate gradients: parity with the oracle (fp32 arithmetic on the GPU, the
    gates themselves are fp32: rtol 1e-5), exact zeros for unselected experts."""
    import paper_2604_19241_amd as moe
    cfg = moe_synth.small_config(**kw)
    say(f"[route-bwd] {cfg.shape_dict()}")
    rng = np.random.default_rng(17)
    logits = rng.normal(0, 1.5, (cfg.T, cfg.E)).astype(np.float32)
    g = rng.normal(0, 1, (cfg.T, cfg.k)).astype(np.float32)
    want_r = oracle.route(cfg.shape_dict(), logits)
    want = oracle.route_backward(cfg.shape_dict(), logits, want_r["topk_idx"], g)
    shape = moe.make_shape(**cfg.shape_dict())
    routing = moe.moe_route(shape, torch.from_numpy(logits).cuda())
    got = moe.moe_route_backward(shape, routing, torch.from_numpy(g).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64)
    assert np.array_equal(routing.topk_idx.cpu().numpy(), want_r["topk_idx"])
    mask = np.zeros((cfg.T, cfg.E), bool)
    np.put_along_axis(mask, want_r["topk_idx"].astype(np.int64), True, axis=1)
    assert (got[~mask] == 0).all()
    assert np.allclose(got, want, rtol=1e-5, atol=2e-7), np.abs(got - want).max()
