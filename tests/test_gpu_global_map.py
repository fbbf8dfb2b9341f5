"""GPU parity of moe_global_map (Algorithm 1 with W > 1 ranks, the part one GPU
runs): W ranks' token batches are routed one after the other on the one GPU,
their histograms stacked (standing in for the AllGather), and every rank's
destination arrays must equal the multi-rank oracle bit for bit."""
import numpy as np
import pytest
import torch

import moe_synth
import oracle
from oracle import global_map as gm
from helpers import say

pytestmark = pytest.mark.gpu

KEYS = ("dst_rank", "dst_expert", "dst_off", "dst_row", "send", "n_dst_ranks")


def run_case(W, E, k, toks, seed, zipf_s=0.0):
    import paper_2604_19241_amd as moe
    say(f"[global map] W={W} E={E} k={k} tokens per rank={toks} zipf={zipf_s}")
    rng = np.random.default_rng(seed)
    bias = -zipf_s * np.log(rng.permutation(E) + 1.0) if zipf_s > 0 else np.zeros(E)
    routings, sels, shapes = [], [], []
    for r in range(W):
        cfg = moe_synth.small_config(T=toks[r], d=64, E=E, k=k, I=64)
        logits = (rng.standard_normal((cfg.T, E)) + bias).astype(np.float32)
        shape = moe.make_shape(**cfg.shape_dict())
        routings.append(moe.moe_route(shape, torch.from_numpy(logits).cuda()))
        shapes.append(shape)
        sels.append(oracle.route(cfg.shape_dict(), logits)["topk_idx"])
        assert np.array_equal(routings[-1].topk_idx.cpu().numpy(), sels[-1])
    want = gm.global_map(sels, E)
    c_all = torch.stack([r.counts for r in routings]).contiguous()     # the AllGather's result
    assert np.array_equal(c_all.cpu().numpy(), want["c_all"])
    for r in range(W):
        got = moe.moe_global_map(shapes[r], W, r, routings[r], c_all)
        torch.cuda.synchronize()
        for key in KEYS:
            assert np.array_equal(getattr(got, key).cpu().numpy(), want["ranks"][r][key]), (r, key)
        assert np.array_equal(got.recv_offsets.cpu().numpy(), want["recv_offsets"][r]), r
    return want


@pytest.mark.parametrize("W,E,k,toks", [
    (8, 128, 8, [300, 512, 0, 700, 256, 1, 333, 640]),   # ragged batches, one rank without tokens
    (2, 8, 2, [1000, 37]),
    (4, 1024, 16, [130, 64, 200, 99]),                   # the shape limits
    (1, 16, 4, [500]),                                   # one rank: the local stable sort itself
    (64, 64, 6, [40] * 64),                              # one expert per rank, the rank limit
    (8, 512, 10, [257] * 8),
])
def test_global_map_matches_oracle(W, E, k, toks):
    run_case(W, E, k, toks, seed=7 * W + E)


def test_global_map_skewed_routing_and_statistics():
    """Zipf-biased routing; also the distinct-destination count of uniform top-8 over 8 ranks,
    which for distinct experts (16 per rank) averages 8 (1 - C(112,8)/C(128,8)) = 5.34."""
    run_case(8, 128, 8, [400] * 8, seed=3, zipf_s=1.2)
    want = run_case(8, 128, 8, [2000] * 8, seed=4)
    x = np.concatenate([r["n_dst_ranks"] for r in want["ranks"]])
    from math import comb
    assert abs(x.mean() - 8 * (1 - comb(112, 8) / comb(128, 8))) < 0.03


def test_global_map_is_bitwise_repeatable():
    import paper_2604_19241_amd as moe
    cfg = moe_synth.small_config(T=3000, d=64, E=128, k=8, I=64)
    rng = np.random.default_rng(11)
    logits = torch.from_numpy(rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)).cuda()
    shape = moe.make_shape(**cfg.shape_dict())
    r = moe.moe_route(shape, logits)
    c_all = torch.stack([r.counts] * 8).contiguous()
    first = moe.moe_global_map(shape, 8, 5, r, c_all)
    for _ in range(5):
        again = moe.moe_global_map(shape, 8, 5, r, c_all)
        for key in KEYS + ("recv_offsets",):
            assert torch.equal(getattr(first, key), getattr(again, key)), key
