"""The library's performance model and configuration search (host code behind the
C ABI: moe_perf_model_eval, moe_perf_model_search) against the Python oracle:
every intermediate of Algorithm 2's loop body to 1e-12 relative on random
hardware / problems / configurations, and the search result (configuration
chosen, counts of enumerated and valid configurations) exactly, on the paper's
two clusters, an MI355X-like parameter set and small chips where part of the
space is invalid.  No GPU is needed: the entry points never touch one."""
import math
import random

import pytest

import moe_synth
import paper_2604_19241_amd as moe
from oracle import perf_model as pm

HW = {
    "hopper_132": dict(n_sm=132, p_peak=989e12, beta_hbm=3.35e12, beta_link=200e9),
    "hopper_78": dict(n_sm=78, p_peak=148e12, beta_hbm=3.90e12, beta_link=400e9),
    # 256 CUs, dense bf16 MFMA peak, HBM3E, one xGMI link direction; waves of 64 lanes
    "mi355x_like": dict(n_sm=256, p_peak=2.5e15, beta_hbm=8e12, beta_link=153e9 / 2),
    "tiny_16": dict(n_sm=16, p_peak=1e14, beta_hbm=1e12, beta_link=1e11),
    "tiny_9": dict(n_sm=9, p_peak=1e14, beta_hbm=1e12, beta_link=1e11, w_sat=64, tau_sync=5e-6, mu=(0.5, 0.45, 0.4)),
}


def both(hw_kw, pr_kw):
    return (pm.Hardware(**hw_kw), pm.Problem(**pr_kw)), (moe.make_perf_hw(**hw_kw), moe.make_perf_problem(**pr_kw))


def model_problem(mid, n_tok, world, b_m=128, b_n=128):
    name, d, inter, e, k = moe_synth.MODEL_SHAPES[mid]
    return dict(n_tok=n_tok, h_dim=d, h_inter=inter, n_exp=e, top_k=k, world=world, b_m=b_m, b_n=b_n)


def random_valid_configs(rng, h, n):
    out = []
    while len(out) < n:
        n_disp = rng.choice(pm.comm_choices(h.n_sm))
        c = pm.Config(n_disp, rng.choice(pm.relay_choices(n_disp)), rng.choice(pm.comm_choices(h.n_sm)),
                      rng.choice(pm.reduce_choices(h.n_sm)), rng.choice(pm.WARP_CHOICES))
        if pm.is_valid(h, c):
            out.append(c)
    return out


@pytest.mark.parametrize("hw_name", list(HW))
def test_eval_matches_oracle_on_random_configurations(hw_name):
    rng = random.Random(hash(hw_name) & 0xffff)
    hw_kw = HW[hw_name]
    for trial in range(40):
        mid = rng.choice(sorted(moe_synth.MODEL_SHAPES))
        pr_kw = model_problem(mid, rng.choice([1, 7, 512, 4096, 32768]), rng.choice([1, 2, 4, 8]),
                              rng.choice([64, 128, 256]), rng.choice([128, 256]))
        (oh, op), (ch, cp) = both(hw_kw, pr_kw)
        for c in random_valid_configs(rng, oh, 5):
            want = pm.evaluate(oh, op, c)
            got = moe.moe_perf_model_eval(ch, cp, (c.n_disp, c.n_relay, c.n_comb, c.n_red, c.warps))
            for key, v in want.items():
                assert math.isclose(got[key], v, rel_tol=1e-12, abs_tol=0.0), (key, got[key], v, pr_kw, c)


# the oracle walks the space in pure Python (about 30 us per configuration): 34 200 configurations on
# 78 workers, 286 110 on 132; the 256-worker space (3.4 million) is left to the property test below
SEARCH_CASES = [("hopper_78", mid, 32768, 8) for mid in (1, 5, 6, 9, 11)] + [
    ("hopper_132", 6, 8192, 8), ("tiny_16", 10, 512, 4), ("tiny_9", 2, 64, 2), ("hopper_78", 6, 1, 1),
]


@pytest.mark.parametrize("hw_name,mid,n_tok,world", SEARCH_CASES)
def test_search_matches_oracle(hw_name, mid, n_tok, world):
    (oh, op), (ch, cp) = both(HW[hw_name], model_problem(mid, n_tok, world))
    best, l_min, n_enum, n_valid = pm.search(oh, op)
    got = moe.moe_perf_model_search(ch, cp)
    assert got["config"] == (best.n_disp, best.n_relay, best.n_comb, best.n_red, best.warps)
    assert (got["n_enumerated"], got["n_valid"]) == (n_enum, n_valid)
    assert math.isclose(got["latency"]["l_total"], l_min, rel_tol=1e-12)
    want = pm.evaluate(oh, op, best)
    for key, v in want.items():
        assert math.isclose(got["latency"][key], v, rel_tol=1e-12), key


def test_search_on_256_workers_is_a_minimum_of_sampled_configurations():
    (oh, op), (ch, cp) = both(HW["mi355x_like"], model_problem(6, 8192, 8, b_m=256, b_n=256))
    got = moe.moe_perf_model_search(ch, cp)
    relay_total = sum(len(pm.relay_choices(n)) for n in pm.comm_choices(256))
    assert got["n_enumerated"] == relay_total * 64 * len(pm.reduce_choices(256)) * 3
    best = pm.Config(*got["config"])
    assert pm.is_valid(oh, best)
    l_best = pm.evaluate(oh, op, best)["l_total"]
    assert math.isclose(l_best, got["latency"]["l_total"], rel_tol=1e-12)
    rng = random.Random(11)
    for c in random_valid_configs(rng, oh, 3000):
        assert pm.evaluate(oh, op, c)["l_total"] >= l_best
    # and no neighbour in any single coordinate is better
    d, r, cb, rd, w = got["config"]
    for c in [pm.Config(d + s, r, cb, rd, w) for s in (-4, 4)] + [pm.Config(d, r + s, cb, rd, w) for s in (-4, 4)] + \
             [pm.Config(d, r, cb + s, rd, w) for s in (-4, 4)] + [pm.Config(d, r, cb, x, w) for x in pm.reduce_choices(256)] + \
             [pm.Config(d, r, cb, rd, x) for x in pm.WARP_CHOICES]:
        if pm.is_valid(oh, c) and c.n_disp >= 4 and c.n_comb >= 4 and c.n_relay >= 1:
            assert pm.evaluate(oh, op, c)["l_total"] >= l_best, c


def test_argument_checks():
    hw = moe.make_perf_hw(**HW["hopper_132"])
    pr = moe.make_perf_problem(**model_problem(6, 4096, 8))
    ok = (12, 5, 20, 132, 32)
    moe.moe_perf_model_eval(hw, pr, ok)
    for bad in [(132, 1, 20, 1, 32), (12, 5, 132, 1, 32), (128, 5, 20, 1, 32), (12, 0, 20, 1, 32),
                (12, 5, 20, 0, 32), (12, 5, 20, 133, 32), (12, 5, 20, 1, 24), (0, 1, 20, 1, 8)]:
        with pytest.raises(moe.MoEError) as e:
            moe.moe_perf_model_eval(hw, pr, bad)
        assert e.value.code == -2, bad
    with pytest.raises(moe.MoEError):
        moe.moe_perf_model_eval(hw, moe.make_perf_problem(**model_problem(6, 4096, 7)), ok)   # 128 % 7 != 0
    with pytest.raises(moe.MoEError):
        moe.moe_perf_model_eval(moe.make_perf_hw(n_sm=132, p_peak=0.0, beta_hbm=1e12, beta_link=1e11), pr, ok)
    with pytest.raises(moe.MoEError):   # more workers than the search is sized for
        moe.moe_perf_model_search(moe.make_perf_hw(n_sm=1025, p_peak=1e14, beta_hbm=1e12, beta_link=1e11), pr)
    with pytest.raises(moe.MoEError):   # four workers: no valid configuration at all
        moe.moe_perf_model_search(moe.make_perf_hw(n_sm=4, p_peak=1e14, beta_hbm=1e12, beta_link=1e11), pr)
    lib = moe.load_library()
    assert lib.moe_perf_model_eval(None, None, None, None) == -1
    assert lib.moe_perf_model_search(None, None, None, None, None, None) == -1
