"""Pins of the performance-model oracle (Section 4.2, Algorithm 2; search space of
Section 6.2) against what the paper prints and what the equations fix:
hand-worked configurations through both branches of each stage, the printed
constants and choice counts, the tuned configurations of the paper's table as
members of the enumerated space, saturation points of the effective bandwidth,
time-scale homogeneity, and optimality of the search result over the space."""
import json
import math
import random
from pathlib import Path

import pytest

from oracle import perf_model as pm

GOLDEN = Path(__file__).parent / "golden"
PAPER = json.loads((GOLDEN / "perf_model_paper_values.json").read_text())
WORKED = json.loads((GOLDEN / "perf_model_worked_example.json").read_text())

HOPPER_132 = pm.Hardware(n_sm=132, p_peak=989e12, beta_hbm=3.35e12, beta_link=200e9)
HOPPER_78 = pm.Hardware(n_sm=78, p_peak=148e12, beta_hbm=3.90e12, beta_link=400e9)


def worked_hw():
    h = WORKED["hardware"]
    return pm.Hardware(n_sm=h["n_sm"], p_peak=h["p_peak"], beta_hbm=h["beta_hbm"], beta_link=h["beta_link"],
                       w_sat=h["w_sat"], tau_sync=h["tau_sync"], mu=tuple(h["mu"]))


def test_defaults_are_the_printed_constants():
    h = HOPPER_132
    assert h.w_sat == PAPER["w_sat"] and h.tau_sync == PAPER["tau_sync_s"]
    for w, mu in PAPER["mu"].items():
        assert h.mu[pm.WARP_CHOICES.index(int(w))] == mu
    assert len(pm.WARP_CHOICES) == PAPER["space_132_sms"]["warp_choices"]


def test_expected_destinations_matches_the_printed_value():
    assert abs(pm.expected_destinations(8, 8) - PAPER["expected_destinations_top8_w8"]) < 5e-3
    assert pm.expected_destinations(1, 8) == 1.0            # one rank: every slot stays there
    assert abs(pm.expected_destinations(64, 1) - 1.0) < 1e-12   # top-1: one destination


def test_worked_volumes():
    p = pm.Problem(**WORKED["problem"])
    v = WORKED["volumes"]
    assert pm.v_nvl(p) == v["v_nvl"] and pm.v_hbm_dispatch(p) == v["v_hbm_dispatch"]
    assert pm.v_hbm_total(p) == v["v_hbm_total"]
    assert (pm.row_tiles(p), pm.n_tiles_up(p), pm.n_tiles_down(p)) == (v["row_tiles"], v["n_tiles_up"], v["n_tiles_down"])


@pytest.mark.parametrize("case", WORKED["cases"], ids=["comm_bound_no_leftover", "compute_bound_leftover"])
def test_worked_configurations(case):
    got = pm.evaluate(worked_hw(), pm.Problem(**WORKED["problem"]), pm.Config(**case["config"]))
    for key, want in case["expect"].items():
        assert math.isclose(got[key], want, rel_tol=1e-12), (key, got[key], want)


def test_effective_bandwidth_saturates_at_w_sat_warps():
    beta = 3.35e12
    assert pm.effective_bandwidth(32, beta, 32, 1024) == beta          # 32 workers x 32 warps = w_sat
    assert pm.effective_bandwidth(16, beta, 32, 1024) == beta / 2
    assert pm.effective_bandwidth(132, beta, 32, 1024) == beta
    assert pm.effective_bandwidth(1, beta, 8, 1024) == beta / 128


def test_search_space_counts_on_132_sms():
    s = PAPER["space_132_sms"]
    assert len(pm.comm_choices(132)) == s["n_disp_choices"] == s["n_comb_choices"]
    relay_total = sum(len(pm.relay_choices(n)) for n in pm.comm_choices(132))
    assert relay_total == 289                                          # 1,1,2,2,...,16,16,17
    assert int(relay_total / len(pm.comm_choices(132))) == s["n_relay_choices_on_average"]
    # steps of 16 from 1 give 9 values on 132 SMs, and N_SM itself is appended: the printed 8 is
    # the rounded N_SM / 16, as the printed total is the product of rounded factors
    assert pm.reduce_choices(132) == [1, 17, 33, 49, 65, 81, 97, 113, 129, 132]
    assert 132 // 16 == s["n_red_choices"]
    assert 33 * 33 * 8 * 8 * 3 == s["printed_total"]
    n_enum = sum(1 for _ in pm.search_space(HOPPER_132))
    assert n_enum == relay_total * 33 * 10 * 3


def test_every_tuned_configuration_of_the_paper_is_in_the_space():
    space = set(pm.search_space(HOPPER_78))
    for row in PAPER["tuned_cluster2_78_sms"]:
        c = pm.Config(row["n_disp"], row["n_relay"], row["n_comb"], row["n_red"], row["warps"])
        assert c in space, row
        assert pm.is_valid(HOPPER_78, c), row


def test_time_scale_homogeneity():
    p = pm.Problem(n_tok=4096, h_dim=2048, h_inter=768, n_exp=128, top_k=8, world=8)
    rng = random.Random(5)
    space = [c for c in pm.search_space(HOPPER_132) if pm.is_valid(HOPPER_132, c)]
    s = 4.0   # a machine four times faster in every rate, with a quarter of the sync overhead
    fast = pm.Hardware(n_sm=132, p_peak=989e12 * s, beta_hbm=3.35e12 * s, beta_link=200e9 * s, tau_sync=2e-6 / s)
    for c in rng.sample(space, 200):
        a, b = pm.evaluate(HOPPER_132, p, c), pm.evaluate(fast, p, c)
        for key in a:
            assert math.isclose(a[key], s * b[key], rel_tol=1e-12), key


def test_search_returns_the_first_minimum_of_the_space():
    p = pm.Problem(n_tok=2048, h_dim=2048, h_inter=768, n_exp=128, top_k=8, world=8)
    best, l_min, n_enum, n_valid = pm.search(HOPPER_78, p)
    assert pm.is_valid(HOPPER_78, best) and 0 < n_valid <= n_enum
    seen_best = False
    for c in pm.search_space(HOPPER_78):
        if not pm.is_valid(HOPPER_78, c):
            continue
        l = pm.evaluate(HOPPER_78, p, c)["l_total"]
        assert l >= l_min
        if c == best:
            seen_best = True
            assert l == l_min
        elif not seen_best:
            assert l > l_min     # nothing earlier in the enumeration ties with the winner


def test_invalid_configurations_are_skipped():
    h = pm.Hardware(n_sm=16, p_peak=1e14, beta_hbm=1e12, beta_link=1e11)
    assert not pm.is_valid(h, pm.Config(16, 1, 4, 1, 8))     # no compute worker left in stage 1
    assert not pm.is_valid(h, pm.Config(4, 1, 16, 1, 8))     # none in stage 2
    assert not pm.is_valid(h, pm.Config(12, 5, 4, 1, 8))     # N_disp + N_relay must stay below N_SM
    assert pm.is_valid(h, pm.Config(12, 1, 4, 16, 8))
    best, _, n_enum, n_valid = pm.search(h, pm.Problem(n_tok=512, h_dim=1024, h_inter=512, n_exp=16, top_k=2, world=4))
    assert n_valid < n_enum and pm.is_valid(h, best)
