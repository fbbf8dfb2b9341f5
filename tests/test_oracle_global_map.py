"""Pins of the multi-rank token-mapping oracle (oracle/global_map.py) against
what the paper and the mathematics fix: a hand-worked example, the defining
property (the destination order equals one stable sort of the rank-concatenated
tokens, Section 3.1), bijectivity, the one-rank special case, and the
distinct-destination statistics of Section 3.2's probability table."""
import json
import math
from itertools import product
from pathlib import Path

import numpy as np
import pytest

from oracle import global_map as gm

GOLDEN = Path(__file__).resolve().parent / "golden"


def random_selection(rng, n_tok, n_exp, k):
    """Distinct experts per token, as top-k produces them."""
    return np.stack([rng.permutation(n_exp)[:k] for _ in range(n_tok)]).astype(np.int32) \
        if n_tok else np.zeros((0, k), np.int32)


def test_hand_worked_example():
    ex = json.loads((GOLDEN / "global_map_worked_example.json").read_text())
    out = gm.global_map([np.array(e, np.int32) for e in ex["e_sel_per_rank"]], ex["n_exp"])
    assert out["c_all"].tolist() == ex["c_all"]
    assert out["o_all"].tolist() == ex["o_all"]
    assert out["recv_offsets"].tolist() == ex["recv_offsets"]
    for got, want in zip(out["ranks"], ex["ranks"]):
        for key, v in want.items():
            assert got[key].tolist() == v, key


@pytest.mark.parametrize("W,n_exp,k,toks", [
    (2, 8, 2, [5, 9]), (4, 16, 4, [7, 0, 12, 3]), (8, 64, 8, [20] * 8), (1, 6, 3, [11]),
    (4, 8, 8, [6, 6, 6, 6]),
])
def test_destination_order_is_the_stable_sort_of_the_concatenated_tokens(W, n_exp, k, toks):
    rng = np.random.default_rng(1234 + W * 100 + n_exp)
    sel = [random_selection(rng, n, n_exp, k) for n in toks]
    out = gm.global_map(sel, n_exp)
    n_epr = n_exp // W
    flat = np.concatenate([s.reshape(-1) for s in sel])       # (rank, token, slot) order
    order = np.argsort(flat, kind="stable")                   # library routine
    pos = np.empty_like(order)
    pos[order] = np.arange(order.size)                        # global sorted position of every slot
    first_of_expert = np.searchsorted(np.sort(flat, kind="stable"), np.arange(n_exp))
    got_row = np.concatenate([r["dst_row"].reshape(-1) for r in out["ranks"]])
    got_off = np.concatenate([r["dst_off"].reshape(-1) for r in out["ranks"]])
    got_rank = np.concatenate([r["dst_rank"].reshape(-1) for r in out["ranks"]])
    got_eloc = np.concatenate([r["dst_expert"].reshape(-1) for r in out["ranks"]])
    assert np.array_equal(got_rank, flat // n_epr)
    assert np.array_equal(got_eloc, flat % n_epr)
    # inside its expert: rank among all slots of that expert in (rank, token, slot) order
    assert np.array_equal(got_off, pos - first_of_expert[flat])
    # inside its destination rank: sorted position minus everything sorted before that rank
    assert np.array_equal(got_row, pos - first_of_expert[(flat // n_epr) * n_epr])
    # every destination rank's rows are a bijection onto [0, rows it receives)
    for rt in range(W):
        rows = np.sort(got_row[got_rank == rt])
        assert np.array_equal(rows, np.arange(rows.size))
        assert out["recv_offsets"][rt, -1] == rows.size


def test_one_rank_reduces_to_the_local_stable_sort():
    rng = np.random.default_rng(5)
    sel = random_selection(rng, 40, 8, 2)
    out = gm.global_map([sel], 8)
    r = out["ranks"][0]
    assert (r["dst_rank"] == 0).all() and np.array_equal(r["dst_expert"], sel)
    assert np.array_equal(r["dst_row"], r["m_loc"])
    assert np.array_equal(r["dst_row"].reshape(-1),
                          np.argsort(np.argsort(sel.reshape(-1), kind="stable"), kind="stable"))
    assert (r["send"][:, 0] == 1).all() and (r["n_dst_ranks"] == 1).all()


def test_send_marks_first_slot_per_destination_rank_brute_force():
    """All 4^4 assignments of four slots to four ranks (one expert per rank, repeats allowed):
    the number of distinct ranks follows C(4,x) x! S2(4,x) / 4^4, and `send` is the indicator of
    a first occurrence."""
    sel = np.array(list(product(range(4), repeat=4)), np.int32)
    out = gm.global_map([sel], 4)       # W = 1 would put all experts on one rank: use 4 ranks below
    out4 = gm.global_map([sel, np.zeros((0, 4), np.int32), np.zeros((0, 4), np.int32),
                          np.zeros((0, 4), np.int32)], 4)
    r = out4["ranks"][0]
    for t, row in enumerate(sel):
        want = [1 if row[j] not in row[:j] else 0 for j in range(4)]
        assert r["send"][t].tolist() == want
        assert r["n_dst_ranks"][t] == len(set(row.tolist())) == sum(want)
    stirling = {1: 1, 2: 7, 3: 6, 4: 1}
    hist = np.bincount(r["n_dst_ranks"], minlength=5)
    for x in range(1, 5):
        assert hist[x] == math.comb(4, x) * math.factorial(x) * stirling[x]
    assert (out["ranks"][0]["n_dst_ranks"] == 1).all()


def test_distinct_destination_statistics_match_the_printed_table():
    tab = json.loads((GOLDEN / "prob_saving_table.json").read_text())
    W, k = tab["ranks"], tab["slots"]
    rng = np.random.default_rng(20260419)
    n_tok = 40000
    # independent uniform choices, as the table assumes (8^8 equally likely assignments)
    sel = rng.integers(0, 64, size=(n_tok, k)).astype(np.int32)
    out = gm.global_map([sel] + [np.zeros((0, k), np.int32)] * (W - 1), 64)
    x = out["ranks"][0]["n_dst_ranks"]
    mean = x.mean()
    assert abs(mean - tab["expected_distinct"]) < 0.03          # sigma of the mean is 0.005
    assert abs((1 - mean / k) - tab["traffic_reduction"]) < 0.01
    assert out["ranks"][0]["send"].sum() == x.sum()
    hist = np.bincount(x, minlength=k + 1) / n_tok
    for key, p in tab["p_printed"].items():
        sigma = math.sqrt(p * (1 - p) / n_tok)
        half_last_digit = 0.5 * 10 ** (math.floor(math.log10(p)) - tab["printed_digits"][key] + 1)
        assert abs(hist[int(key)] - p) <= 4 * sigma + half_last_digit + 1e-4, (key, hist[int(key)], p)
    # the closed form 8 (1 - (7/8)^8) that the printed expectation rounds
    assert abs(W * (1 - (1 - 1 / W) ** k) - tab["expected_distinct"]) < 0.005
