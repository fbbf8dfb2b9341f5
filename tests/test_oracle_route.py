"""Pins of the oracle's routing / index stage against things other than itself.

Reference points: the hand-worked example in tests/golden (Algorithm 1 with one
rank), a full lexicographic sort per row (library sort) for top-k, numpy's
stable argsort for the permutation, an O(A^2) rank count straight from the
definition, and the invariants the paper states (unique, conflict-free
destination rows; contiguous per-expert segments in source order).
"""
import json
from pathlib import Path

import numpy as np
import pytest

GOLD = Path(__file__).parent / "golden"
ACCS = ["f64", "f32"]


def shape(T, E, k, e_start=0, e_count=None, d=8, I=8):
    return dict(T=T, d=d, E=E, k=k, I=I, e_start=e_start,
                e_count=E if e_count is None else e_count)


def brute_topk(logits, k):
    """Full sort of (-value, index) per row; the first k are the selection."""
    T, E = logits.shape
    out = np.empty((T, k), np.int32)
    for t in range(T):
        order = np.lexsort((np.arange(E), -logits[t].astype(np.float64)))
        out[t] = order[:k]
    return out


def brute_index(topk_idx, e_start, e_count):
    """Rows from the definition: offsets[e] + #{same-expert flat slots f' < f}."""
    flat = topk_idx.reshape(-1)
    F = flat.size
    local = (flat >= e_start) & (flat < e_start + e_count)
    counts = np.array([(flat == e_start + e).sum() for e in range(e_count)], np.int32)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    inv = np.full(F, -1, np.int32)
    for f in range(F):
        if local[f]:
            rank = int(((flat[:f] == flat[f])).sum())
            inv[f] = offsets[flat[f] - e_start] + rank
    perm = np.full(F, -1, np.int32)
    for f in range(F):
        if inv[f] >= 0:
            perm[inv[f]] = f
    return counts, offsets, perm, inv.reshape(topk_idx.shape)


@pytest.mark.parametrize("acc", ACCS)
def test_hand_worked_example(oracle_mod, acc):
    g = json.loads((GOLD / "route_worked_example.json").read_text())
    r = oracle_mod.route(g["shape"], np.array(g["logits"], np.float32), acc=acc)
    for key in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(r[key], np.array(g[key], np.int32)), key
    assert np.allclose(r["topk_w"], np.array(g["topk_w"]), rtol=0, atol=1e-7)


@pytest.mark.parametrize("acc", ACCS)
@pytest.mark.parametrize("T,E,k", [(37, 8, 2), (64, 16, 4), (50, 128, 8), (9, 5, 5), (33, 7, 1)])
def test_topk_matches_full_sort(oracle_mod, acc, T, E, k):
    rng = np.random.default_rng(T * 1000 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    r = oracle_mod.route(shape(T, E, k), logits, acc=acc)
    assert np.array_equal(r["topk_idx"], brute_topk(logits, k))


def test_topk_ties_go_to_lower_expert(oracle_mod):
    E, k = 12, 4
    rows = [
        np.ones(E),                                   # all equal -> 0,1,2,3
        np.array([0, 2, 2, 2, 1, 2, 0, 0, 0, 0, 0, 2]),  # five 2s -> 1,2,3,5
        np.array([5, 5, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1]),  # 0,1 then the 1s -> 2,3
        -np.arange(E),                                # descending -> 0..3
        np.arange(E),                                 # ascending -> 11,10,9,8
    ]
    # quantised random rows: many exact ties
    rng = np.random.default_rng(3)
    rows += [rng.integers(0, 3, E) for _ in range(40)]
    logits = np.array(rows, np.float32)
    r = oracle_mod.route(shape(len(rows), E, k), logits)
    assert r["topk_idx"][0].tolist() == [0, 1, 2, 3]
    assert r["topk_idx"][1].tolist() == [1, 2, 3, 5]
    assert r["topk_idx"][2].tolist() == [0, 1, 2, 3]
    assert r["topk_idx"][3].tolist() == [0, 1, 2, 3]
    assert r["topk_idx"][4].tolist() == [11, 10, 9, 8]
    assert np.array_equal(r["topk_idx"], brute_topk(logits, k))


@pytest.mark.parametrize("acc", ACCS)
def test_gate_weights_are_renormalised_softmax(oracle_mod, acc):
    T, E, k = 200, 64, 8
    rng = np.random.default_rng(11)
    logits = (rng.standard_normal((T, E)) * 1.5).astype(np.float32)
    r = oracle_mod.route(shape(T, E, k), logits, acc=acc)
    l64 = logits.astype(np.float64)
    p = np.exp(l64 - l64.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    sel = np.take_along_axis(p, r["topk_idx"].astype(np.int64), axis=1)
    w = sel / sel.sum(1, keepdims=True)
    tol = 1e-7 if acc == "f64" else 1e-6
    assert np.allclose(r["topk_w"], w, rtol=tol, atol=tol)
    assert np.allclose(r["topk_w"].astype(np.float64).sum(1), 1.0, atol=1e-6)
    # slots are ordered by decreasing logit, hence by decreasing gate
    assert (np.diff(r["topk_w"], axis=1) <= 1e-7).all()


@pytest.mark.parametrize("T,E,k,e_start,e_count", [
    (40, 8, 2, 0, 8), (40, 8, 2, 2, 3), (64, 32, 8, 8, 8), (31, 16, 4, 12, 4), (17, 6, 6, 0, 6),
    (25, 8, 1, 7, 1)])
def test_index_matches_definition_and_stable_argsort(oracle_mod, T, E, k, e_start, e_count):
    rng = np.random.default_rng(T + 31 * E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    r = oracle_mod.route(shape(T, E, k, e_start, e_count), logits)
    counts, offsets, perm, inv = brute_index(r["topk_idx"], e_start, e_count)
    assert np.array_equal(r["counts"], counts)
    assert np.array_equal(r["offsets"], offsets)
    assert np.array_equal(r["perm"], perm)
    assert np.array_equal(r["inv_perm"], inv)
    # library routine: a stable argsort of the flat expert ids of the local slots
    flat = r["topk_idx"].reshape(-1)
    local = np.nonzero((flat >= e_start) & (flat < e_start + e_count))[0]
    order = local[np.argsort(flat[local], kind="stable")]
    A = int(offsets[-1])
    assert A == local.size
    assert np.array_equal(r["perm"][:A], order.astype(np.int32))
    assert (r["perm"][A:] == -1).all()


def test_index_invariants_skewed_and_empty(oracle_mod):
    """All tokens to few experts, some experts empty (Zipf-like bias)."""
    T, E, k = 300, 32, 4
    rng = np.random.default_rng(5)
    bias = -3.0 * np.log(rng.permutation(E) + 1.0)
    logits = (rng.standard_normal((T, E)) * 0.3 + bias).astype(np.float32)
    r = oracle_mod.route(shape(T, E, k), logits)
    A = int(r["offsets"][-1])
    assert A == T * k == int(r["counts"].sum())
    assert (r["counts"] == 0).any(), "test wants at least one empty expert"
    assert (np.diff(r["offsets"]) == r["counts"]).all()
    # unique, conflict-free destination rows (bijection on [0, A))
    assert np.array_equal(np.sort(r["perm"][:A]), np.arange(A))
    inv = r["inv_perm"].reshape(-1)
    assert np.array_equal(r["perm"][inv], np.arange(T * k))
    # per-expert segments hold that expert's slots in increasing flat order
    flat = r["topk_idx"].reshape(-1)
    for e in range(E):
        seg = r["perm"][r["offsets"][e]:r["offsets"][e + 1]]
        assert (flat[seg] == e).all()
        assert (np.diff(seg) > 0).all()


def test_all_tokens_one_expert(oracle_mod):
    T, E, k = 50, 4, 1
    logits = np.zeros((T, E), np.float32)
    logits[:, 2] = 1.0
    r = oracle_mod.route(shape(T, E, k), logits)
    assert r["counts"].tolist() == [0, 0, T, 0]
    assert r["offsets"].tolist() == [0, 0, 0, T, T]
    assert np.array_equal(r["perm"], np.arange(T))
    assert np.allclose(r["topk_w"], 1.0)


def test_bad_shapes_rejected(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.route(shape(4, 4, 5), np.zeros((4, 4), np.float32))
    with pytest.raises(ValueError):
        oracle_mod.route(shape(4, 4, 2, 3, 2), np.zeros((4, 4), np.float32))
