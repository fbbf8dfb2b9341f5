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


# ------------------------------------------------------------------ router gradient

def _gates_torch(logits, idx):
    import torch
    p = torch.softmax(logits, dim=-1)
    sel = torch.gather(p, 1, idx)
    return sel / sel.sum(dim=1, keepdim=True)


def test_route_backward_matches_autograd_and_finite_differences(oracle_mod):
    """Library pin (torch.autograd over the gate definition in float64) and central finite
    differences; a wrong sign, a dropped renormalisation term or a transposed index fails both."""
    import torch
    rng = np.random.default_rng(5)
    T, E, k = 7, 12, 4
    shape = dict(T=T, d=64, E=E, k=k, I=64, e_start=0, e_count=E)
    logits = rng.normal(0, 1.5, (T, E)).astype(np.float32)
    r = oracle_mod.route(shape, logits)
    g = rng.normal(0, 1, (T, k)).astype(np.float32)
    got = oracle_mod.route_backward(shape, logits, r["topk_idx"], g)

    lt = torch.tensor(logits, dtype=torch.float64, requires_grad=True)
    idx = torch.tensor(r["topk_idx"], dtype=torch.int64)
    w = _gates_torch(lt, idx)
    (w * torch.tensor(g, dtype=torch.float64)).sum().backward()
    assert np.allclose(got, lt.grad.numpy(), rtol=1e-9, atol=1e-12)

    def loss(l):
        with torch.no_grad():
            return float((_gates_torch(torch.tensor(l, dtype=torch.float64), idx)
                          * torch.tensor(g, dtype=torch.float64)).sum())
    eps = 1e-5
    l64 = logits.astype(np.float64)
    for (t, e) in [(0, 0), (3, int(r["topk_idx"][3, 0])), (6, int(r["topk_idx"][6, k - 1])), (2, 5)]:
        lp, lm = l64.copy(), l64.copy()
        lp[t, e] += eps
        lm[t, e] -= eps
        fd = (loss(lp) - loss(lm)) / (2 * eps)
        assert abs(fd - got[t, e]) <= 1e-7 + 1e-6 * abs(fd), (t, e, fd, got[t, e])


def test_route_backward_closed_forms(oracle_mod):
    """Unselected logits do not move the gates; the gradient of every row sums to zero (gates are
    invariant under a shift of the row); k = 1 gives a constant gate, so a zero gradient; equal
    upstream gradients give zero (the gates sum to one)."""
    rng = np.random.default_rng(6)
    T, E, k = 9, 10, 3
    shape = dict(T=T, d=64, E=E, k=k, I=64, e_start=0, e_count=E)
    logits = rng.normal(0, 1, (T, E)).astype(np.float32)
    r = oracle_mod.route(shape, logits)
    g = rng.normal(0, 1, (T, k)).astype(np.float32)
    d = oracle_mod.route_backward(shape, logits, r["topk_idx"], g)
    mask = np.zeros((T, E), bool)
    np.put_along_axis(mask, r["topk_idx"].astype(np.int64), True, axis=1)
    assert np.abs(d[~mask]).max() <= 1e-15
    assert np.abs(d.sum(1)).max() <= 1e-14
    # closed form on the selected entries: w_i (g_i - sum_j w_j g_j)
    w = r["topk_w"].astype(np.float64)
    want = w * (g - (w * g).sum(1, keepdims=True))
    assert np.allclose(np.take_along_axis(d, r["topk_idx"].astype(np.int64), 1), want, rtol=1e-6, atol=1e-9)
    same = oracle_mod.route_backward(shape, logits, r["topk_idx"], np.full((T, k), 0.7, np.float32))
    assert np.abs(same).max() <= 1e-15
    shape1 = dict(shape, k=1)
    r1 = oracle_mod.route(shape1, logits)
    d1 = oracle_mod.route_backward(shape1, logits, r1["topk_idx"], rng.normal(0, 1, (T, 1)).astype(np.float32))
    assert np.abs(d1).max() <= 1e-15
