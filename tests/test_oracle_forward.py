"""Pins of the oracle's forward pass against things other than itself.

* dense brute force: every token through every expert with numpy matmul, scaled
  by a gate matrix that is zero off the top-k (what the routed layer must equal);
* E=1, k=1 reduces to a textbook SwiGLU MLP evaluated by torch in fp64;
* identity-like experts reproduce the input (top-1 and top-k with gates summing
  to one: permute, then un-permute, is the identity);
* the bf16 rounding rule against torch's float32 -> bfloat16 cast;
* rounded outputs are bf16 values, and rounding moves results by bf16 noise only.
"""
import numpy as np
import pytest
import torch

import moe_synth


def f64_inputs(cfg, seed):
    inp = moe_synth.make_inputs(cfg, seed=seed)
    out = {key: v.double().numpy() for key, v in inp.items() if key != "logits"}
    out["logits"] = inp["logits"].numpy()
    return inp, out


def dense_brute_force(x, wg, wu, wd, logits, k, e_start, e_count):
    """y = sum_e gate[t,e] * MLP_e(x[t]) with a dense gate (zero off the top-k, zero for
    non-local experts).  numpy fp64, library matmul."""
    T, E = logits.shape
    l64 = logits.astype(np.float64)
    order = np.stack([np.lexsort((np.arange(E), -l64[t])) for t in range(T)])[:, :k]
    p = np.exp(l64 - l64.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    sel = np.take_along_axis(p, order, 1)
    w = sel / sel.sum(1, keepdims=True)
    gate = np.zeros((T, E))
    np.put_along_axis(gate, order, w, 1)
    y = np.zeros_like(x)
    for el in range(e_count):
        G = x @ wg[el]
        U = x @ wu[el]
        h = G / (1.0 + np.exp(-G)) * U
        y += gate[:, e_start + el:e_start + el + 1] * (h @ wd[el])
    return y


@pytest.mark.parametrize("T,d,E,k,I,e_start,e_count", [
    (48, 32, 8, 2, 40, 0, 8), (33, 24, 16, 4, 16, 0, 16), (40, 16, 16, 4, 24, 4, 8),
    (21, 8, 6, 6, 8, 0, 6), (30, 16, 8, 1, 8, 0, 8)])
def test_routed_equals_dense_masked_brute_force(oracle_mod, T, d, E, k, I, e_start, e_count):
    cfg = moe_synth.small_config(T=T, d=d, E=E, k=k, I=I, e_start=e_start, e_count=e_count)
    _, a = f64_inputs(cfg, seed=7 + T)
    # larger weights so that silu is exercised away from its linear region
    wg, wu, wd = a["w_gate"] * 20, a["w_up"] * 20, a["w_down"] * 20
    r = oracle_mod.route(cfg.shape_dict(), a["logits"])
    got = oracle_mod.forward(cfg.shape_dict(), a["x"], wg, wu, wd, r, round_bf16=False)["y"]
    want = dense_brute_force(a["x"], wg, wu, wd, a["logits"], k, e_start, e_count)
    scale = np.abs(want).max()
    assert scale > 1e-3
    # the fp32 gate the interface carries limits agreement to ~1e-7 relative
    assert np.abs(got - want).max() <= 3e-7 * scale


def test_single_expert_is_a_swiglu_mlp(oracle_mod):
    cfg = moe_synth.small_config(T=29, d=48, E=1, k=1, I=72)
    _, a = f64_inputs(cfg, seed=3)
    wg, wu, wd = a["w_gate"] * 10, a["w_up"] * 10, a["w_down"] * 10
    r = oracle_mod.route(cfg.shape_dict(), a["logits"])
    assert np.array_equal(r["perm"], np.arange(cfg.T))
    assert np.allclose(r["topk_w"], 1.0)
    got = oracle_mod.forward(cfg.shape_dict(), a["x"], wg, wu, wd, r, round_bf16=False,
                             stages=True)
    X = torch.from_numpy(a["x"])
    Gt = X @ torch.from_numpy(wg[0])
    Ut = X @ torch.from_numpy(wu[0])
    ht = torch.nn.functional.silu(Gt) * Ut
    want = ht @ torch.from_numpy(wd[0])
    assert np.allclose(got["G"], Gt.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(got["U"], Ut.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(got["h"], ht.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(got["o"], want.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(got["y"], want.numpy(), rtol=1e-12, atol=1e-12)


def identity_like_experts(E, n, c=2.0):
    """x[:,0] = 1, W_gate = c in row 0 (so G == c), W_up = I, W_down = I / silu(c):
    each expert returns its input."""
    wg = np.zeros((E, n, n))
    wg[:, 0, :] = c
    wu = np.stack([np.eye(n)] * E)
    silu_c = c / (1.0 + np.exp(-c))
    wd = np.stack([np.eye(n) / silu_c] * E)
    return wg, wu, wd


@pytest.mark.parametrize("k", [1, 3])
def test_identity_experts_reproduce_input(oracle_mod, k):
    T, n, E = 37, 20, 6
    rng = np.random.default_rng(k)
    x = rng.standard_normal((T, n))
    x[:, 0] = 1.0
    logits = rng.standard_normal((T, E)).astype(np.float32)
    sh = dict(T=T, d=n, E=E, k=k, I=n, e_start=0, e_count=E)
    wg, wu, wd = identity_like_experts(E, n)
    r = oracle_mod.route(sh, logits)
    out = oracle_mod.forward(sh, x, wg, wu, wd, r, round_bf16=False, stages=True)
    # every permuted row carries its token's input (dispatch is a pure permutation)
    assert np.allclose(out["o"], x[r["perm"][:T * k] // k], rtol=0, atol=1e-13)
    # combine with gates summing to one undoes it
    assert np.allclose(out["y"], x, rtol=0, atol=2e-7)


def test_rounding_rule_matches_library_cast(oracle_mod):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000) * np.exp(rng.uniform(-30, 30, 4000)),
        # exact ties at 8 significant bits: 1 + (2m+1) * 2^-8
        1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8,
        -(1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8) * 2.0 ** 5,
        [0.0, 1.0, -1.0, 255.0, 256.0, 257.0, 2.0 ** -130, 3.3e38],
    ]).astype(np.float32).astype(np.float64)      # float32-exact, so torch rounds once
    want = torch.from_numpy(vals.astype(np.float32)).to(torch.bfloat16).double().numpy()
    for acc in ("f64", "f32"):
        got = oracle_mod.round_bf16(vals, acc=acc)
        assert np.array_equal(got, want), acc
    # a double that float32 would first round onto a tie must still round once
    v = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40])   # just above the tie -> rounds up
    assert oracle_mod.round_bf16(v)[0] == 1.0 + 2.0 ** -7


def _is_bf16(a):
    f = a.astype(np.float32)
    return np.array_equal(f.astype(np.float64), a) and \
        ((f.view(np.uint32) & 0xFFFF) == 0).all()


@pytest.mark.parametrize("acc", ["f64", "f32"])
def test_rounded_mode_is_bf16_valued_and_close(oracle_mod, acc):
    cfg = moe_synth.small_config(T=64, d=64, E=8, k=2, I=96)
    inp = moe_synth.make_inputs(cfg, seed=5)
    bits = {key: oracle_mod.bf16_bits(inp[key] * (8 if key.startswith("w_") else 1))
            for key in ("x", "w_gate", "w_up", "w_down")}
    r = oracle_mod.route(cfg.shape_dict(), inp["logits"].numpy(), acc=acc)
    rounded = oracle_mod.forward(cfg.shape_dict(), bits["x"], bits["w_gate"], bits["w_up"],
                                 bits["w_down"], r, round_bf16=True, acc=acc, stages=True)
    exact = oracle_mod.forward(cfg.shape_dict(), bits["x"], bits["w_gate"], bits["w_up"],
                               bits["w_down"], r, round_bf16=False, acc="f64", stages=True)
    for key in ("h", "o", "y"):
        assert _is_bf16(rounded[key]), key
        err = np.linalg.norm(rounded[key] - exact[key]) / np.linalg.norm(exact[key])
        assert err < 6e-3, (key, err)
    # h is exactly the one-rounding image of silu(G)*U computed from the unrounded G, U
    G, U = rounded["G"], rounded["U"]
    if acc == "f64":
        hh = G * (1.0 / (1.0 + np.exp(-G))) * U
        assert np.array_equal(rounded["h"], oracle_mod.round_bf16(hh))


def test_f32_and_f64_accumulate_agree_to_float_noise(oracle_mod):
    cfg = moe_synth.small_config(T=40, d=256, E=4, k=2, I=128)
    inp = moe_synth.make_inputs(cfg, seed=9)
    b = {key: oracle_mod.bf16_bits(inp[key]) for key in ("x", "w_gate", "w_up", "w_down")}
    r = oracle_mod.route(cfg.shape_dict(), inp["logits"].numpy())
    y64 = oracle_mod.forward(cfg.shape_dict(), b["x"], b["w_gate"], b["w_up"], b["w_down"], r,
                             round_bf16=False, acc="f64")["y"]
    y32 = oracle_mod.forward(cfg.shape_dict(), b["x"], b["w_gate"], b["w_up"], b["w_down"], r,
                             round_bf16=False, acc="f32")["y"]
    assert np.linalg.norm(y32 - y64) / np.linalg.norm(y64) < 1e-5


def test_token_sampled_entry_equals_whole_layer(oracle_mod):
    cfg = moe_synth.small_config(T=50, d=32, E=16, k=4, I=48, e_start=4, e_count=8)
    inp = moe_synth.make_inputs(cfg, seed=2)
    b = {key: oracle_mod.bf16_bits(inp[key]) for key in ("x", "w_gate", "w_up", "w_down")}
    r = oracle_mod.route(cfg.shape_dict(), inp["logits"].numpy())
    full = oracle_mod.forward(cfg.shape_dict(), b["x"], b["w_gate"], b["w_up"], b["w_down"], r,
                              stages=True)
    toks = np.array([0, 7, 49, 13, 13], np.int32)
    part = oracle_mod.forward_tokens(cfg.shape_dict(), b["x"], b["w_gate"], b["w_up"],
                                     b["w_down"], r, toks, with_o=True)
    assert np.array_equal(part["y"], full["y"][toks])
    for i, t in enumerate(toks):
        for j in range(cfg.k):
            row = r["inv_perm"][t, j]
            if row >= 0:
                assert np.array_equal(part["o"][i, j], full["o"][row])
            else:
                assert (part["o"][i, j] == 0).all()
