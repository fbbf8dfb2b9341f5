"""Pins of the oracle's backward pass against things other than itself.

* torch.autograd (fp64) over the dense masked formulation of the layer;
* central finite differences of the oracle's own unrounded fp64 forward;
* an expert that received no token has exactly zero weight gradient;
* doubling dY doubles every gradient exactly (also with bf16 rounding on,
  since rounding commutes with a power-of-two scale);
* the sampled entry points equal the whole-layer result.
"""
import numpy as np
import pytest
import torch

import moe_synth


def f64_inputs(cfg, seed, wscale=20.0):
    inp = moe_synth.make_inputs(cfg, seed=seed, with_dy=True)
    a = {key: v.double().numpy() for key, v in inp.items() if key != "logits"}
    for key in ("w_gate", "w_up", "w_down"):
        a[key] = a[key] * wscale
    a["logits"] = inp["logits"].numpy()
    return a


def autograd_dense(a, routing, cfg):
    """Gradients of L = <y, dY> for the dense masked layer, with the gate values as a leaf."""
    T, E, k = cfg.T, cfg.E, cfg.k
    x = torch.tensor(a["x"], requires_grad=True)
    wg = torch.tensor(a["w_gate"], requires_grad=True)
    wu = torch.tensor(a["w_up"], requires_grad=True)
    wd = torch.tensor(a["w_down"], requires_grad=True)
    w = torch.tensor(routing["topk_w"].astype(np.float64), requires_grad=True)
    idx = torch.tensor(routing["topk_idx"].astype(np.int64))
    gate = torch.zeros(T, E, dtype=torch.float64).scatter(1, idx, w)
    y = torch.zeros(T, cfg.d, dtype=torch.float64)
    for el in range(cfg.e_count):
        h = torch.nn.functional.silu(x @ wg[el]) * (x @ wu[el])
        y = y + gate[:, cfg.e_start + el:cfg.e_start + el + 1] * (h @ wd[el])
    (y * torch.tensor(a["dy"])).sum().backward()
    return {"dx": x.grad.numpy(), "dw_gate": wg.grad.numpy(), "dw_up": wu.grad.numpy(),
            "dw_down": wd.grad.numpy(), "dtopk_w": w.grad.numpy()}


def close(got, want, rel):
    scale = max(np.abs(want).max(), 1e-30)
    return np.abs(got - want).max() <= rel * scale


@pytest.mark.parametrize("T,d,E,k,I,e_start,e_count", [
    (40, 24, 8, 2, 32, 0, 8), (36, 16, 16, 4, 24, 4, 8), (25, 8, 5, 5, 16, 0, 5),
    (30, 16, 8, 1, 8, 0, 8)])
def test_gradients_match_autograd_of_dense_layer(oracle_mod, T, d, E, k, I, e_start, e_count):
    cfg = moe_synth.small_config(T=T, d=d, E=E, k=k, I=I, e_start=e_start, e_count=e_count)
    a = f64_inputs(cfg, seed=100 + T)
    r = oracle_mod.route(cfg.shape_dict(), a["logits"])
    got = oracle_mod.backward(cfg.shape_dict(), a["x"], a["dy"], a["w_gate"], a["w_up"],
                              a["w_down"], r, round_bf16=False)
    want = autograd_dense(a, r, cfg)
    local = (r["inv_perm"] >= 0)
    for key in ("dx", "dw_gate", "dw_up", "dw_down"):
        assert close(got[key], want[key], 1e-11), key
    assert close(got["dtopk_w"][local], want["dtopk_w"][local], 1e-11)
    assert (got["dtopk_w"][~local] == 0).all()


def test_gradients_match_finite_differences(oracle_mod):
    cfg = moe_synth.small_config(T=7, d=6, E=4, k=2, I=5)
    a = f64_inputs(cfg, seed=42, wscale=25.0)
    sh = cfg.shape_dict()
    r = oracle_mod.route(sh, a["logits"])
    g = oracle_mod.backward(sh, a["x"], a["dy"], a["w_gate"], a["w_up"], a["w_down"], r,
                            round_bf16=False)

    def loss(x, wg, wu, wd):
        y = oracle_mod.forward(sh, x, wg, wu, wd, r, round_bf16=False)["y"]
        return float((y * a["dy"]).sum())

    rng = np.random.default_rng(1)
    eps = 1e-6
    names = ["x", "w_gate", "w_up", "w_down"]
    gkeys = ["dx", "dw_gate", "dw_up", "dw_down"]
    for which, (name, gkey) in enumerate(zip(names, gkeys)):
        arr = a[name]
        checked = 0
        for _ in range(200):
            pos = tuple(int(rng.integers(0, s)) for s in arr.shape)
            if name != "x" and r["counts"][pos[0]] == 0:
                continue
            args_p = [a[n].copy() for n in names]
            args_m = [a[n].copy() for n in names]
            args_p[which][pos] += eps
            args_m[which][pos] -= eps
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            an = g[gkey][pos]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 1e-7, (name, pos, fd, an)
            checked += 1
            if checked >= 25:
                break
        assert checked >= 10


@pytest.mark.parametrize("rounded", [False, True])
def test_empty_expert_has_zero_gradient_and_scaling_is_exact(oracle_mod, rounded):
    cfg = moe_synth.small_config(T=24, d=32, E=8, k=2, I=32)
    inp = moe_synth.make_inputs(cfg, seed=8, with_dy=True)
    logits = inp["logits"].numpy().copy()
    logits[:, 5] = -50.0                 # expert 5 is never chosen
    r = oracle_mod.route(cfg.shape_dict(), logits)
    assert r["counts"][5] == 0
    b = {key: oracle_mod.bf16_bits(inp[key]) for key in ("x", "dy", "w_gate", "w_up", "w_down")}
    g1 = oracle_mod.backward(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"],
                             b["w_down"], r, round_bf16=rounded)
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert (g1[key][5] == 0).all()
        assert np.abs(g1[key][0]).max() > 0
    dy2 = oracle_mod.bf16_bits(inp["dy"] * 2)
    g2 = oracle_mod.backward(cfg.shape_dict(), b["x"], dy2, b["w_gate"], b["w_up"], b["w_down"],
                             r, round_bf16=rounded)
    for key in g1:
        assert np.array_equal(g2[key], 2 * g1[key]), key


def _is_bf16(a):
    f = a.astype(np.float32)
    return np.array_equal(f.astype(np.float64), a) and ((f.view(np.uint32) & 0xFFFF) == 0).all()


@pytest.mark.parametrize("acc", ["f64", "f32"])
def test_rounded_backward_is_bf16_valued_and_close(oracle_mod, acc):
    cfg = moe_synth.small_config(T=48, d=64, E=8, k=2, I=64)
    inp = moe_synth.make_inputs(cfg, seed=12, with_dy=True)
    b = {key: oracle_mod.bf16_bits(inp[key] * (8 if key.startswith("w_") else 1))
         for key in ("x", "dy", "w_gate", "w_up", "w_down")}
    r = oracle_mod.route(cfg.shape_dict(), inp["logits"].numpy())
    args = (cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r)
    rounded = oracle_mod.backward(*args, round_bf16=True, acc=acc, stages=True)
    exact = oracle_mod.backward(*args, round_bf16=False, acc="f64", stages=True)
    for key in ("dx", "dw_gate", "dw_up", "dw_down", "dG", "dU", "dXp", "dO"):
        assert _is_bf16(rounded[key]), key
        err = np.linalg.norm(rounded[key] - exact[key]) / np.linalg.norm(exact[key])
        assert err < 8e-3, (key, err)
    err = np.linalg.norm(rounded["dtopk_w"] - exact["dtopk_w"]) / np.linalg.norm(exact["dtopk_w"])
    assert err < 8e-3


def test_sampled_entries_equal_whole_layer(oracle_mod):
    cfg = moe_synth.small_config(T=40, d=32, E=16, k=4, I=24, e_start=4, e_count=8)
    inp = moe_synth.make_inputs(cfg, seed=6, with_dy=True)
    b = {key: oracle_mod.bf16_bits(inp[key]) for key in ("x", "dy", "w_gate", "w_up", "w_down")}
    r = oracle_mod.route(cfg.shape_dict(), inp["logits"].numpy())
    args = (cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r)
    full = oracle_mod.backward(*args)
    ex = np.array([7, 0, 3], np.int32)
    pe = oracle_mod.backward_experts(*args, ex)
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert np.array_equal(pe[key], full[key][ex]), key
    toks = np.array([0, 39, 17, 5], np.int32)
    pt = oracle_mod.backward_tokens(*args, toks)
    assert np.array_equal(pt["dx"], full["dx"][toks])
    assert np.array_equal(pt["dtopk_w"], full["dtopk_w"][toks])
