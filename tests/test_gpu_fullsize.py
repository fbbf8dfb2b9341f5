"""Full-size parity at the benchmark's configurations, in the launch
configuration bench.py times (default options: persistent MegaKernels).

The oracle cannot run these sizes whole in seconds, so it computes sampled
outputs one by one (token rows of y and dX, dtopk_w rows, whole weight-gradient
matrices of sampled experts); properties that hold at any size cover the rest
(bit-exact routing, exact zeros, bitwise repeatability)."""
import numpy as np
import pytest
import torch

import moe_synth
import oracle
from helpers import gpu_routing_as_np, max_abs, max_abs_beyond_ulp, rel_l2, say, to_f64

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, GRAD_REL_L2 = 2e-2, 5e-3, 1e-2


def run_gpu(cfg, inp, backward):
    import paper_2604_19241_amd as moe
    shape = moe.make_shape(**cfg.shape_dict())
    sizes = moe.moe_workspace_bytes(shape)
    dev = {k: v.cuda() for k, v in inp.items()}
    routing = moe.moe_route(shape, dev["logits"])
    saved = moe.alloc_saved(shape, "cuda") if backward else None
    ws = torch.empty(sizes["fwd"], dtype=torch.uint8, device="cuda")
    y = moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"], routing,
                              saved=saved, ws=ws)
    assert moe.moe_device_status(ws) == 0
    grads = None
    if backward:
        wsb = torch.empty(sizes["bwd"], dtype=torch.uint8, device="cuda")
        grads = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"],
                                       dev["w_down"], routing, saved, ws=wsb)
        assert moe.moe_device_status(wsb) == 0
    torch.cuda.synchronize()
    return y, routing, grads, dev


def sample_tokens(cfg, r, n, rng):
    """Random tokens plus, when the share is partial, tokens with and without local slots."""
    toks = set(int(t) for t in rng.integers(0, cfg.T, n))
    local = (r["inv_perm"] >= 0).sum(1)
    for want in (0, local.max()):
        idx = np.nonzero(local == want)[0]
        if idx.size:
            toks.add(int(idx[0]))
    return np.array(sorted(toks), np.int32)


@pytest.mark.parametrize("cid", [2, 1, 3, 4])
def test_fullsize_sampled_parity(cid):
    cfg = moe_synth.CONFIGS[cid]
    say(f"[full] config {cid} {cfg.name}: generating inputs")
    inp = moe_synth.make_inputs(cfg)
    logits = inp["logits"].numpy()
    r = oracle.route(cfg.shape_dict(), logits)
    say(f"[full] config {cid}: GPU route + forward{' + backward' if cfg.backward else ''}")
    y, routing, grads, dev = run_gpu(cfg, inp, cfg.backward)
    g = gpu_routing_as_np(routing)
    for key in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(g[key], r[key]), key
    say(f"[full] config {cid}: load {moe_synth.histogram_summary(r['counts'])}")

    rng = np.random.default_rng(100 + cid)
    keys = ("x", "w_gate", "w_up", "w_down") + (("dy",) if cfg.backward else ())
    b = {k: oracle.bf16_bits(inp[k]) for k in keys}
    toks = sample_tokens(cfg, r, 24, rng)
    say(f"[full] config {cid}: oracle forward on {len(toks)} sampled tokens")
    want = oracle.forward_tokens(cfg.shape_dict(), b["x"], b["w_gate"], b["w_up"], b["w_down"], r,
                                 toks)["y"]
    got = to_f64(y[torch.from_numpy(toks).long().cuda()])
    e_abs, e_rel, e_ulp = max_abs(got, want), rel_l2(got, want), max_abs_beyond_ulp(got, want)
    say(f"   y: max_abs={e_abs:.3e} (beyond one bf16 ulp: {e_ulp:.3e}) rel_l2={e_rel:.3e} "
        f"max|y|={np.abs(want).max():.2f}")
    assert e_ulp <= MAX_ABS and e_rel <= REL_L2
    # tokens without a local slot give exact zeros
    none_local = np.nonzero((r["inv_perm"] >= 0).sum(1) == 0)[0]
    if none_local.size:
        assert (y[torch.from_numpy(none_local[:64]).long().cuda()] == 0).all()

    if not cfg.backward:
        return
    say(f"[full] config {cid}: oracle backward on {len(toks)} sampled tokens")
    wb = oracle.backward_tokens(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"],
                                b["w_down"], r, toks)
    idx = torch.from_numpy(toks).long().cuda()
    e_dx = rel_l2(to_f64(grads["dx"][idx]), wb["dx"])
    e_dw = rel_l2(to_f64(grads["dtopk_w"][idx]), wb["dtopk_w"])
    say(f"   dx rel_l2={e_dx:.3e}  dtopk_w rel_l2={e_dw:.3e}")
    assert e_dx <= GRAD_REL_L2 and e_dw <= GRAD_REL_L2
    # whole weight-gradient matrices of sampled experts: a median-sized one, the
    # smallest non-empty one, and (if any) an empty one
    counts = r["counts"]
    order = np.argsort(counts)
    nonempty = order[counts[order] > 0]
    picks = [int(nonempty[len(nonempty) // 2]), int(nonempty[0])]
    if (counts == 0).any():
        picks.append(int(np.nonzero(counts == 0)[0][0]))
    picks = sorted(set(picks))
    say(f"[full] config {cid}: oracle weight gradients of experts {picks} (rows {counts[picks].tolist()})")
    we = oracle.backward_experts(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"],
                                 b["w_down"], r, np.array(picks, np.int32))
    for i, e in enumerate(picks):
        for key in ("dw_gate", "dw_up", "dw_down"):
            gg = to_f64(grads[key][e])
            if counts[e] == 0:
                assert (gg == 0).all(), (key, e)
            else:
                err = rel_l2(gg, we[key][i])
                say(f"   expert {e} {key} rel_l2={err:.3e}")
                assert err <= GRAD_REL_L2, (key, e, err)


@pytest.mark.parametrize("cid", [2, 4])
def test_fullsize_bitwise_repeatable(cid):
    """10 runs, bitwise identical outputs and gradients (the paper's max_diff = 0, %non-bw = 0
    criterion, applied run to run on the skewed and the balanced workload)."""
    cfg = moe_synth.CONFIGS[cid]
    say(f"[full] determinism config {cid}")
    inp = moe_synth.make_inputs(cfg)
    y0, _, g0, _ = run_gpu(cfg, inp, True)
    ref = {"y": y0.clone(), **{k: v.clone() for k, v in g0.items()}}
    for i in range(9):
        y, _, g, _ = run_gpu(cfg, inp, True)
        assert torch.equal(ref["y"], y), i
        for key, v in g.items():
            assert torch.equal(ref[key], v), (key, i)
