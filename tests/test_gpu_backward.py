"""GPU parity of moe_fused_backward against the oracle: dX, dW_gate, dW_up,
dW_down, dtopk_w element by element on sizes with several tiles and ragged
tails, both schedules and tile heights; exact zeros for idle experts; bitwise
repeatability (the paper's max_diff = 0 criterion applied run to run)."""
import numpy as np
import pytest
import torch

import moe_synth
import oracle
from helpers import bits, check_elementwise, rel_l2, say, scaled_inputs, to_f64

pytestmark = pytest.mark.gpu

GRAD_REL_L2 = 1e-2   # the benchmark spec tolerance for gradients
KEYS = ("dx", "dw_gate", "dw_up", "dw_down")


def gpu_fwd_bwd(cfg, inp, schedule, tile_rows, workers=0, want_dtopk_w=True, split=0):
    import paper_2604_19241_amd as moe
    shape = moe.make_shape(**cfg.shape_dict())
    dev = {key: v.cuda() for key, v in inp.items()}
    routing = moe.moe_route(shape, dev["logits"])
    saved = moe.alloc_saved(shape, "cuda")
    sizes = moe.moe_workspace_bytes(shape)
    ws = torch.empty(sizes["fwd"], dtype=torch.uint8, device="cuda")
    opts = moe.make_opts(schedule=schedule, tile_rows=tile_rows, workers=workers,
                         spin_limit_ms=500, dw_split_rows=split)
    wsb = torch.empty(moe.moe_backward_workspace_bytes(shape, opts), dtype=torch.uint8, device="cuda")
    assert split or wsb.numel() == sizes["bwd"]
    moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"], routing,
                          saved=saved, ws=ws, opts=opts)
    g = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"],
                               dev["w_down"], routing, saved, want_dtopk_w=want_dtopk_w, ws=wsb,
                               opts=opts)
    assert moe.moe_device_status(ws) == 0
    assert moe.moe_device_status(wsb) == 0
    return g, routing


def check_backward(cfg, seed, schedule, tile_rows, wscale):
    say(f"[bwd] {cfg.shape_dict()} schedule={schedule} tile_rows={tile_rows} wscale={wscale}")
    inp = scaled_inputs(cfg, seed, wscale)
    b = bits(inp, ("x", "dy", "w_gate", "w_up", "w_down"))
    r = oracle.route(cfg.shape_dict(), inp["logits"].numpy())
    g, _ = gpu_fwd_bwd(cfg, inp, schedule, tile_rows)
    for acc in ("f64", "f32"):
        want = oracle.backward(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"],
                               b["w_down"], r, round_bf16=True, acc=acc)
        errs = {key: rel_l2(to_f64(g[key]), want[key]) for key in KEYS}
        errs["dtopk_w"] = rel_l2(to_f64(g["dtopk_w"]), want["dtopk_w"])
        say(f"   vs oracle[{acc}]: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
        for key, v in errs.items():
            assert v <= GRAD_REL_L2, (key, v)
        for key in KEYS:
            check_elementwise(key, to_f64(g[key]), want[key])
        check_elementwise("dtopk_w", to_f64(g["dtopk_w"]), want["dtopk_w"], whole_array_rms=True)
        # idle experts: exact zeros
        for e in np.nonzero(r["counts"] == 0)[0]:
            for key in ("dw_gate", "dw_up", "dw_down"):
                assert (g[key][int(e)] == 0).all(), (key, e)
    return g


SMALL = [
    dict(T=700, d=320, E=4, k=2, I=320),
    dict(T=256, d=512, E=8, k=2, I=1024),
    dict(T=300, d=256, E=16, k=4, I=192, e_start=4, e_count=8),
    dict(T=97, d=128, E=32, k=8, I=64),
]


@pytest.mark.parametrize("kw", SMALL)
@pytest.mark.parametrize("schedule", [2, 1, 3])
@pytest.mark.parametrize("tile_rows", [128, 256])
def test_backward_matches_oracle(kw, schedule, tile_rows):
    cfg = moe_synth.small_config(**kw)
    check_backward(cfg, seed=13, schedule=schedule, tile_rows=tile_rows, wscale=4.0)


def test_backward_config0_default_options():
    check_backward(moe_synth.CONFIGS[0], seed=None, schedule=0, tile_rows=0, wscale=1.0)


def test_backward_idle_experts_and_skew():
    cfg = moe_synth.small_config(T=500, d=128, E=16, k=2, I=128, zipf_s=3.0)
    inp = scaled_inputs(cfg, 5, 4.0)
    r = oracle.route(cfg.shape_dict(), inp["logits"].numpy())
    assert (r["counts"] == 0).any() and r["counts"].max() > 300
    check_backward(cfg, seed=5, schedule=1, tile_rows=0, wscale=4.0)


@pytest.mark.parametrize("tile_rows", [128, 256])
def test_backward_long_reduction(tile_rows):
    """One expert with well over a thousand rows: the weight-gradient tiles reduce over many more
    K stages than their index ring holds (its slots are reused and the clamped tail stages run),
    compared element by element."""
    cfg = moe_synth.small_config(T=1600, d=256, E=2, k=1, I=192)
    inp = scaled_inputs(cfg, 41, 4.0)
    inp["logits"][:, 0] += 0.9      # nearly every token picks expert 0
    r = oracle.route(cfg.shape_dict(), inp["logits"].numpy())
    assert r["counts"].max() >= 1500 and r["counts"].min() >= 1
    say(f"[bwd] long reduction: rows per expert {r['counts'].tolist()}")
    b = bits(inp, ("x", "dy", "w_gate", "w_up", "w_down"))
    g, _ = gpu_fwd_bwd(cfg, inp, 0, tile_rows)
    want = oracle.backward(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r,
                           round_bf16=True, acc="f32")
    for key in KEYS:
        err = rel_l2(to_f64(g[key]), want[key])
        say(f"   {key} rel_l2={err:.2e}")
        assert err <= GRAD_REL_L2, (key, err)
        check_elementwise(key, to_f64(g[key]), want[key])


def test_backward_is_bitwise_repeatable_and_schedule_independent():
    cfg = moe_synth.small_config(T=900, d=256, E=16, k=4, I=256, zipf_s=1.2)
    inp = scaled_inputs(cfg, 22, 4.0)
    say("[bwd] determinism 10 runs, persistent")
    ref, _ = gpu_fwd_bwd(cfg, inp, 1, 0)
    ref = {k: v.clone() for k, v in ref.items()}
    for i in range(9):
        again, _ = gpu_fwd_bwd(cfg, inp, 1, 0)
        for key in ref:
            assert torch.equal(ref[key], again[key]), (key, i + 1)
    say("[bwd] determinism across schedules, worker counts and tile heights")
    for schedule, workers, tile_rows in ((2, 0, 0), (0, 0, 0), (3, 3, 0), (1, 5, 0), (1, 64, 0), (1, 0, 128), (1, 0, 256)):
        other, _ = gpu_fwd_bwd(cfg, inp, schedule, tile_rows, workers=workers)
        for key in ref:
            assert torch.equal(ref[key], other[key]), (key, schedule, workers, tile_rows)


def test_backward_without_dtopk_w():
    cfg = moe_synth.small_config(T=200, d=128, E=8, k=2, I=128)
    inp = scaled_inputs(cfg, 9, 4.0)
    g1, _ = gpu_fwd_bwd(cfg, inp, 1, 0, want_dtopk_w=True)
    g2, _ = gpu_fwd_bwd(cfg, inp, 1, 0, want_dtopk_w=False)
    assert g2["dtopk_w"] is None
    for key in KEYS:
        assert torch.equal(g1[key], g2[key])


@pytest.mark.parametrize("tile_rows", [0, 256])
def test_forward_backward_maximum_experts_and_topk(tile_rows):
    """The shape limits at once: E = 1024 experts, k = 16 slots, most experts empty or with a
    handful of rows; exercises the 1024-expert scan, sort and list planning of the prologues."""
    cfg = moe_synth.small_config(T=130, d=128, E=1024, k=16, I=64)
    check_backward(cfg, seed=21, schedule=1, tile_rows=tile_rows, wscale=4.0)


def test_forward_backward_empty_batch():
    """T = 0: nothing to route; y and dX are empty, every weight gradient is exactly zero."""
    import paper_2604_19241_amd as moe
    cfg = moe_synth.small_config(T=0, d=128, E=8, k=2, I=64)
    shape = moe.make_shape(**cfg.shape_dict())
    dev = {
        "logits": torch.empty((0, cfg.E), dtype=torch.float32, device="cuda"),
        "x": torch.empty((0, cfg.d), dtype=torch.bfloat16, device="cuda"),
        "dy": torch.empty((0, cfg.d), dtype=torch.bfloat16, device="cuda"),
        "w_gate": torch.randn((cfg.E, cfg.d, cfg.I), device="cuda").bfloat16(),
        "w_up": torch.randn((cfg.E, cfg.d, cfg.I), device="cuda").bfloat16(),
        "w_down": torch.randn((cfg.E, cfg.I, cfg.d), device="cuda").bfloat16(),
    }
    routing = moe.moe_route(shape, dev["logits"])
    assert int(routing.offsets[-1]) == 0 and int(routing.counts.sum()) == 0
    saved = moe.alloc_saved(shape, "cuda")
    sizes = moe.moe_workspace_bytes(shape)
    ws = torch.empty(sizes["fwd"], dtype=torch.uint8, device="cuda")
    wsb = torch.empty(sizes["bwd"], dtype=torch.uint8, device="cuda")
    y = moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"], routing,
                              saved=saved, ws=ws)
    g = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"],
                               dev["w_down"], routing, saved, ws=wsb)
    assert moe.moe_device_status(ws) == 0 and moe.moe_device_status(wsb) == 0
    assert y.shape == (0, cfg.d) and g["dx"].shape == (0, cfg.d)
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert (g[key] == 0).all(), key


@pytest.mark.parametrize("schedule,tile_rows", [(0, 0), (1, 0), (2, 0), (0, 128)])
def test_backward_accumulates_weight_gradients_in_fp32(schedule, tile_rows):
    """opts.dw_accumulate: the fp32 accumulators are added to the caller's fp32 buffers.  Onto
    zeros the result rounds to exactly the bf16 gradients of the plain call; a second call
    doubles it exactly; onto a non-zero buffer it is the fp32 sum, element for element; experts
    without rows are not touched (a -0.0 stays -0.0); dX and dtopk_w do not change."""
    import paper_2604_19241_amd as moe
    cfg = moe_synth.small_config(T=1100, d=320, E=12, k=3, I=448, e_start=2, e_count=9)
    inp = scaled_inputs(cfg, 31, 4.0)
    inp["logits"][:, 5] = -30.0   # a local expert that no token selects
    say(f"[bwd accumulate] {cfg.shape_dict()} schedule={schedule} tile_rows={tile_rows}")
    plain, routing = gpu_fwd_bwd(cfg, inp, schedule, tile_rows)
    counts = routing.counts.cpu().numpy()
    assert (counts == 0).any() and (counts > 256).any()
    shape = moe.make_shape(**cfg.shape_dict())
    dev = {key: v.cuda() for key, v in inp.items()}
    saved = moe.alloc_saved(shape, "cuda")
    moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"], routing, saved=saved)
    opts = moe.make_opts(schedule=schedule, tile_rows=tile_rows, spin_limit_ms=500, dw_accumulate=1)
    wkeys = ("dw_gate", "dw_up", "dw_down")

    def run(main):
        out = {"dx": torch.empty_like(dev["x"]), "dtopk_w": torch.empty((shape.T, shape.k), dtype=torch.float32, device="cuda")}
        out.update(main)
        return moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"],
                                      routing, saved, opts=opts, out=out)

    zeros = {key: torch.zeros_like(dev["w_" + key[3:]], dtype=torch.float32) for key in wkeys}
    once = run(zeros)
    first = {key: once[key].clone() for key in wkeys}
    for key in wkeys:
        assert torch.equal(first[key].to(torch.bfloat16), plain[key]), key
    assert torch.equal(once["dx"], plain["dx"]) and torch.equal(once["dtopk_w"], plain["dtopk_w"])
    twice = run(once)     # the same buffers again
    for key in wkeys:
        assert torch.equal(twice[key], 2.0 * first[key]), key
    gen = torch.Generator(device="cuda").manual_seed(77)
    main = {key: torch.randn(first[key].shape, generator=gen, device="cuda", dtype=torch.float32) for key in wkeys}
    idle = [int(e) for e in np.nonzero(counts == 0)[0]]
    for key in wkeys:
        for e in idle:
            main[key][e].fill_(-0.0)
    want = {key: main[key] + first[key] for key in wkeys}
    got = run({key: main[key].clone() for key in wkeys})
    for key in wkeys:
        busy = [e for e in range(cfg.e_count) if e not in idle]
        assert torch.equal(got[key][busy], want[key][busy]), key
        for e in idle:
            assert torch.equal(got[key][e].view(torch.int32), main[key][e].view(torch.int32)), (key, e)


@pytest.mark.parametrize("split", [256, 512])
def test_backward_split_weight_gradient_reduction(split):
    """opts.dw_split_rows: the weight-gradient reduction of an expert with more rows than that is
    cut at fixed points and its partial tiles are added in part order.  Experts at or below the
    threshold, dX and dtopk_w are bitwise what the unsplit call gives; the split experts agree with
    the oracle to the same element-wise bounds; the result is bitwise the same from run to run,
    across schedules, worker counts and tile heights; a threshold no expert exceeds changes nothing;
    the fp32-accumulate form rounds to the same bf16 values."""
    import paper_2604_19241_amd as moe
    cfg = moe_synth.small_config(T=1500, d=320, E=6, k=2, I=320)
    inp = scaled_inputs(cfg, 51, 4.0)
    inp["logits"][:, 2] += 2.0      # one expert takes nearly every token, a second one about a third
    inp["logits"][:, 4] += 0.6
    inp["logits"][:, 5] = -30.0     # and one takes none
    r = oracle.route(cfg.shape_dict(), inp["logits"].numpy())
    counts = r["counts"]
    say(f"[bwd split {split}] rows per expert {counts.tolist()}")
    assert counts.max() > 2 * split and (counts == 0).any() and ((counts > 0) & (counts <= split)).any()
    plain, _ = gpu_fwd_bwd(cfg, inp, 0, 0)
    got, _ = gpu_fwd_bwd(cfg, inp, 0, 0, split=split)
    assert torch.equal(got["dx"], plain["dx"]) and torch.equal(got["dtopk_w"], plain["dtopk_w"])
    small = [int(e) for e in np.nonzero(counts <= split)[0]]
    big = [int(e) for e in np.nonzero(counts > split)[0]]
    b = bits(inp, ("x", "dy", "w_gate", "w_up", "w_down"))
    want = oracle.backward(cfg.shape_dict(), b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r,
                           round_bf16=True, acc="f32")
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert torch.equal(got[key][small], plain[key][small]), key
        err = rel_l2(to_f64(got[key]), want[key])
        differ = float((got[key][big] != plain[key][big]).float().mean())
        say(f"   {key} rel_l2={err:.2e}; elements of the split experts that differ from the unsplit sum: {differ:.3f}")
        assert err <= GRAD_REL_L2, (key, err)
        check_elementwise(key, to_f64(got[key]), want[key])
    ref = {k: v.clone() for k, v in got.items()}
    for schedule, workers, tile_rows in ((0, 0, 0), (2, 0, 0), (1, 0, 0), (3, 3, 0), (1, 64, 0), (0, 0, 128)):
        other, _ = gpu_fwd_bwd(cfg, inp, schedule, tile_rows, workers=workers, split=split)
        for key in ref:
            assert torch.equal(ref[key], other[key]), (key, schedule, workers, tile_rows)
    same, _ = gpu_fwd_bwd(cfg, inp, 0, 0, split=4096)   # no expert has that many rows
    for key in ref:
        assert torch.equal(same[key], plain[key]), key
    # added to fp32 buffers
    shape = moe.make_shape(**cfg.shape_dict())
    dev = {key: v.cuda() for key, v in inp.items()}
    routing = moe.moe_route(shape, dev["logits"])
    saved = moe.alloc_saved(shape, "cuda")
    moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"], routing, saved=saved)
    opts = moe.make_opts(spin_limit_ms=500, dw_accumulate=1, dw_split_rows=split)
    out = {"dx": torch.empty_like(dev["x"]), "dtopk_w": None}
    out.update({key: torch.zeros_like(dev["w_" + key[3:]], dtype=torch.float32) for key in ("dw_gate", "dw_up", "dw_down")})
    acc = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"],
                                 routing, saved, opts=opts, out=out, want_dtopk_w=False)
    for key in ("dw_gate", "dw_up", "dw_down"):
        assert torch.equal(acc[key].to(torch.bfloat16), ref[key]), key
