"""GPU parity at the layer shapes of the paper's model table (Table "MoE Model
Configurations Evaluated"): the real H_dim, H_inter, N_exp and top-k of each
model, with fewer tokens and a window of local experts so that the oracle
finishes in seconds.  These shapes bring what the power-of-two configs do not:
H_inter = 1408, 896, 384 (ragged column tiles in GEMM1 and the weight-gradient
GEMMs), H_dim = 1280, 2304, top-k = 6 and 10, 512 experts."""
import numpy as np
import pytest
import torch

import moe_synth
import oracle
from helpers import bits, check_elementwise, gpu_routing_as_np, max_abs_beyond_ulp, rel_l2, say, to_f64
from test_gpu_backward import GRAD_REL_L2, KEYS, gpu_fwd_bwd
from test_gpu_forward import MAX_ABS, REL_L2

pytestmark = pytest.mark.gpu

# (model id, tokens, e_start, e_count, tile_rows); tile_rows 0 = the default 256-row tiles
CASES = [
    (1, 2048, 8, 8, 0),      # I = 1408: 5.5 column tiles of 256
    (2, 2048, 8, 16, 0),     # d = 1280, I = 896, k = 6
    (4, 8192, 40, 4, 0),     # d = 5120, 160 experts
    (7, 4096, 0, 4, 0),      # d = 4096, I = 1536
    (8, 1024, 158, 2, 0),    # d = 6144, I = 2560, the last two experts, ~50 rows each
    (8, 1024, 158, 2, 128),  # the same on 128-row tiles (4 waves)
    (9, 8192, 100, 16, 0),   # 512 experts, k = 10, I = 512
    (10, 4096, 96, 32, 0),   # I = 384
    (10, 1024, 0, 128, 0),   # every expert local, ~50 rows each
    (10, 1024, 0, 128, 128),
    (12, 8192, 32, 8, 0),    # d = 2304
]


@pytest.mark.parametrize("mid,tokens,e_start,e_count,tile_rows", CASES)
def test_model_shape_forward_backward(mid, tokens, e_start, e_count, tile_rows):
    cfg = moe_synth.model_config(mid, tokens=tokens, e_start=e_start, e_count=e_count)
    say(f"[model shape] {cfg.name} {cfg.shape_dict()} tile_rows={tile_rows}")
    inp = moe_synth.make_inputs(cfg, seed=100 + mid, with_dy=True)
    b = bits(inp, ("x", "dy", "w_gate", "w_up", "w_down"))
    sh = cfg.shape_dict()
    r = oracle.route(sh, inp["logits"].numpy())
    g, routing = gpu_fwd_bwd(cfg, inp, schedule=0, tile_rows=tile_rows)
    got = gpu_routing_as_np(routing)
    for key in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(got[key], r[key]), key
    say(f"   routed rows {int(r['offsets'][-1])}, rows per expert {r['counts'].min()}..{r['counts'].max()}")

    import paper_2604_19241_amd as moe
    shape = moe.make_shape(**sh)
    y = moe.moe_fused_forward(shape, inp["x"].cuda(), inp["w_gate"].cuda(), inp["w_up"].cuda(),
                              inp["w_down"].cuda(), routing, opts=moe.make_opts(tile_rows=tile_rows))
    want = oracle.forward(sh, b["x"], b["w_gate"], b["w_up"], b["w_down"], r, round_bf16=True,
                          acc="f32")
    yg = to_f64(y)
    e_ulp, e_rel = max_abs_beyond_ulp(yg, want["y"]), rel_l2(yg, want["y"])
    say(f"   y: max_abs beyond one bf16 ulp={e_ulp:.3e} rel_l2={e_rel:.3e}")
    assert e_ulp <= MAX_ABS and e_rel <= REL_L2
    check_elementwise("y", yg, want["y"])

    wantb = oracle.backward(sh, b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r,
                            round_bf16=True, acc="f32")
    errs = {key: rel_l2(to_f64(g[key]), wantb[key]) for key in KEYS}
    errs["dtopk_w"] = rel_l2(to_f64(g["dtopk_w"]), wantb["dtopk_w"])
    say("   grads: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for key, v in errs.items():
        assert v <= GRAD_REL_L2, (key, v)
    for key in KEYS:
        check_elementwise(key, to_f64(g[key]), wantb[key])
    check_elementwise("dtopk_w", to_f64(g["dtopk_w"]), wantb["dtopk_w"], whole_array_rms=True)
    for e in np.nonzero(r["counts"] == 0)[0]:
        for key in ("dw_gate", "dw_up", "dw_down"):
            assert (g[key][int(e)] == 0).all(), (key, e)
