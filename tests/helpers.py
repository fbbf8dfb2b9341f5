"""Shared helpers of the GPU parity tests (no arithmetic of the method here)."""
import sys

import numpy as np
import torch

import moe_synth
import oracle


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rel_l2(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / (den if den > 0 else 1.0))


def max_abs(got, want):
    return float(np.abs(np.asarray(got, np.float64) - np.asarray(want, np.float64)).max()) \
        if np.size(got) else 0.0


def max_abs_beyond_ulp(got, want):
    """Largest |got - want| after allowing one bf16 unit in the last place of the reference
    element (2^-7 |want| bounds it): both sides are bf16 values, so wherever the output exceeds
    ~2.5 in magnitude the smallest possible disagreement already exceeds an absolute 2e-2."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if got.size == 0:
        return 0.0
    return float(np.maximum(np.abs(got - want) - 2.0 ** -7 * np.abs(want), 0.0).max())


def to_f64(t):
    return t.detach().float().cpu().double().numpy()


def bits(inp, keys):
    return {key: oracle.bf16_bits(inp[key]) for key in keys}


def oracle_routing_to_np(r):
    return {key: np.asarray(v) for key, v in r.items()}


def gpu_routing_as_np(r):
    return {key: getattr(r, key).cpu().numpy() for key in
            ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm")}


def scaled_inputs(cfg, seed, wscale=1.0):
    """Synthetic inputs; wscale multiplies the N(0,0.02^2) weights (exactly, power of two)."""
    inp = moe_synth.make_inputs(cfg, seed=seed, with_dy=True)
    if wscale != 1.0:
        for key in ("w_gate", "w_up", "w_down"):
            inp[key] = (inp[key].float() * wscale).to(torch.bfloat16)
    return inp
