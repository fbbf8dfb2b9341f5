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


def max_abs_beyond_ulp(got, want, only_below=None):
    """Largest |got - want| after allowing one bf16 unit in the last place of the reference
    element (2^-7 |want| bounds it): both sides are bf16 values, so wherever the output exceeds
    ~2.5 in magnitude the smallest possible disagreement already exceeds an absolute 2e-2.
    only_below: restrict to elements with |want| <= only_below (the absolute bound is stated for
    outputs of magnitude O(1); elements beyond it are held to the element-wise relative bound)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if got.size == 0:
        return 0.0
    ex = np.maximum(np.abs(got - want) - 2.0 ** -7 * np.abs(want), 0.0)
    if only_below is not None:
        ex = np.where(np.abs(want) <= only_below, ex, 0.0)
    return float(ex.max())


def bf16_ulp(v):
    """Spacing of bf16 numbers at |v| (8 significant bits): 2^(floor(log2|v|) - 7); 0 at v = 0."""
    a = np.abs(np.asarray(v, np.float64))
    out = np.zeros_like(a)
    nz = a > 0
    out[nz] = np.exp2(np.floor(np.log2(a[nz])) - 7.0)
    return out


# Element-wise bound of every GPU-against-oracle comparison:
#     |got - want| <= C_ULP * ulp_bf16(want) + c_rms * 2^-8 * max(rms(row of want), |want|)
# Both sides round the same fp32 sum (different summation order, ~1e-6 relative apart) to bf16, so
# an element can differ by one bf16 step where the two sums straddle a rounding boundary: C_ULP = 1,
# and nothing else for values computed from exact inputs (G, U, h: measured excess 0).
# The second term covers what the element inherits from the bf16 values it was computed FROM:
#  - one-step flips of those inputs (h for o; o for y; dO, gate * h, dG|dU for the gradients): a
#    flipped input moves a sum over n terms by about 2^-8 rms(row) / sqrt(n), and a few percent
#    of the inputs flip; y adds k rows of o weighted by the gates (sum 1) and can inherit a whole
#    ulp of an o element that is larger than y itself;
#  - for everything behind the SwiGLU backward (dX, dW_gate, dW_up, dtopk_w), the bf16 rounding
#    of the stashed G and U, which the oracle does not have (it differentiates with unrounded
#    G, U): a relative 2^-9 on G and on U moves every element of dG|dU by a relative 2^-8 or so,
#    i.e. noise with a standard deviation of about 4e-3 of the element's scale on every output
#    element, whose maximum over 10^6..10^8 elements is 5-6 standard deviations; where an expert
#    has only a handful of rows the sum is as noisy as its largest term, which is why the scale
#    is the larger of the row's rms and the element itself.
# c_rms per quantity = about twice the largest excess measured over all parity cases (small cases
# with weights scaled by 4, the model shapes, the full-size configurations; measured with the row
# rms alone as the scale: o 0.92, y 5.2, dW_down 5.3 (gate folded into h), dX 7.6, dW_gate 12.8, dW_up 14.4 and 24 on a
# two-row expert, dtopk_w 9.6).  A wrong tile row or a misplaced 16-byte piece is off by about
# rms(row) itself, a ratio of 256.
C_ULP = 1.0
C_RMS = {"G": 0.25, "U": 0.25, "h": 0.25, "o": 2.0, "y": 8.0, "dw_down": 8.0,
         "dx": 16.0, "dw_gate": 24.0, "dw_up": 24.0, "dtopk_w": 16.0}


def elementwise_ratio(got, want, axis=-1):
    """max over elements of (|got - want| - C_ULP * ulp_bf16(want)) / (2^-8 * max(rms(row), |want|)),
    rows along `axis`; a row of zeros in `want` must be reproduced exactly."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if got.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(want * want, axis=axis, keepdims=True))
    excess = np.maximum(np.abs(got - want) - C_ULP * bf16_ulp(want), 0.0)
    scale = np.maximum(np.where(rms > 0, rms, 1e-300), np.abs(want))
    return float((excess / (2.0 ** -8 * scale)).max())


def check_elementwise(name, got, want, key=None, axis=-1, whole_array_rms=False):
    """Asserts the element-wise bound for quantity `key` (default: name) and reports the measured ratio."""
    key = key or name
    if whole_array_rms:     # rows too short for an rms of their own (dtopk_w: k values per row)
        got = np.asarray(got, np.float64).reshape(1, -1)
        want = np.asarray(want, np.float64).reshape(1, -1)
    r = elementwise_ratio(got, want, axis=axis)
    say(f"   {name}: element-wise excess over one bf16 ulp = {r:.3f} x 2^-8 max(rms(row), |want|)  (bound {C_RMS[key]})")
    assert r <= C_RMS[key], (name, r, C_RMS[key])
    return r


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
