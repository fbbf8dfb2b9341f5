"""Seeded synthetic inputs for the fused-MoE hot path.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no top-k, no permutation, no expert math).  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here, so
the two sides see bit-identical inputs.

Shapes follow the MoE layers the paper evaluates (Table "MoE Model
Configurations Evaluated": MoE-6 = Qwen3-30B-A3B, MoE-5 = DeepSeek-R1 shape)
plus a Mixtral-shaped and a tiny correctness config.  Value distributions:
x, dY ~ N(0,1); W_gate, W_up, W_down, W_r ~ N(0, 0.02^2); everything that the
layer consumes in bf16 is rounded to bf16 (round-to-nearest-even, by torch).
Router logits are the harness-side product float32(x) @ float32(W_r), summed in
fp64 and rounded once to fp32 (the paper leaves gating outside the measured
path, Section 6.4 "excluding gating"), so every consumer ranks the very same
fp32 numbers.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, asdict

import torch

BASE_SEED = 20260419


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int          # tokens held by this GPU
    d: int          # hidden size
    E: int          # experts the router ranks (global)
    k: int          # top-k
    I: int          # expert intermediate size
    e_start: int    # first local expert
    e_count: int    # number of local experts
    zipf_s: float = 0.0   # >0: bias router logits by -s*ln(rank) (skewed load)
    backward: bool = False

    def shape_dict(self):
        return {key: getattr(self, key) for key in ("T", "d", "E", "k", "I", "e_start", "e_count")}

    def asdict(self):
        return asdict(self)


CONFIGS = {
    0: MoEConfig("tiny", T=256, d=512, E=8, k=2, I=1024, e_start=0, e_count=8, backward=True),
    1: MoEConfig("mixtral-8x7b-shaped", T=4096, d=4096, E=8, k=2, I=14336, e_start=0, e_count=8),
    2: MoEConfig("qwen3-30b-a3b-shaped", T=8192, d=2048, E=128, k=8, I=768, e_start=0, e_count=128,
                 backward=True),
    3: MoEConfig("deepseek-v3-one-rank-share", T=8192, d=7168, E=256, k=8, I=2048, e_start=0,
                 e_count=32, backward=True),
    4: MoEConfig("qwen3-30b-a3b-zipf1.2", T=8192, d=2048, E=128, k=8, I=768, e_start=0, e_count=128,
                 zipf_s=1.2, backward=True),
}


# The twelve layer shapes of the paper's Table "MoE Model Configurations Evaluated":
# id -> (model name, H_dim, H_inter, N_exp, top-k).
MODEL_SHAPES = {
    1: ("DeepSeek-MoE-16B", 2048, 1408, 64, 6),
    2: ("DeepSeek-OCR-2", 1280, 896, 64, 6),
    3: ("DeepSeek-V2-Lite", 2048, 1408, 64, 6),
    4: ("DeepSeek-V2-Chat", 5120, 1536, 160, 6),
    5: ("DeepSeek-R1", 7168, 2048, 256, 8),
    6: ("Qwen3-30B-A3B", 2048, 768, 128, 8),
    7: ("Qwen3-235B-A22B", 4096, 1536, 128, 8),
    8: ("Qwen3-Coder-480B", 6144, 2560, 160, 8),
    9: ("Qwen3-Next-80B", 2048, 512, 512, 10),
    10: ("Qwen3-Omni-30B", 1024, 384, 128, 6),
    11: ("Kimi-K2", 7168, 2048, 384, 8),
    12: ("Kimi-Linear-48B", 2304, 1024, 256, 8),
}


def model_config(mid: int, tokens: int = 8192, ep: int = 1, e_start: int | None = None,
                 e_count: int | None = None) -> MoEConfig:
    """Layer shape MoE-<mid> of the paper's model table as a one-GPU workload.

    ep = 1: `tokens` tokens, every expert local.  ep = W > 1: one rank's share of W-way
    expert parallelism at `tokens` tokens per rank: the W*tokens tokens of all ranks are
    resident, the first N_exp/W experts are local, so about tokens*k rows are routed here
    (the paper's evaluation setting, Section 6.1, without the token exchange).
    e_start/e_count override the local expert range (smaller shares for parity tests)."""
    name, d, inter, n_exp, k = MODEL_SHAPES[mid]
    assert n_exp % ep == 0
    if e_count is None:
        e_count = n_exp // ep
    return MoEConfig(f"moe-{mid}-{name.lower()}" + (f"-ep{ep}" if ep > 1 else ""),
                     T=tokens * ep, d=d, E=n_exp, k=k, I=inter,
                     e_start=0 if e_start is None else e_start, e_count=e_count, backward=True)


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _normal_bf16(shape, std: float, g: torch.Generator) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 on the CPU, rounded to bf16 (RNE).

    Large tensors are drawn slab by slab along dim 0 to bound the fp32
    temporary; the stream of random numbers is the same either way because the
    slabs are consumed in order from one generator."""
    shape = tuple(shape)
    out = torch.empty(shape, dtype=torch.bfloat16)
    if len(shape) == 0 or out.numel() == 0:
        return out
    lead = shape[0]
    per = out.numel() // lead
    step = max(1, (1 << 26) // max(per, 1))
    for i in range(0, lead, step):
        j = min(lead, i + step)
        blk = torch.randn((j - i,) + shape[1:], generator=g, dtype=torch.float32)
        if std != 1.0:
            blk.mul_(std)
        out[i:j] = blk.to(torch.bfloat16)
    return out


def make_logits(x_bf16: torch.Tensor, w_r_bf16: torch.Tensor) -> torch.Tensor:
    """Router product done once by the harness: fp64 accumulate, one rounding to fp32."""
    return (x_bf16.double() @ w_r_bf16.double()).float().contiguous()


def zipf_bias(E: int, s: float, g: torch.Generator) -> torch.Tensor:
    """-s*ln(rank(e)) with rank a seeded random permutation of 1..E (fp32)."""
    rank = torch.randperm(E, generator=g).double() + 1.0
    return (-s * torch.log(rank)).float()


def make_inputs(cfg: MoEConfig, seed: int | None = None, with_dy: bool | None = None,
                with_weights: bool = True) -> dict:
    """All inputs of one MoE layer call, as CPU tensors.

    Keys: x [T,d] bf16, logits [T,E] f32, w_gate/w_up [e_count,d,I] bf16,
    w_down [e_count,I,d] bf16, dy [T,d] bf16 (if requested).  Only the local
    experts' weights are materialised (one rank's share)."""
    if seed is None:
        seed = BASE_SEED
    if with_dy is None:
        with_dy = cfg.backward
    g = _gen(seed)
    out = {}
    out["x"] = _normal_bf16((cfg.T, cfg.d), 1.0, g)
    w_r = _normal_bf16((cfg.d, cfg.E), 0.02, g)
    logits = make_logits(out["x"], w_r)
    if cfg.zipf_s > 0:
        logits = (logits + zipf_bias(cfg.E, cfg.zipf_s, g)[None, :]).contiguous()
    out["logits"] = logits
    if with_dy:
        out["dy"] = _normal_bf16((cfg.T, cfg.d), 1.0, g)
    if with_weights:
        out["w_gate"] = _normal_bf16((cfg.e_count, cfg.d, cfg.I), 0.02, g)
        out["w_up"] = _normal_bf16((cfg.e_count, cfg.d, cfg.I), 0.02, g)
        out["w_down"] = _normal_bf16((cfg.e_count, cfg.I, cfg.d), 0.02, g)
    return out


def make_inputs_device(cfg: MoEConfig, device, seed: int | None = None, with_dy: bool = True) -> dict:
    """The same tensors drawn directly on `device` (timing sweeps over large shapes, where
    drawing tens of GB on the host would take minutes).  Same distributions as make_inputs,
    a different random stream, logits as a plain fp32 product: parity tests never use these."""
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED if seed is None else seed)

    def normal(shape, std):
        out = torch.empty(shape, dtype=torch.bfloat16, device=device)
        lead = shape[0]
        step = max(1, (1 << 28) // max(out.numel() // max(lead, 1), 1))
        for i in range(0, lead, step):
            j = min(lead, i + step)
            out[i:j] = (torch.randn((j - i,) + tuple(shape[1:]), generator=g, device=device,
                                    dtype=torch.float32) * std).to(torch.bfloat16)
        return out

    out = {"x": normal((cfg.T, cfg.d), 1.0)}
    w_r = normal((cfg.d, cfg.E), 0.02)
    logits = out["x"].float() @ w_r.float()
    if cfg.zipf_s > 0:
        logits = logits + zipf_bias(cfg.E, cfg.zipf_s, _gen(BASE_SEED))[None, :].to(device)
    out["logits"] = logits.contiguous()
    if with_dy:
        out["dy"] = normal((cfg.T, cfg.d), 1.0)
    out["w_gate"] = normal((cfg.e_count, cfg.d, cfg.I), 0.02)
    out["w_up"] = normal((cfg.e_count, cfg.d, cfg.I), 0.02)
    out["w_down"] = normal((cfg.e_count, cfg.I, cfg.d), 0.02)
    return out


def small_config(T=96, d=128, E=8, k=2, I=192, e_start=0, e_count=None, zipf_s=0.0,
                 name="small") -> MoEConfig:
    return MoEConfig(name, T=T, d=d, E=E, k=k, I=I, e_start=e_start,
                     e_count=E if e_count is None else e_count, zipf_s=zipf_s, backward=True)


def histogram_summary(counts) -> dict:
    """Realised per-expert load, printed next to every skewed-routing result."""
    c = [int(v) for v in counts]
    tot = max(1, sum(c))
    srt = sorted(c, reverse=True)
    return {
        "assignments": sum(c),
        "max_share": srt[0] / tot,
        "top8_share": sum(srt[:8]) / tot,
        "empty_experts": sum(1 for v in c if v == 0),
        "min": srt[-1],
        "max": srt[0],
        "mean": tot / len(c),
        "std": math.sqrt(sum((v - tot / len(c)) ** 2 for v in c) / len(c)),
    }
