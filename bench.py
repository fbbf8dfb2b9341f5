#!/usr/bin/env python3
"""Benchmark of the fused MoE hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch that is already
resident in HBM: moe_route -> moe_fused_forward -> moe_fused_backward (when the
workload has a backward).  Prints ONE JSON line:

  value       useful TFLOP/s of the whole step (6*A*d*I forward + 12*A*d*I
              backward, A = realised routed rows) -- the metric the benchmark spec names
  roofline    the dominant kernel (the backward GEMM MegaKernel when the workload has a
              backward, else the forward one) against the bf16 dense MFMA peak, timed by HIP
              events around the call without its tail kernel; roofline_forward carries the
              forward GEMM MegaKernel beside it
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
  measured_ceilings  what this GPU sustains on a matrix-instruction-only kernel and on a plain
              copy, with the shader clock under that load, measured in this run; the
              roofline fractions stay against the published peaks

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N]
       python bench.py --model-shapes all [--tokens 8192] [--ep 8]   (sweep, one line per shape)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak (published)
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the shader clock needs some tens of milliseconds of load to ramp up: warm up for ~0.3 s
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2, help="index into BASELINE.json configs")
    ap.add_argument("--schedule", type=int, default=0)
    ap.add_argument("--tile-rows", type=int, default=0)
    ap.add_argument("--workers", type=int, default=0)
    ap.add_argument("--dw-split-rows", type=int, default=0,
                    help="backward: cut the weight-gradient reduction of experts with more rows than this "
                         "at fixed points (moe_opts_t.dw_split_rows); 0 = one sum per element")
    ap.add_argument("--no-backward", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--model-shapes", type=str, default="",
                    help="sweep instead of the contract line: comma-separated ids 1..12 of the "
                         "paper's model-shape table (or 'all'); one JSON line per shape")
    ap.add_argument("--tokens", type=int, default=8192, help="sweep: tokens (per rank)")
    ap.add_argument("--ep", type=int, default=1,
                    help="sweep: 1 = all experts local; W = one rank's share of W-way expert "
                         "parallelism (W*tokens resident tokens, N_exp/W local experts)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also launch the plain copy kernel on this many MiB, 5 times "
                         "(scale for the HBM byte counters of a rocprofv3 --pmc run)")
    ap.add_argument("--ceilings-only", action="store_true",
                    help="print only the measured matrix-instruction / copy / clock ceilings (one JSON line)")
    return ap.parse_args()


def event_ms(fn, n, before=None):
    """(average, median, min) milliseconds of fn() over n calls, HIP events on torch's current
    stream (the stream the library launches on).  `before` runs untimed ahead of every call."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n)]
    for a, b in evs:
        if before is not None:
            before()
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


def measured_traffic(cfg_name, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary
    (profiles/hbm_traffic_<workload>.txt, written by profile_summary.py
    from a FETCH_SIZE and a WRITE_SIZE run scaled by the calibration copy), or None."""
    path = ROOT / "profiles" / f"hbm_traffic_{cfg_name.replace('-', '_')}.txt"
    if not path.exists():
        return None
    for line in path.read_text().splitlines():
        if line.startswith(kernel) and "traffic_bytes_per_launch=" in line:
            return float(line.split("traffic_bytes_per_launch=")[1].split()[0])
    return None


def cpu_model():
    try:
        for line in Path("/proc/cpuinfo").read_text().splitlines():
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def measured_ceilings(moe):
    """Sustained matrix-instruction and copy rates of this GPU, measured here: a kernel of
    independent bf16 MFMA chains (no memory traffic) on every CU, and the library's copy kernel on
    1 GiB.  The shader clock is the kernel's own cycle counter over its 100 MHz wall clock."""
    import torch
    props = torch.cuda.get_device_properties(0)
    cus = props.multi_processor_count
    for _ in range(2):   # the first run ramps the clock up
        moe.moe_calibration_mfma(cus, 8, 20000)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    r = moe.moe_calibration_mfma(cus, 8, 40000)
    b.record()
    torch.cuda.synchronize()
    mfma_tflops = r["flop"] / (a.elapsed_time(b) * 1e-3) / 1e12
    clock_mhz = 100.0 * r["shader_clocks"] / max(1, r["ticks_100mhz"])
    src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ms = event_ms(lambda: moe.moe_calibration_copy(dst, src), 10)
    del src, dst
    return {"mfma_bf16_tflops": mfma_tflops, "shader_clock_mhz_under_mfma_load": clock_mhz,
            "copy_gbs_read_plus_write": 2.0 * (1 << 30) / (ms[1] * 1e-3) / 1e9,
            "published": {"mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS, "hbm_gbs": HBM_PEAK_GBS}}


def cpu_baseline(cfg, inp, has_bwd, budget_s):
    """The oracle as it stands, on the rows of the first S local experts (same inputs)."""
    import numpy as np
    import moe_synth
    import oracle
    sh_full = cfg.shape_dict()
    logits = inp["logits"].numpy()

    def run(S):
        sh = dict(sh_full, e_start=cfg.e_start, e_count=S)
        b = {k: oracle.bf16_bits(inp[k][:S] if k.startswith("w_") else inp[k])
             for k in ("x", "w_gate", "w_up", "w_down") + (("dy",) if has_bwd else ())}
        t0 = time.perf_counter()
        r = oracle.route(sh, logits, acc="f32")
        oracle.forward(sh, b["x"], b["w_gate"], b["w_up"], b["w_down"], r, acc="f32")
        if has_bwd:
            oracle.backward(sh, b["x"], b["dy"], b["w_gate"], b["w_up"], b["w_down"], r, acc="f32")
        dt = time.perf_counter() - t0
        rows = int(r["offsets"][-1])
        return dt, rows

    dt1, rows1 = run(1)
    per_expert = max(dt1, 1e-3)
    S = int(max(1, min(cfg.e_count, budget_s / per_expert)))
    dt, rows = (dt1, rows1) if S == 1 else run(S)
    flops = (18 if has_bwd else 6) * rows * cfg.d * cfg.I
    return {
        "value": flops / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.threads(),   # omp_get_max_threads() of the oracle's library
        "cpu_model": cpu_model(),
        "kind": "oracle",
        "sample": f"rows of the first {S} of {cfg.e_count} local experts ({rows} of the routed rows), "
                  f"route+forward{'+backward' if has_bwd else ''}, fp32 accumulate, {dt:.1f} s",
    }


def sweep_model_shapes(args):
    """Forward and backward MegaKernel timings over the paper's model-shape table (synthetic
    inputs drawn on the device).  One JSON line per shape; not the contract line."""
    import torch
    import moe_synth
    import paper_2604_19241_amd as moe
    ids = list(moe_synth.MODEL_SHAPES) if args.model_shapes == "all" else \
        [int(v) for v in args.model_shapes.split(",")]
    opts = moe.make_opts(schedule=args.schedule, tile_rows=args.tile_rows, workers=args.workers)
    for mid in ids:
        cfg = moe_synth.model_config(mid, tokens=args.tokens, ep=args.ep)
        shape = moe.make_shape(**cfg.shape_dict())
        sizes = moe.moe_workspace_bytes(shape)
        dev = moe_synth.make_inputs_device(cfg, "cuda")
        ws = {k: torch.empty(sizes[k], dtype=torch.uint8, device="cuda") for k in ("route", "fwd", "bwd")}
        saved = moe.alloc_saved(shape, "cuda")
        y = torch.empty((cfg.T, cfg.d), dtype=torch.bfloat16, device="cuda")
        state, grads = {}, {}

        def route():
            state["r"] = moe.moe_route(shape, dev["logits"], ws=ws["route"])

        def fwd():
            moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"],
                                  state["r"], y=y, saved=saved, ws=ws["fwd"], opts=opts)

        def bwd():
            grads["out"] = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"],
                                                  dev["w_up"], dev["w_down"], state["r"], saved,
                                                  ws=ws["bwd"], opts=opts, out=grads.get("out"))

        route()
        t_end = time.perf_counter() + 0.4          # clocks ramp up under load
        while time.perf_counter() < t_end:
            fwd()
            bwd()
            torch.cuda.synchronize()
        assert moe.moe_device_status(ws["fwd"]) == 0 and moe.moe_device_status(ws["bwd"]) == 0
        n = max(5, min(args.steps, 30))
        ms_r, ms_f, ms_b = event_ms(route, n), event_ms(fwd, n), event_ms(bwd, n)
        A = int(state["r"].offsets[-1].item())
        f_fwd = 6.0 * A * cfg.d * cfg.I
        counts = state["r"].counts.cpu().tolist()
        print(json.dumps({
            "sweep": "model-shapes", "id": mid, "workload": cfg.name, "T": cfg.T, "d": cfg.d,
            "I": cfg.I, "E": cfg.E, "k": cfg.k, "local_experts": cfg.e_count, "routed_rows": A,
            "rows_per_expert_mean": A / cfg.e_count, "rows_per_expert_max": max(counts),
            "route_ms": ms_r[1], "forward_ms": ms_f[1], "backward_ms": ms_b[1],
            "forward_tflops": f_fwd / (ms_f[1] * 1e-3) / 1e12,
            "backward_tflops": 2 * f_fwd / (ms_b[1] * 1e-3) / 1e12,
            "step_tflops": 3 * f_fwd / ((ms_r[1] + ms_f[1] + ms_b[1]) * 1e-3) / 1e12,
            "dtype": "bf16", "data": "synthetic (drawn on the device)", "timing": "median of HIP events",
        }), flush=True)
        del dev, ws, saved, y, grads, state
        torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.model_shapes:
        import torch
        assert torch.cuda.is_available(), "bench.py needs an MI355X"
        torch.cuda.set_device(0)
        sweep_model_shapes(args)
        return
    if args.ceilings_only:
        import torch
        import paper_2604_19241_amd as moe
        assert torch.cuda.is_available(), "bench.py needs an MI355X"
        torch.cuda.set_device(0)
        print(json.dumps({"measured_ceilings": measured_ceilings(moe)}), flush=True)
        return
    import torch
    import moe_synth
    import paper_2604_19241_amd as moe

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    cfg = moe_synth.CONFIGS[args.config]
    shape = moe.make_shape(**cfg.shape_dict())
    sizes = moe.moe_workspace_bytes(shape)
    has_bwd = cfg.backward and not args.no_backward and sizes["bwd"] > 256

    inp = moe_synth.make_inputs(cfg, with_dy=has_bwd)
    dev = {k: v.cuda() for k, v in inp.items()}
    opts = moe.make_opts(schedule=args.schedule, tile_rows=args.tile_rows, workers=args.workers,
                         dw_split_rows=args.dw_split_rows)
    ws_route = torch.empty(sizes["route"], dtype=torch.uint8, device="cuda")
    ws_fwd = torch.empty(sizes["fwd"], dtype=torch.uint8, device="cuda")
    ws_bwd = (torch.empty(moe.moe_backward_workspace_bytes(shape, opts), dtype=torch.uint8, device="cuda")
              if has_bwd else None)
    saved = moe.alloc_saved(shape, "cuda") if has_bwd else None
    y = torch.empty((cfg.T, cfg.d), dtype=torch.bfloat16, device="cuda")
    state = {}

    def route():
        state["r"] = moe.moe_route(shape, dev["logits"], ws=ws_route)

    def fwd():
        moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"],
                              state["r"], y=y, saved=saved, ws=ws_fwd, opts=opts)

    grads = {}

    def bwd():
        out = moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"],
                                     dev["w_down"], state["r"], saved, ws=ws_bwd, opts=opts,
                                     out=grads.get("out"))
        grads["out"] = out

    def step():
        route()
        fwd()
        if has_bwd:
            bwd()

    if args.calibration_copy_mib > 0:
        src = torch.zeros(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            moe.moe_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert moe.moe_device_status(ws_fwd) == 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    A = int(state["r"].offsets[-1].item())
    f_fwd = 6.0 * A * cfg.d * cfg.I
    f_bwd = 12.0 * A * cfg.d * cfg.I if has_bwd else 0.0
    value = (f_fwd + f_bwd) / (ms_per_step * 1e-3) / 1e12

    # per-call timings with HIP events on the launch stream
    n = max(10, min(args.steps, 100))
    ms_route = event_ms(route, n)
    ms_fwd = event_ms(fwd, n)
    ms_bwd = event_ms(bwd, n) if has_bwd else None
    # not part of the step on one GPU: the W > 1 index stage (Algorithm 1, lines 3-14) for one
    # rank of 8, with the realised histogram standing in for every rank's
    ms_gmap = None
    if cfg.e_count == cfg.E and cfg.E % 8 == 0:
        c_all = torch.stack([state["r"].counts] * 8).contiguous()
        ws_g = torch.empty(8 * cfg.E, dtype=torch.uint8, device="cuda")
        ms_gmap = event_ms(lambda: moe.moe_global_map(shape, 8, 3, state["r"], c_all, ws=ws_g), n)
    # the same with cold caches: a 512 MiB streaming copy ahead of every call evicts the weights,
    # activations and routing tables from the L2s and the 256 MB Infinity Cache
    flush_src = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda")
    flush_dst = torch.empty_like(flush_src)

    def flush():
        moe.moe_calibration_copy(flush_dst, flush_src)

    nc = min(n, 30)
    cold_fwd = event_ms(fwd, nc, before=flush)
    cold_bwd = event_ms(bwd, nc, before=flush) if has_bwd else None
    del flush_src, flush_dst
    fwd_tflops = f_fwd / (ms_fwd[0] * 1e-3) / 1e12
    # The GEMM MegaKernels alone: the same calls without their tail kernel (combine / dX).  With
    # the other schedules the tail runs inside the worker launches and the whole call is timed.
    split = args.schedule in (0, 3)
    opts_mega = moe.make_opts(schedule=args.schedule, tile_rows=args.tile_rows, workers=args.workers,
                              skip_tail=1 if split else 0, dw_split_rows=args.dw_split_rows)

    def fwd_mega():
        moe.moe_fused_forward(shape, dev["x"], dev["w_gate"], dev["w_up"], dev["w_down"],
                              state["r"], y=y, saved=saved, ws=ws_fwd, opts=opts_mega)

    def bwd_mega():
        moe.moe_fused_backward(shape, dev["dy"], dev["x"], dev["w_gate"], dev["w_up"],
                               dev["w_down"], state["r"], saved, ws=ws_bwd, opts=opts_mega,
                               out=grads.get("out"))

    ms_fwd_mega = event_ms(fwd_mega, n)
    ms_bwd_mega = event_ms(bwd_mega, n) if has_bwd else None
    fwd()                       # leave complete outputs behind
    if has_bwd:
        bwd()

    ceilings = measured_ceilings(moe)

    def roof(kernel, what, flops, ms, ms_call):
        tf = flops / (ms[0] * 1e-3) / 1e12
        return {
            "kernel": f"{kernel} ({what}; the HIP events also span its prologue launches, "
                      f"15-22 us, and with schedule 1 or 2 the tail tasks)",
            "bound": "mfma",
            "achieved": tf,
            "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": tf / MFMA_BF16_PEAK_TFLOPS,
            "traffic": measured_traffic(cfg.name, kernel),
            "traffic_source": f"profiles/hbm_traffic_{cfg.name.replace('-', '_')}.txt (committed summary of "
                              f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command; not measured in this run)",
            "frac_of_measured_mfma": tf / ceilings["mfma_bf16_tflops"],
            "flops_per_launch": flops,
            "avg_ms": ms[0], "median_ms": ms[1], "min_ms": ms[2],
            "tail_kernel_ms": (ms_call[0] - ms[0]) if split else None,
        }

    roof_fwd = roof("fwd_worker_kernel", "forward GEMM MegaKernel, 6*A*d*I flop per launch",
                    f_fwd, ms_fwd_mega, ms_fwd)
    roof_bwd = roof("bwd_worker_kernel", "backward GEMM MegaKernel, 12*A*d*I flop per launch",
                    f_bwd, ms_bwd_mega, ms_bwd) if has_bwd else None
    roofline = roof_bwd if has_bwd else roof_fwd
    counts = state["r"].counts.cpu().tolist()
    out = {
        "metric": "fused MoE fwd+bwd TFLOP/s" if has_bwd else "fused MoE fwd TFLOP/s",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} "
                               f"k={cfg.k} I={cfg.I} local_experts={cfg.e_count}, route+forward"
                               f"{'+backward' if has_bwd else ''}",
                   "routed_rows": A, "schedule": args.schedule, "tile_rows": args.tile_rows,
                   "dw_split_rows": args.dw_split_rows},
        "tokens_per_s": cfg.T / (ms_per_step * 1e-3),
        "pct_of_bf16_mfma_peak": 100.0 * value / MFMA_BF16_PEAK_TFLOPS,
        "phases_ms": {"route": ms_route[0], "forward": ms_fwd[0],
                      "backward": ms_bwd[0] if ms_bwd else None},
        "global_map_w8_ms": ms_gmap[1] if ms_gmap else None,
        "phases_ms_median_min": {"route": ms_route[1:], "forward": ms_fwd[1:],
                                 "backward": ms_bwd[1:] if ms_bwd else None},
        "phases_ms_cold_caches": {"forward": cold_fwd[0], "backward": cold_bwd[0] if cold_bwd else None},
        "forward_tflops": fwd_tflops,
        "backward_tflops": (f_bwd / (ms_bwd[0] * 1e-3) / 1e12) if ms_bwd else None,
        "expert_load": moe_synth.histogram_summary(counts),
        "roofline": roofline,
        "measured_ceilings": ceilings,
    }
    if has_bwd:
        out["roofline_forward"] = roof_fwd
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, has_bwd, args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
