"""Thin ctypes binding of libuniep_moe.so (include/uniep_moe.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the hot path runs in the library's kernels.  There is
no CPU fallback: a missing library or a failed call raises.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libuniep_moe.so"

MOE_OK = 0
MOE_ERR_ARG, MOE_ERR_SHAPE, MOE_ERR_WORKSPACE, MOE_ERR_HIP, MOE_ERR_DEVICE = -1, -2, -3, -4, -5

EXPORTS = ("moe_workspace_bytes", "moe_backward_workspace_bytes", "moe_saved_layout", "moe_route", "moe_fused_forward",
           "moe_fused_backward", "moe_route_backward", "moe_global_map", "moe_device_status",
           "moe_status_string", "moe_calibration_copy", "moe_perf_model_eval",
           "moe_perf_model_search", "moe_route_static", "moe_calibration_mfma")

ROUTE_STATIC_SCRATCH_BYTES = 4 << 20   # MOE_ROUTE_STATIC_SCRATCH_BYTES


class MoEShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "E", "k", "I", "e_start", "e_count")]


class MoERoutingC(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm")]


class MoEOpts(ctypes.Structure):
    _fields_ = [("schedule", ctypes.c_int32), ("workers", ctypes.c_int32),
                ("spin_limit_ms", ctypes.c_int32), ("tile_rows", ctypes.c_int32),
                ("skip_tail", ctypes.c_int32), ("dw_accumulate", ctypes.c_int32),
                ("dw_split_rows", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 1)]


class MoEError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


_lib = None


def load_library():
    """Load the HIP library; raises if it was not built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_19241_amd.build` "
                "(hipcc, gfx950). There is no CPU fallback.")
        lib = ctypes.CDLL(str(LIB_PATH))
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS:
            getattr(lib, name)   # AttributeError if a declared symbol is not exported
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load_library().moe_status_string(int(code)).decode()


def _check(code: int, where: str):
    if code != MOE_OK:
        raise MoEError(code, where)


def make_shape(T, d, E, k, I, e_start=0, e_count=None) -> MoEShape:
    return MoEShape(int(T), int(d), int(E), int(k), int(I), int(e_start),
                    int(E if e_count is None else e_count))


def make_opts(schedule=0, workers=0, spin_limit_ms=0, tile_rows=0, skip_tail=0,
              dw_accumulate=0, dw_split_rows=0) -> MoEOpts:
    o = MoEOpts()
    o.schedule, o.workers, o.spin_limit_ms, o.tile_rows = schedule, workers, spin_limit_ms, tile_rows
    o.skip_tail = skip_tail
    o.dw_accumulate = dw_accumulate
    o.dw_split_rows = dw_split_rows
    return o


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def moe_workspace_bytes(shape: MoEShape) -> dict:
    vals = [ctypes.c_size_t(0) for _ in range(4)]
    _check(load_library().moe_workspace_bytes(ctypes.byref(shape), *[ctypes.byref(v) for v in vals]),
           "moe_workspace_bytes")
    return dict(zip(("route", "fwd", "bwd", "saved"), (int(v.value) for v in vals)))


def moe_backward_workspace_bytes(shape: MoEShape, opts: MoEOpts | None = None) -> int:
    v = ctypes.c_size_t(0)
    _check(load_library().moe_backward_workspace_bytes(
        ctypes.byref(shape), ctypes.byref(opts) if opts is not None else None, ctypes.byref(v)),
        "moe_backward_workspace_bytes")
    return int(v.value)


def moe_saved_layout(shape: MoEShape) -> dict:
    vals = [ctypes.c_size_t(0) for _ in range(3)]
    _check(load_library().moe_saved_layout(ctypes.byref(shape), *[ctypes.byref(v) for v in vals]),
           "moe_saved_layout")
    return dict(zip(("gu", "h", "o"), (int(v.value) for v in vals)))


@dataclass
class Routing:
    topk_idx: torch.Tensor   # [T,k] i32
    topk_w: torch.Tensor     # [T,k] f32
    counts: torch.Tensor     # [e_count] i32
    offsets: torch.Tensor    # [e_count+1] i32
    perm: torch.Tensor       # [T*k] i32
    inv_perm: torch.Tensor   # [T,k] i32

    def c_struct(self) -> MoERoutingC:
        return MoERoutingC(*(t.data_ptr() for t in (self.topk_idx, self.topk_w, self.counts,
                                                    self.offsets, self.perm, self.inv_perm)))


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def moe_route(shape: MoEShape, logits: torch.Tensor, ws: torch.Tensor | None = None) -> Routing:
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
    assert tuple(logits.shape) == (shape.T, shape.E)
    dev = logits.device
    T, k, ec = shape.T, shape.k, shape.e_count
    r = Routing(torch.empty((T, k), dtype=torch.int32, device=dev),
                torch.empty((T, k), dtype=torch.float32, device=dev),
                torch.empty(ec, dtype=torch.int32, device=dev),
                torch.empty(ec + 1, dtype=torch.int32, device=dev),
                torch.empty(T * k, dtype=torch.int32, device=dev),
                torch.empty((T, k), dtype=torch.int32, device=dev))
    if ws is None:
        ws = _ws(moe_workspace_bytes(shape)["route"], dev)
    cs = r.c_struct()
    _check(load_library().moe_route(ctypes.byref(shape), _ptr(logits), ctypes.byref(cs), _ptr(ws),
                                    ctypes.c_size_t(ws.numel()), _stream(dev)), "moe_route")
    return r


def moe_route_static(shape: MoEShape, logits: torch.Tensor, out: Routing) -> Routing:
    """moe_route without a workspace: the library's file-scope scratch holds the histogram.
    The caller brings the six output arrays (`out`), so the call itself allocates nothing."""
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
    assert tuple(logits.shape) == (shape.T, shape.E)
    cs = out.c_struct()
    _check(load_library().moe_route_static(ctypes.byref(shape), _ptr(logits), ctypes.byref(cs),
                                           _stream(logits.device)), "moe_route_static")
    return out


def alloc_routing(shape: MoEShape, device) -> Routing:
    T, k, ec = shape.T, shape.k, shape.e_count
    return Routing(torch.empty((T, k), dtype=torch.int32, device=device),
                   torch.empty((T, k), dtype=torch.float32, device=device),
                   torch.empty(ec, dtype=torch.int32, device=device),
                   torch.empty(ec + 1, dtype=torch.int32, device=device),
                   torch.empty(T * k, dtype=torch.int32, device=device),
                   torch.empty((T, k), dtype=torch.int32, device=device))


def moe_calibration_mfma(workgroups: int, waves: int, iters: int, device="cuda") -> dict:
    """Runs the dependent-free MFMA stream once and returns its shader clocks and 100 MHz ticks
    (synchronises to read them).  The caller times the call itself for TFLOP/s."""
    import numpy as np
    rng = np.random.default_rng(3)
    # pairs of bf16 values in +-[0.5, 2): random mantissas, two exponents, random signs
    hi = 0x3F00 + rng.integers(0, 256, (1024, 2)) + (rng.integers(0, 2, (1024, 2)) << 15)
    seed = torch.from_numpy((hi[:, 0] | (hi[:, 1] << 16)).astype(np.uint32).view(np.int32)).to(device)
    sink = torch.zeros(1, dtype=torch.float32, device=device)
    clocks = torch.zeros(2, dtype=torch.int64, device=device)
    _check(load_library().moe_calibration_mfma(ctypes.c_int32(workgroups), ctypes.c_int32(waves),
                                               ctypes.c_int32(iters), _ptr(seed), _ptr(sink),
                                               _ptr(clocks), _stream(torch.device(device))),
           "moe_calibration_mfma")
    c = clocks.cpu().tolist()
    return {"shader_clocks": int(c[0]), "ticks_100mhz": int(c[1]),
            "flop": float(workgroups) * waves * iters * 8 * 32768.0}


def moe_fused_forward(shape: MoEShape, x, w_gate, w_up, w_down, routing: Routing, y=None,
                      saved: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                      opts: MoEOpts | None = None) -> torch.Tensor:
    dev = x.device
    for t in (x, w_gate, w_up, w_down):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
    assert tuple(x.shape) == (shape.T, shape.d)
    assert tuple(w_gate.shape) == (shape.e_count, shape.d, shape.I) == tuple(w_up.shape)
    assert tuple(w_down.shape) == (shape.e_count, shape.I, shape.d)
    if y is None:
        y = torch.empty((shape.T, shape.d), dtype=torch.bfloat16, device=dev)
    if ws is None:
        ws = _ws(moe_workspace_bytes(shape)["fwd"], dev)
    cs = routing.c_struct()
    _check(load_library().moe_fused_forward(
        ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down), ctypes.byref(cs),
        _ptr(y), _ptr(saved), _ptr(ws), ctypes.c_size_t(ws.numel()),
        ctypes.byref(opts) if opts is not None else None, _stream(dev)), "moe_fused_forward")
    return y


def moe_fused_backward(shape: MoEShape, dy, x, w_gate, w_up, w_down, routing: Routing,
                       saved: torch.Tensor, want_dtopk_w: bool = True,
                       ws: torch.Tensor | None = None, opts: MoEOpts | None = None,
                       out: dict | None = None) -> dict:
    dev = x.device
    for t in (dy, x, w_gate, w_up, w_down):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
    assert tuple(dy.shape) == (shape.T, shape.d)
    if opts is not None and opts.dw_accumulate:
        # the caller's fp32 gradient buffers are added to
        assert out is not None, "dw_accumulate needs the caller's fp32 dw_gate / dw_up / dw_down in `out`"
        for key, w in (("dw_gate", w_gate), ("dw_up", w_up), ("dw_down", w_down)):
            g = out[key]
            assert g.is_cuda and g.dtype == torch.float32 and g.is_contiguous() and g.shape == w.shape
    if out is None:
        out = {
            "dx": torch.empty_like(x),
            "dw_gate": torch.empty_like(w_gate),
            "dw_up": torch.empty_like(w_up),
            "dw_down": torch.empty_like(w_down),
            "dtopk_w": torch.empty((shape.T, shape.k), dtype=torch.float32, device=dev)
            if want_dtopk_w else None,
        }
    if ws is None:
        ws = _ws(moe_backward_workspace_bytes(shape, opts), dev)
    cs = routing.c_struct()
    _check(load_library().moe_fused_backward(
        ctypes.byref(shape), _ptr(dy), _ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
        ctypes.byref(cs), _ptr(saved), _ptr(out["dx"]), _ptr(out["dw_gate"]), _ptr(out["dw_up"]),
        _ptr(out["dw_down"]), _ptr(out.get("dtopk_w")), _ptr(ws), ctypes.c_size_t(ws.numel()),
        ctypes.byref(opts) if opts is not None else None, _stream(dev)), "moe_fused_backward")
    return out


def moe_route_backward(shape: MoEShape, routing: "Routing", dtopk_w: torch.Tensor,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dlogits [T,E] fp32 from the gate gradients dtopk_w [T,k] fp32 and the routing moe_route made."""
    dev = dtopk_w.device
    assert dtopk_w.dtype == torch.float32 and dtopk_w.is_contiguous()
    if out is None:
        out = torch.empty((shape.T, shape.E), dtype=torch.float32, device=dev)
    lib = load_library()
    lib.moe_route_backward.argtypes = [ctypes.c_void_p] * 6
    _check(lib.moe_route_backward(ctypes.byref(shape), _ptr(routing.topk_idx), _ptr(routing.topk_w),
                                  _ptr(dtopk_w), _ptr(out), _stream(dev)), "moe_route_backward")
    return out


class MoEGlobalMapC(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("dst_rank", "dst_expert", "dst_off", "dst_row", "send", "n_dst_ranks",
                 "recv_offsets")]


@dataclass
class GlobalMap:
    dst_rank: torch.Tensor      # [T,k] i32
    dst_expert: torch.Tensor    # [T,k] i32
    dst_off: torch.Tensor       # [T,k] i32
    dst_row: torch.Tensor       # [T,k] i32
    send: torch.Tensor          # [T,k] i32
    n_dst_ranks: torch.Tensor   # [T] i32
    recv_offsets: torch.Tensor  # [E/W + 1] i32


def moe_global_map(shape: MoEShape, W: int, rank: int, routing: "Routing", c_all: torch.Tensor,
                   ws: Optional[torch.Tensor] = None) -> GlobalMap:
    """Destination (rank, local expert, offset, row) of every slot of this rank's tokens, from
    the all-gathered histograms c_all [W,E] int32 (device)."""
    dev = c_all.device
    assert c_all.is_cuda and c_all.dtype == torch.int32 and c_all.is_contiguous()
    assert tuple(c_all.shape) == (W, shape.E)
    T, k = shape.T, shape.k

    def i32(*size):
        return torch.empty(size, dtype=torch.int32, device=dev)

    g = GlobalMap(i32(T, k), i32(T, k), i32(T, k), i32(T, k), i32(T, k), i32(T),
                  i32(shape.E // max(W, 1) + 1))
    if ws is None:
        ws = _ws(8 * shape.E, dev)
    cs = routing.c_struct()
    gs = MoEGlobalMapC(*(t.data_ptr() for t in (g.dst_rank, g.dst_expert, g.dst_off, g.dst_row,
                                                g.send, g.n_dst_ranks, g.recv_offsets)))
    lib = load_library()
    lib.moe_global_map.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_size_t, ctypes.c_void_p]
    _check(lib.moe_global_map(ctypes.byref(shape), int(W), int(rank), ctypes.byref(cs), _ptr(c_all),
                              ctypes.byref(gs), _ptr(ws), ctypes.c_size_t(ws.numel()),
                              _stream(dev)), "moe_global_map")
    return g


def moe_device_status(ws: torch.Tensor) -> int:
    return int(load_library().moe_device_status(_ptr(ws), _stream(ws.device)))


def moe_calibration_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain streaming copy kernel of known traffic (profiler counter calibration)."""
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    lib = load_library()
    lib.moe_calibration_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    _check(lib.moe_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(src.device)),
           "moe_calibration_copy")


def alloc_saved(shape: MoEShape, device) -> torch.Tensor:
    return _ws(moe_workspace_bytes(shape)["saved"], device)


def saved_views(shape: MoEShape, saved: torch.Tensor) -> dict:
    """bf16 views of the stash: gu [A_cap,2I], h [A_cap,I], o [A_cap,d]."""
    L = moe_saved_layout(shape)
    A = shape.T * shape.k

    def view(off, cols):
        return saved[off:off + A * cols * 2].view(torch.bfloat16).view(A, cols)

    return {"gu": view(L["gu"], 2 * shape.I), "h": view(L["h"], shape.I), "o": view(L["o"], shape.d)}


# ---- analytical performance model and configuration search (host only) -------

class MoEPerfHw(ctypes.Structure):
    _fields_ = [("n_sm", ctypes.c_int32), ("w_sat", ctypes.c_int32), ("p_peak", ctypes.c_double),
                ("beta_hbm", ctypes.c_double), ("beta_link", ctypes.c_double),
                ("tau_sync", ctypes.c_double), ("mu", ctypes.c_double * 3)]


class MoEPerfProblem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_tok", "h_dim", "h_inter", "n_exp", "top_k", "world",
                                              "b_m", "b_n", "elem_bytes")]


class MoEPerfConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_disp", "n_relay", "n_comb", "n_red", "warps")]


PERF_LATENCY_FIELDS = ("t_up", "t_down", "l_swiglu", "l_disp", "l_up", "l_s1", "l_comb", "t_red",
                       "l_down", "l_s2", "l_total")


class MoEPerfLatency(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in PERF_LATENCY_FIELDS]


def make_perf_hw(n_sm, p_peak, beta_hbm, beta_link, w_sat=1024, tau_sync=2e-6,
                 mu=(0.7, 0.65, 0.6)) -> MoEPerfHw:
    return MoEPerfHw(int(n_sm), int(w_sat), float(p_peak), float(beta_hbm), float(beta_link),
                     float(tau_sync), (ctypes.c_double * 3)(*map(float, mu)))


def make_perf_problem(n_tok, h_dim, h_inter, n_exp, top_k, world, b_m=128, b_n=128,
                      elem_bytes=2) -> MoEPerfProblem:
    return MoEPerfProblem(*map(int, (n_tok, h_dim, h_inter, n_exp, top_k, world, b_m, b_n, elem_bytes)))


def moe_perf_model_eval(hw: MoEPerfHw, problem: MoEPerfProblem, config) -> dict:
    c = config if isinstance(config, MoEPerfConfig) else MoEPerfConfig(*map(int, config))
    out = MoEPerfLatency()
    _check(load_library().moe_perf_model_eval(ctypes.byref(hw), ctypes.byref(problem), ctypes.byref(c),
                                              ctypes.byref(out)), "moe_perf_model_eval")
    return {n: getattr(out, n) for n in PERF_LATENCY_FIELDS}


def moe_perf_model_search(hw: MoEPerfHw, problem: MoEPerfProblem) -> dict:
    best, lat = MoEPerfConfig(), MoEPerfLatency()
    n_enum, n_valid = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load_library().moe_perf_model_search(ctypes.byref(hw), ctypes.byref(problem), ctypes.byref(best),
                                                ctypes.byref(lat), ctypes.byref(n_enum),
                                                ctypes.byref(n_valid)), "moe_perf_model_search")
    return {"config": (best.n_disp, best.n_relay, best.n_comb, best.n_red, best.warps),
            "latency": {n: getattr(lat, n) for n in PERF_LATENCY_FIELDS},
            "n_enumerated": int(n_enum.value), "n_valid": int(n_valid.value)}
