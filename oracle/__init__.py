"""ctypes front end of the CPU oracle (oracle/moe_oracle.c).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this package.  It never imports the
HIP package and shares nothing with it.

The C file is built twice, once per accumulate type:
  acc="f64"  double accumulate (the default for pins and parity),
  acc="f32"  float accumulate.
Inputs are numpy arrays: uint16 bf16 bit patterns (in_dtype 0) or float64
(in_dtype 1); floating outputs are float64 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "moe_oracle.c"
_LIBS: dict = {}

SHAPE_KEYS = ("T", "d", "E", "k", "I", "e_start", "e_count")


def lib_path(acc: str) -> Path:
    return _HERE / f"libmoe_oracle_{acc}.so"


def build(force: bool = True) -> None:
    """Compile both accumulate-type variants with gcc (-O3, no fast-math, OpenMP)."""
    for acc, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(acc)
        if out.exists() and not force and out.stat().st_mtime >= _SRC.stat().st_mtime:
            continue
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math",
               f"-DACC_T={ctype}", f"-DSFX={acc}", str(_SRC), "-o", str(out), "-lm"]
        subprocess.run(cmd, check=True)


def _load(acc: str):
    if acc not in ("f64", "f32"):
        raise ValueError("acc must be 'f64' or 'f32'")
    if acc not in _LIBS:
        p = lib_path(acc)
        if not p.exists() or p.stat().st_mtime < _SRC.stat().st_mtime:
            build(force=False)
        _LIBS[acc] = ctypes.CDLL(str(p))
    return _LIBS[acc]


def threads() -> int:
    """Threads the oracle's parallel loops run on: omp_get_max_threads() of the loaded library."""
    fn = getattr(_load("f32"), "oracle_max_threads_f32")
    fn.restype = ctypes.c_int
    return max(1, int(fn()))


def _shape_arr(shape: dict) -> np.ndarray:
    return np.array([int(shape[key]) for key in SHAPE_KEYS], dtype=np.int32)


def _p(a):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"], "oracle inputs must be C-contiguous"
    return ctypes.c_void_p(a.ctypes.data)


def _in(a):
    """-> (array kept alive, in_dtype) for x / dy / weights."""
    if a is None:
        return None, 0
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return a, 0
    if a.dtype == np.float64:
        return a, 1
    raise TypeError(f"oracle inputs must be uint16 (bf16 bits) or float64, got {a.dtype}")


def _same_dtype(*arrs):
    dts = {a[1] for a in arrs if a[0] is not None}
    if len(dts) != 1:
        raise TypeError("x, dy and the weights must share one dtype")
    return dts.pop()


def route(shape: dict, logits: np.ndarray, acc: str = "f64") -> dict:
    """topk_idx [T,k] i32, topk_w [T,k] f32, counts [e_count], offsets [e_count+1],
    perm [T*k] (row -> flat slot, -1 beyond A), inv_perm [T,k] (slot -> row or -1)."""
    lib = _load(acc)
    sh = _shape_arr(shape)
    T, k, ec = int(shape["T"]), int(shape["k"]), int(shape["e_count"])
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    assert logits.shape == (T, int(shape["E"]))
    out = {
        "topk_idx": np.empty((T, k), np.int32),
        "topk_w": np.empty((T, k), np.float32),
        "counts": np.empty(ec, np.int32),
        "offsets": np.empty(ec + 1, np.int32),
        "perm": np.empty(T * k, np.int32),
        "inv_perm": np.empty((T, k), np.int32),
    }
    rc = getattr(lib, f"oracle_route_{acc}")(
        _p(sh), _p(logits), _p(out["topk_idx"]), _p(out["topk_w"]), _p(out["counts"]),
        _p(out["offsets"]), _p(out["perm"]), _p(out["inv_perm"]))
    if rc != 0:
        raise ValueError("oracle_route: bad shape")
    return out


def route_backward(shape: dict, logits: np.ndarray, topk_idx: np.ndarray, dtopk_w: np.ndarray,
                   acc: str = "f64") -> np.ndarray:
    """dlogits [T,E] (float64): gradient of the gates with respect to the logits, selection fixed."""
    lib = _load(acc)
    sh = _shape_arr(shape)
    T, E, k = int(shape["T"]), int(shape["E"]), int(shape["k"])
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    g = np.ascontiguousarray(dtopk_w, dtype=np.float32)
    assert logits.shape == (T, E) and idx.shape == (T, k) and g.shape == (T, k)
    out = np.empty((T, E), np.float64)
    rc = getattr(lib, f"oracle_route_backward_{acc}")(_p(sh), _p(logits), _p(idx), _p(g), _p(out))
    if rc != 0:
        raise ValueError("oracle_route_backward: bad shape")
    return out


def forward(shape: dict, x, w_gate, w_up, w_down, routing: dict, round_bf16: bool = True,
            acc: str = "f64", stages: bool = False) -> dict:
    """y [T,d]; with stages=True also G,U,h [A,I] and o [A,d] (row order)."""
    lib = _load(acc)
    sh = _shape_arr(shape)
    T, d, I = int(shape["T"]), int(shape["d"]), int(shape["I"])
    xs, wgs, wus, wds = _in(x), _in(w_gate), _in(w_up), _in(w_down)
    dt = _same_dtype(xs, wgs, wus, wds)
    A = int(routing["offsets"][-1])
    out = {"y": np.empty((T, d), np.float64)}
    if stages:
        for key, cols in (("G", I), ("U", I), ("h", I), ("o", d)):
            out[key] = np.empty((A, cols), np.float64)
    tw = np.ascontiguousarray(routing["topk_w"], dtype=np.float32)
    getattr(lib, f"oracle_forward_{acc}")(
        _p(sh), ctypes.c_int(dt), _p(xs[0]), _p(wgs[0]), _p(wus[0]), _p(wds[0]), _p(tw),
        _p(routing["offsets"]), _p(routing["perm"]), _p(routing["inv_perm"]),
        ctypes.c_int(1 if round_bf16 else 0), _p(out["y"]), _p(out.get("G")), _p(out.get("U")),
        _p(out.get("h")), _p(out.get("o")))
    return out


def forward_tokens(shape: dict, x, w_gate, w_up, w_down, routing: dict, tokens,
                   round_bf16: bool = True, acc: str = "f64", with_o: bool = False) -> dict:
    lib = _load(acc)
    sh = _shape_arr(shape)
    d, k = int(shape["d"]), int(shape["k"])
    xs, wgs, wus, wds = _in(x), _in(w_gate), _in(w_up), _in(w_down)
    dt = _same_dtype(xs, wgs, wus, wds)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    out = {"y": np.empty((len(tok), d), np.float64)}
    if with_o:
        out["o"] = np.empty((len(tok), k, d), np.float64)
    tw = np.ascontiguousarray(routing["topk_w"], dtype=np.float32)
    ti = np.ascontiguousarray(routing["topk_idx"], dtype=np.int32)
    getattr(lib, f"oracle_forward_tokens_{acc}")(
        _p(sh), ctypes.c_int(dt), _p(xs[0]), _p(wgs[0]), _p(wus[0]), _p(wds[0]), _p(ti), _p(tw),
        ctypes.c_int(1 if round_bf16 else 0), ctypes.c_int(len(tok)), _p(tok), _p(out["y"]),
        _p(out.get("o")))
    return out


def backward(shape: dict, x, dy, w_gate, w_up, w_down, routing: dict, round_bf16: bool = True,
             acc: str = "f64", stages: bool = False) -> dict:
    """dx [T,d], dw_gate/dw_up [e_count,d,I], dw_down [e_count,I,d], dtopk_w [T,k];
    with stages=True also dG,dU [A,I], dXp,dO [A,d]."""
    lib = _load(acc)
    sh = _shape_arr(shape)
    T, d, I, k, ec = (int(shape[key]) for key in ("T", "d", "I", "k", "e_count"))
    xs, dys, wgs, wus, wds = _in(x), _in(dy), _in(w_gate), _in(w_up), _in(w_down)
    dt = _same_dtype(xs, dys, wgs, wus, wds)
    A = int(routing["offsets"][-1])
    out = {
        "dx": np.empty((T, d), np.float64),
        "dw_gate": np.empty((ec, d, I), np.float64),
        "dw_up": np.empty((ec, d, I), np.float64),
        "dw_down": np.empty((ec, I, d), np.float64),
        "dtopk_w": np.empty((T, k), np.float64),
    }
    if stages:
        for key, cols in (("dG", I), ("dU", I), ("dXp", d), ("dO", d)):
            out[key] = np.empty((A, cols), np.float64)
    tw = np.ascontiguousarray(routing["topk_w"], dtype=np.float32)
    getattr(lib, f"oracle_backward_{acc}")(
        _p(sh), ctypes.c_int(dt), _p(xs[0]), _p(dys[0]), _p(wgs[0]), _p(wus[0]), _p(wds[0]),
        _p(tw), _p(routing["offsets"]), _p(routing["perm"]), _p(routing["inv_perm"]),
        ctypes.c_int(1 if round_bf16 else 0), _p(out["dx"]), _p(out["dw_gate"]),
        _p(out["dw_up"]), _p(out["dw_down"]), _p(out["dtopk_w"]), _p(out.get("dG")),
        _p(out.get("dU")), _p(out.get("dXp")), _p(out.get("dO")))
    return out


def backward_experts(shape: dict, x, dy, w_gate, w_up, w_down, routing: dict, experts,
                     round_bf16: bool = True, acc: str = "f64") -> dict:
    """Weight gradients of the listed local experts, packed in list order."""
    lib = _load(acc)
    sh = _shape_arr(shape)
    d, I = int(shape["d"]), int(shape["I"])
    xs, dys, wgs, wus, wds = _in(x), _in(dy), _in(w_gate), _in(w_up), _in(w_down)
    dt = _same_dtype(xs, dys, wgs, wus, wds)
    ex = np.ascontiguousarray(experts, dtype=np.int32)
    out = {
        "dw_gate": np.empty((len(ex), d, I), np.float64),
        "dw_up": np.empty((len(ex), d, I), np.float64),
        "dw_down": np.empty((len(ex), I, d), np.float64),
    }
    tw = np.ascontiguousarray(routing["topk_w"], dtype=np.float32)
    getattr(lib, f"oracle_backward_experts_{acc}")(
        _p(sh), ctypes.c_int(dt), _p(xs[0]), _p(dys[0]), _p(wgs[0]), _p(wus[0]), _p(wds[0]),
        _p(tw), _p(routing["offsets"]), _p(routing["perm"]),
        ctypes.c_int(1 if round_bf16 else 0), ctypes.c_int(len(ex)), _p(ex), _p(out["dw_gate"]),
        _p(out["dw_up"]), _p(out["dw_down"]))
    return out


def backward_tokens(shape: dict, x, dy, w_gate, w_up, w_down, routing: dict, tokens,
                    round_bf16: bool = True, acc: str = "f64") -> dict:
    lib = _load(acc)
    sh = _shape_arr(shape)
    d, k = int(shape["d"]), int(shape["k"])
    xs, dys, wgs, wus, wds = _in(x), _in(dy), _in(w_gate), _in(w_up), _in(w_down)
    dt = _same_dtype(xs, dys, wgs, wus, wds)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    out = {"dx": np.empty((len(tok), d), np.float64),
           "dtopk_w": np.empty((len(tok), k), np.float64)}
    tw = np.ascontiguousarray(routing["topk_w"], dtype=np.float32)
    ti = np.ascontiguousarray(routing["topk_idx"], dtype=np.int32)
    getattr(lib, f"oracle_backward_tokens_{acc}")(
        _p(sh), ctypes.c_int(dt), _p(xs[0]), _p(dys[0]), _p(wgs[0]), _p(wus[0]), _p(wds[0]),
        _p(ti), _p(tw), ctypes.c_int(1 if round_bf16 else 0), ctypes.c_int(len(tok)), _p(tok),
        _p(out["dx"]), _p(out["dtopk_w"]))
    return out


def bf16_bits(t) -> np.ndarray:
    """torch bf16 tensor (CPU) -> numpy uint16 bit patterns (no arithmetic)."""
    import torch
    assert t.dtype == torch.bfloat16
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def round_bf16(values, acc: str = "f64") -> np.ndarray:
    """The oracle's bf16 rounding rule applied to float64 values (for its pin)."""
    lib = _load(acc)
    a = np.ascontiguousarray(values, dtype=np.float64)
    out = np.empty_like(a)
    getattr(lib, f"oracle_round_bf16_{acc}")(_p(a), _p(out), ctypes.c_int64(a.size))
    return out
