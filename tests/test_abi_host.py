"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]


@pytest.fixture(scope="module")
def lib():
    from paper_2604_19241_amd import binding
    if not binding.LIB_PATH.exists():
        from paper_2604_19241_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = (ROOT / "include" / "uniep_moe.h").read_text()
    names = set(re.findall(r"^(?:int|const char\*)\s+(moe_\w+)\s*\(", header, flags=re.M))
    assert {"moe_route", "moe_fused_forward", "moe_fused_backward", "moe_route_backward",
            "moe_workspace_bytes", "moe_saved_layout", "moe_device_status", "moe_status_string",
            "moe_calibration_copy", "moe_global_map"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    from paper_2604_19241_amd import binding as b
    for code in (0, -1, -2, -3, -4, -5):
        assert b.status_string(code)
    assert b.status_string(-99) == "unknown status"


def test_struct_sizes_match_header(lib):
    from paper_2604_19241_amd import binding as b
    assert ctypes.sizeof(b.MoEShape) == 28
    assert ctypes.sizeof(b.MoEOpts) == 32
    assert ctypes.sizeof(b.MoERoutingC) == 48
    assert ctypes.sizeof(b.MoEGlobalMapC) == 56


@pytest.mark.parametrize("kw", [
    dict(T=8, d=100, E=8, k=2, I=64),        # d not a multiple of 64
    dict(T=8, d=64, E=8, k=2, I=96),         # I not a multiple of 64
    dict(T=8, d=64, E=4, k=5, I=64),         # k > E
    dict(T=8, d=64, E=8, k=17, I=64),        # k > 16
    dict(T=8, d=64, E=2048, k=2, I=64),      # E > 1024
    dict(T=8, d=64, E=8, k=2, I=64, e_start=6, e_count=3),   # window past E
    dict(T=8, d=64, E=8, k=2, I=64, e_start=0, e_count=0),
    dict(T=-1, d=64, E=8, k=2, I=64),
])
def test_bad_shapes_are_rejected(lib, kw):
    from paper_2604_19241_amd import binding as b
    s = b.make_shape(**kw)
    sizes = [ctypes.c_size_t(0) for _ in range(4)]
    rc = lib.moe_workspace_bytes(ctypes.byref(s), *[ctypes.byref(v) for v in sizes])
    assert rc == b.MOE_ERR_SHAPE
    rc = lib.moe_route(ctypes.byref(s), None, None, None, ctypes.c_size_t(0), None)
    assert rc == b.MOE_ERR_SHAPE


def test_workspace_sizes_and_layout(lib):
    from paper_2604_19241_amd import binding as b
    s = b.make_shape(T=256, d=512, E=8, k=2, I=1024)
    w = b.moe_workspace_bytes(s)
    A = 256 * 2
    assert w["saved"] >= A * (2 * 1024 + 1024 + 512) * 2
    assert w["fwd"] >= A * (1024 + 512) * 2
    assert w["route"] >= 256 and w["bwd"] >= 256
    L = b.moe_saved_layout(s)
    assert L["gu"] == 0 and L["h"] >= A * 2048 * 2 and L["o"] >= L["h"] + A * 1024 * 2
    assert all(v % 256 == 0 for v in L.values())


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(lib):
    from paper_2604_19241_amd import binding as b
    s = b.make_shape(T=8, d=64, E=8, k=2, I=64)
    fake = ctypes.c_void_p(0x1000)            # never dereferenced: checks come first
    r_ok = b.MoERoutingC(*([0x1000] * 6))
    r_null = b.MoERoutingC(0x1000, 0, 0x1000, 0x1000, 0x1000, 0x1000)
    big = ctypes.c_size_t(1 << 40)
    # routing struct with a null member
    assert lib.moe_route(ctypes.byref(s), fake, ctypes.byref(r_null), fake, big, None) == b.MOE_ERR_ARG
    # workspace too small
    assert lib.moe_route(ctypes.byref(s), fake, ctypes.byref(r_ok), fake, ctypes.c_size_t(8), None) \
        == b.MOE_ERR_WORKSPACE
    # forward: null weights, misaligned x, small workspace, bad option
    args = dict(x=fake, wg=fake, wu=fake, wd=fake, y=fake, saved=None, ws=fake)

    def fwd(x=fake, wg=fake, wu=fake, wd=fake, y=fake, saved=None, ws=fake, nbytes=big, opts=None):
        return lib.moe_fused_forward(ctypes.byref(s), x, wg, wu, wd, ctypes.byref(r_ok), y, saved,
                                     ws, nbytes, opts, None)

    assert fwd(wg=None) == b.MOE_ERR_ARG
    assert fwd(x=ctypes.c_void_p(0x1002)) == b.MOE_ERR_ARG
    assert fwd(ws=ctypes.c_void_p(0x1010)) == b.MOE_ERR_ARG
    assert fwd(nbytes=ctypes.c_size_t(16)) == b.MOE_ERR_WORKSPACE
    bad = b.make_opts(schedule=7)
    assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    bad = b.make_opts(tile_rows=64)
    assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    bad = b.make_opts(skip_tail=2)
    assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    bad = b.make_opts(dw_accumulate=2)
    assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    for split in (-64, 100, 128, 300):   # negative, not a multiple of 64, below 256
        bad = b.make_opts(dw_split_rows=split)
        assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    bad = b.make_opts()
    bad.reserved[0] = 1
    assert fwd(opts=ctypes.byref(bad)) == b.MOE_ERR_ARG
    assert ctypes.sizeof(b.MoEOpts) == 32
    # backward needs the stash
    rc = lib.moe_fused_backward(ctypes.byref(s), fake, fake, fake, fake, fake, ctypes.byref(r_ok),
                                None, fake, fake, fake, fake, None, fake, big, None, None)
    assert rc == b.MOE_ERR_ARG
    # split weight-gradient reductions need the larger workspace that their own query reports
    stash = ctypes.c_void_p(0x2000)
    split = b.make_opts(dw_split_rows=256)
    assert b.moe_backward_workspace_bytes(s, split) == b.moe_workspace_bytes(s)["bwd"]   # 16 rows: nothing to split
    s = b.make_shape(T=512, d=64, E=8, k=2, I=64)
    base = b.moe_workspace_bytes(s)["bwd"]
    need = b.moe_backward_workspace_bytes(s, split)
    assert need > base and b.moe_backward_workspace_bytes(s, None) == base
    rc = lib.moe_fused_backward(ctypes.byref(s), fake, fake, fake, fake, fake, ctypes.byref(r_ok),
                                stash, fake, fake, fake, fake, None, fake, ctypes.c_size_t(base),
                                ctypes.byref(split), None)
    assert rc == b.MOE_ERR_WORKSPACE


def test_calibration_copy_rejects_bad_arguments(lib):
    from paper_2604_19241_amd import binding as b
    lib.moe_calibration_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert lib.moe_calibration_copy(None, 256, 256, None) == b.MOE_ERR_ARG       # NULL destination
    assert lib.moe_calibration_copy(256, None, 256, None) == b.MOE_ERR_ARG       # NULL source
    assert lib.moe_calibration_copy(256, 264, 256, None) == b.MOE_ERR_ARG        # misaligned source
    assert lib.moe_calibration_copy(256, 512, 100, None) == b.MOE_ERR_ARG        # size not a multiple of 16
    assert lib.moe_calibration_copy(256, 512, 0, None) == b.MOE_OK               # nothing to copy, nothing launched


def test_calibration_mfma_rejects_bad_arguments(lib):
    from paper_2604_19241_amd import binding as b
    lib.moe_calibration_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    ok = (256, 8, 10, 0x1000, 0x1000, 0x1000, None)
    for i, bad in ((0, 0), (1, 0), (1, 9), (2, 0), (3, None), (4, None), (5, None), (3, 0x1002), (5, 0x1004)):
        args = list(ok)
        args[i] = bad
        assert lib.moe_calibration_mfma(*args) == b.MOE_ERR_ARG, (i, bad)


def test_global_map_rejects_bad_arguments(lib):
    from paper_2604_19241_amd import binding as b
    lib.moe_global_map.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_size_t, ctypes.c_void_p]
    fake = 0x1000
    r = b.MoERoutingC(*([fake] * 6))
    g = b.MoEGlobalMapC(*([fake] * 7))

    def call(s, W=4, rank=1, routing=r, c_all=fake, out=g, ws=fake, nbytes=1 << 20):
        return lib.moe_global_map(ctypes.byref(s), W, rank, ctypes.byref(routing) if routing else None,
                                  c_all, ctypes.byref(out) if out else None, ws, nbytes, None)

    ok = b.make_shape(T=8, d=64, E=8, k=2, I=64)
    assert call(b.make_shape(T=8, d=64, E=8, k=2, I=64, e_start=0, e_count=4)) == b.MOE_ERR_SHAPE
    assert call(ok, W=3) == b.MOE_ERR_SHAPE            # E not a multiple of W
    assert call(ok, W=0) == b.MOE_ERR_SHAPE
    assert call(b.make_shape(T=8, d=64, E=128, k=2, I=64), W=128) == b.MOE_ERR_SHAPE   # W > 64
    assert call(ok, rank=4) == b.MOE_ERR_SHAPE
    assert call(ok, rank=-1) == b.MOE_ERR_SHAPE
    assert call(ok, c_all=None) == b.MOE_ERR_ARG
    assert call(ok, routing=None) == b.MOE_ERR_ARG
    assert call(ok, out=None) == b.MOE_ERR_ARG
    assert call(ok, ws=None) == b.MOE_ERR_ARG
    assert call(ok, c_all=0x1002) == b.MOE_ERR_ARG     # misaligned
    assert call(ok, out=b.MoEGlobalMapC(*([fake] * 5 + [0, fake]))) == b.MOE_ERR_ARG
    assert call(ok, nbytes=63) == b.MOE_ERR_WORKSPACE  # needs 8 * E bytes


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2604_19241_amd import binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", tmp_path / "nope.so")
    with pytest.raises(FileNotFoundError):
        b.load_library()
