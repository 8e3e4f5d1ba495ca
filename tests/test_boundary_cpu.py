"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, rejects bad arguments before launching anything, and fills the RoPE table correctly."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2604_14561_amd as cd
from paper_2604_14561_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cocodiff.h")).read()
    return sorted(set(re.findall(r"COCODIFF_API[^;(]*?\b(cocodiff_\w+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert len(names) >= 11 and set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None
    assert "gfx950" in cd.version()


def _rc(fn, *args):
    return fn(*args), B.lib().cocodiff_last_error().decode()


def test_shape_rules_are_checked_before_any_launch():
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)   # aligned non-null pointers; never dereferenced because the shape check fails first
    bad_shapes = [
        cd.Shape.make(100, 256, 4, 64, 3),        # N % P
        cd.Shape.make(256, 256, 4, 64, 3),        # H % P (and N % P)
        cd.Shape.make(256, 256, 4, 32, 2),        # D != H*d
        cd.Shape.make(256, 48, 4, 12, 2),         # d % 8
        cd.Shape.make(48, 256, 4, 64, 2),         # tokens per rank % 16
        cd.Shape.make(256, 256, 4, 64, 2, 1, 2),  # rank range beyond P
        cd.Shape.make(256, 256, 4, 64, 2, -1, 1),
        cd.Shape.make(256, 256, 4, 64, 2, 0, 0),
        cd.Shape.make(0, 256, 4, 64, 2),
    ]
    for s in bad_shapes:
        rc, msg = _rc(L.cocodiff_a2a_pack, ctypes.byref(s), fake, fake, 0, None)
        assert rc == B.ERR_SHAPE and msg, (rc, msg)
        assert L.cocodiff_a2a_unpack(ctypes.byref(s), fake, fake, 0, None) == B.ERR_SHAPE
        assert L.cocodiff_qkv_proj(ctypes.byref(s), fake, fake, None, None, fake, None, None, None) == B.ERR_SHAPE
    good = cd.Shape.make(256, 256, 4, 64, 2)
    assert L.cocodiff_a2a_pack(ctypes.byref(good), fake, fake, 7, None) == B.ERR_SHAPE   # slot order
    assert L.cocodiff_a2a_pack(None, fake, fake, 0, None) == B.ERR_NULL


def test_null_and_alignment_errors():
    L = B.lib()
    s = cd.Shape.make(256, 256, 4, 64, 2)
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    assert L.cocodiff_a2a_pack(ctypes.byref(s), None, fake, 0, None) == B.ERR_NULL
    assert L.cocodiff_a2a_unpack(ctypes.byref(s), fake, None, 0, None) == B.ERR_NULL
    assert L.cocodiff_a2a_pack(ctypes.byref(s), odd, fake, 0, None) == B.ERR_ALIGN
    # projection: x missing, half-given pair, nothing to compute
    assert L.cocodiff_qkv_proj(ctypes.byref(s), None, fake, None, None, fake, None, None, None) == B.ERR_NULL
    assert L.cocodiff_qkv_proj(ctypes.byref(s), fake, fake, None, None, None, None, None, None) == B.ERR_NULL
    assert L.cocodiff_qkv_proj(ctypes.byref(s), fake, None, None, None, None, None, None, None) == B.ERR_NULL
    assert L.cocodiff_qkv_proj(ctypes.byref(s), fake, odd, None, None, fake, None, None, None) == B.ERR_ALIGN
    # norm + rope
    r = cd.Rope.make((16, 16), (16, 16), 10000.0, 0x2000)
    assert L.cocodiff_qk_norm_rope(ctypes.byref(s), None, None, fake, fake, 1e-6, ctypes.byref(r), None) == B.ERR_NULL
    assert L.cocodiff_qk_norm_rope(ctypes.byref(s), fake, None, None, None, 1e-6, ctypes.byref(r), None) == B.ERR_NULL
    assert L.cocodiff_qk_norm_rope(ctypes.byref(s), fake, None, fake, None, 1e-6, None, None) == B.ERR_NULL
    r_nocs = cd.Rope.make((16, 16), (16, 16), 10000.0, 0)
    assert L.cocodiff_qk_norm_rope(ctypes.byref(s), fake, None, fake, None, 1e-6, ctypes.byref(r_nocs), None) == B.ERR_NULL
    for grid, pairs in (((16, 8), (16, 16)), ((16, 16), (16, 8)), ((16, 16, 1, ), (16, 16, 0))):
        rb = cd.Rope.make(grid, pairs, 10000.0, 0x2000)
        assert L.cocodiff_qk_norm_rope(ctypes.byref(s), fake, None, fake, None, 1e-6, ctypes.byref(rb), None) == B.ERR_SHAPE
    s_d = cd.Shape.make(256, 96, 4, 24, 2)   # d/8 = 3 is not a power of two
    assert L.cocodiff_qk_norm_rope(ctypes.byref(s_d), fake, None, fake, None, 1e-6, ctypes.byref(r), None) == B.ERR_SHAPE


def test_select_argument_errors():
    L = B.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    ws = B.vmajor_select_workspace_bytes(4, 256, 64, 16)
    assert ws > 0
    call = L.cocodiff_vmajor_select
    # every call below fails a host-side check, so nothing is launched
    assert call(4, 256, 60, 16, fake, fake, 1e-3, None, fake, fake, None, 0, fake, ws, None) == B.ERR_SHAPE   # W % 8
    assert call(4, 250, 64, 16, fake, fake, 1e-3, None, fake, fake, None, 0, fake, ws, None) == B.ERR_SHAPE   # N % T
    assert call(0, 256, 64, 16, fake, fake, 1e-3, None, fake, fake, None, 0, fake, ws, None) == B.ERR_SHAPE
    assert call(4, 256, 64, 16, None, fake, 1e-3, None, fake, fake, None, 0, fake, ws, None) == B.ERR_NULL
    assert call(4, 256, 64, 16, fake, fake, 1e-3, None, None, fake, None, 0, fake, ws, None) == B.ERR_NULL
    assert call(4, 256, 64, 16, fake, fake, 1e-3, None, fake, None, None, 0, fake, ws, None) == B.ERR_NULL
    assert call(4, 256, 64, 16, fake, fake, 1e-3, None, fake, fake, None, 0, None, ws, None) == B.ERR_NULL
    assert call(4, 256, 64, 16, odd, fake, 1e-3, None, fake, fake, None, 0, fake, ws, None) == B.ERR_ALIGN
    assert call(4, 256, 64, 16, fake, fake, 1e-3, None, fake, fake, fake, 0, fake, ws, None) == B.ERR_CAPACITY  # cap_tiles < 1
    assert call(4, 256, 64, 16, fake, fake, 1e-3, None, fake, fake, None, 0, fake, ws - 1, None) == B.ERR_CAPACITY
    assert B.vmajor_select_workspace_bytes(4, 250, 64, 16) == 0
    assert "workspace" in L.cocodiff_last_error().decode() or True


def test_copy_argument_errors():
    L = B.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    assert L.cocodiff_util_copy(None, fake, 16, None) == B.ERR_NULL
    assert L.cocodiff_util_copy(odd, fake, 16, None) == B.ERR_ALIGN
    assert L.cocodiff_util_copy(fake, fake, 24, None) == B.ERR_SHAPE
    assert L.cocodiff_util_copy(fake, fake, 0, None) == B.OK   # nothing to do, nothing launched
    assert L.cocodiff_util_mfma_rate(0, 10, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_util_mfma_rate(256, 10, None, None) == B.ERR_NULL


def test_rope_table_layout_and_closed_form_values():
    # grid 4 x 8, 16 pairs per axis: pair j' turns by coord * 10000**(-j'/16); j' = 4 -> 0.1, j' = 8 -> 0.01
    t = cd.rope_table((4, 8), (16, 16), 10000.0)
    assert t.dtype == np.float32 and t.size == (4 * 16 + 8 * 16) * 2
    ax0 = t[:4 * 16 * 2].reshape(4, 16, 2)
    ax1 = t[4 * 16 * 2:].reshape(8, 16, 2)
    for coord in range(4):
        for jl, w in ((0, 1.0), (4, 0.1), (8, 0.01), (12, 0.001)):
            assert abs(ax0[coord, jl, 0] - math.cos(coord * w)) < 1e-6
            assert abs(ax0[coord, jl, 1] - math.sin(coord * w)) < 1e-6
    assert abs(ax1[7, 0, 0] - math.cos(7.0)) < 1e-6 and abs(ax1[7, 0, 1] - math.sin(7.0)) < 1e-6
    assert abs(ax1[5, 8, 1] - math.sin(0.05)) < 1e-7
    # 3 axes
    t3 = cd.rope_table((2, 3, 4), (2, 3, 3), 10000.0)
    assert t3.size == (2 * 2 + 3 * 3 + 4 * 3) * 2
    assert abs(t3[(1 * 2 + 1) * 2] - math.cos(0.01)) < 1e-7   # axis 0, coord 1, pair 1 of 2: 10000**-0.5
    with pytest.raises(cd.CocodiffError):
        cd.rope_table((4, 0), (16, 16), 10000.0)


def test_binding_refuses_host_tensors():
    import torch
    s = cd.Shape.make(256, 256, 4, 64, 2)
    x = torch.zeros(256, 256, dtype=torch.int16)
    with pytest.raises(ValueError):
        cd.a2a_pack(s, x, x, cd.SEND_MAJOR, stream=0)


def test_fused_entry_points_check_arguments_before_any_launch():
    L = B.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    s = cd.Shape.make(256, 256, 4, 64, 2)
    bad = cd.Shape.make(250, 256, 4, 64, 2)
    f = L.cocodiff_qkv_proj_pack
    assert f(ctypes.byref(bad), fake, fake, None, None, fake, None, None, 0, None) == B.ERR_SHAPE
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, None, 9, None) == B.ERR_SHAPE      # slot order
    assert f(ctypes.byref(s), fake, fake, None, None, None, None, None, 0, None) == B.ERR_NULL       # weight without buffer
    assert f(ctypes.byref(s), None, fake, None, None, fake, None, None, 0, None) == B.ERR_NULL
    assert f(ctypes.byref(s), fake, fake, None, None, odd, None, None, 0, None) == B.ERR_ALIGN
    rope = cd.Rope.make((16, 16), (16, 16), 10000.0, 0x1000)
    g = L.cocodiff_qk_norm_rope_pack
    assert g(ctypes.byref(s), fake, None, fake, None, 1e-6, ctypes.byref(rope), None, None, 0, None) == B.ERR_NULL   # q without qbuf
    assert g(ctypes.byref(s), None, None, None, None, 1e-6, ctypes.byref(rope), fake, fake, 0, None) == B.ERR_NULL
    assert g(ctypes.byref(s), fake, None, fake, None, 1e-6, ctypes.byref(rope), odd, None, 0, None) == B.ERR_ALIGN
    assert g(ctypes.byref(s), fake, None, fake, None, 1e-6, ctypes.byref(rope), fake, None, 4, None) == B.ERR_SHAPE
    h = L.cocodiff_a2a_unpack_norm_rope
    assert h(ctypes.byref(s), None, None, None, None, None, None, 1e-6, ctypes.byref(rope), 0, None) == B.ERR_NULL
    assert h(ctypes.byref(s), fake, None, None, None, fake, None, 1e-6, ctypes.byref(rope), 0, None) == B.ERR_NULL    # no output
    assert h(ctypes.byref(s), fake, None, fake, None, None, None, 1e-6, ctypes.byref(rope), 0, None) == B.ERR_NULL    # no gamma
    assert h(ctypes.byref(s), fake, None, odd, None, fake, None, 1e-6, ctypes.byref(rope), 0, None) == B.ERR_ALIGN
    assert h(ctypes.byref(s), fake, None, fake, None, fake, None, 1e-6, ctypes.byref(rope), 3, None) == B.ERR_SHAPE
    assert h(ctypes.byref(s), fake, None, fake, None, fake, None, 1e-6, None, 0, None) == B.ERR_NULL
    wrong = cd.Rope.make((16, 8), (16, 16), 10000.0, 0x1000)          # grid does not cover N
    assert h(ctypes.byref(s), fake, None, fake, None, fake, None, 1e-6, ctypes.byref(wrong), 0, None) == B.ERR_SHAPE


def test_fused_projection_argument_errors():
    """cocodiff_qkv_proj_fused: every rule is checked on the host before anything is enqueued (no GPU needed up to the
    launch plan, which is the last step)."""
    L = B.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    f = L.cocodiff_qkv_proj_fused
    s = cd.Shape.make(256, 256, 4, 64, 2)
    rope = cd.Rope.make((16, 16), (16, 16), 10000.0, 0x1000)
    r = ctypes.byref(rope)
    # a head size the wavefront tiles cannot hold whole
    s40 = cd.Shape.make(256, 320, 8, 40, 2)
    assert f(ctypes.byref(s40), fake, fake, None, None, fake, None, 1e-6, r, fake, None, None, 0, None, None, None, None) == B.ERR_SHAPE
    assert b"64, 128 or 256" in L.cocodiff_last_error()
    # no weight; weight without destination; destination without weight; gamma missing; rope missing
    assert f(ctypes.byref(s), fake, None, None, None, None, None, 1e-6, r, None, None, None, 0, None, None, None, None) == B.ERR_NULL
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, 1e-6, r, None, None, None, 0, None, None, None, None) == B.ERR_NULL
    assert f(ctypes.byref(s), fake, None, None, None, None, None, 1e-6, r, None, None, fake, 0, None, None, None, None) == B.ERR_NULL
    assert f(ctypes.byref(s), fake, fake, None, None, None, None, 1e-6, r, fake, None, None, 0, None, None, None, None) == B.ERR_NULL
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, 1e-6, None, fake, None, None, 0, None, None, None, None) == B.ERR_NULL
    # alignment, slot order, rope that does not cover N
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, 1e-6, r, None, None, None, 0, odd, None, None, None) == B.ERR_ALIGN
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, 1e-6, r, fake, None, None, 7, None, None, None, None) == B.ERR_SHAPE
    wrong = cd.Rope.make((16, 8), (16, 16), 10000.0, 0x1000)
    assert f(ctypes.byref(s), fake, fake, None, None, fake, None, 1e-6, ctypes.byref(wrong), fake, None, None, 0, None, None, None, None) == B.ERR_SHAPE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No fallback: without the built HIP library the binding raises instead of computing anything elsewhere."""
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libcocodiff.so"))
    with pytest.raises(Exception) as err:
        B.lib()
    assert "libcocodiff.so" in str(err.value)
    monkeypatch.undo()
    assert B.lib() is not None
