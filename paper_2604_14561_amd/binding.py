"""Thin ctypes binding over libcocodiff.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  Tensors are PyTorch
CUDA(ROCm) tensors used for device memory; only their ``data_ptr()`` crosses the
boundary.  There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcocodiff.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_CAPACITY, ERR_HIP = -1, -2, -3, -4, -5
SEND_MAJOR, RECV_MAJOR = 0, 1

EXPORTS = (
    "cocodiff_qkv_proj", "cocodiff_qk_norm_rope", "cocodiff_qkv_proj_pack", "cocodiff_qkv_proj_hs", "cocodiff_qkv_proj_fused", "cocodiff_qkv_proj_fused_select",
    "cocodiff_qkv_proj_fused_select_workspace_bytes", "cocodiff_qk_norm_rope_pack",
    "cocodiff_a2a_unpack_select", "cocodiff_a2a_unpack_norm_rope", "cocodiff_a2a_pack", "cocodiff_a2a_unpack",
    "cocodiff_vmajor_select", "cocodiff_vmajor_select_static", "cocodiff_vmajor_select_workspace_bytes", "cocodiff_vmajor_gather",
    "cocodiff_vmajor_scatter", "cocodiff_vmajor_token_metric", "cocodiff_vmajor_topk", "cocodiff_cache_active_count",
    "cocodiff_a2a_pack_hs", "cocodiff_a2a_unpack_seq", "cocodiff_rope_table_bytes",
    "cocodiff_rope_table_fill", "cocodiff_qkv_proj_plan", "cocodiff_util_copy", "cocodiff_util_mfma_rate", "cocodiff_version", "cocodiff_last_error",
)


class CocodiffError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"cocodiff error {code}: {message}")
        self.code = code
        self.message = message


class Shape(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("D", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
                ("P", ctypes.c_int32), ("rank_begin", ctypes.c_int32), ("rank_count", ctypes.c_int32)]

    @classmethod
    def make(cls, N: int, D: int, H: int, d: int, P: int, rank_begin: int = 0, rank_count: Optional[int] = None):
        return cls(N, D, H, d, P, rank_begin, P if rank_count is None else rank_count)


class Rope(ctypes.Structure):
    _fields_ = [("n_axes", ctypes.c_int32), ("grid", ctypes.c_int32 * 3), ("pairs", ctypes.c_int32 * 3),
                ("theta", ctypes.c_float), ("cs", ctypes.c_void_p)]

    @classmethod
    def make(cls, grid: Sequence[int], pairs: Sequence[int], theta: float, cs_ptr: int = 0):
        g = (ctypes.c_int32 * 3)(*(list(grid) + [0] * (3 - len(grid))))
        p = (ctypes.c_int32 * 3)(*(list(pairs) + [0] * (3 - len(pairs))))
        return cls(len(grid), g, p, float(theta), cs_ptr or None)


_lib = None


def lib() -> ctypes.CDLL:
    """Load libcocodiff.so (built in-tree by ``paper_2604_14561_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_14561_amd.build` "
                "(there is no fallback path)")
        # PyTorch brings its own HIP runtime; the tensors this binding is handed live in that runtime, so it has to be
        # the one this library binds to as well: load torch first, whatever the caller's import order was
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, i32, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        sp, rp = ctypes.POINTER(Shape), ctypes.POINTER(Rope)
        L.cocodiff_qkv_proj.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.cocodiff_qk_norm_rope.argtypes = [sp, vp, vp, vp, vp, f32, rp, vp]
        L.cocodiff_qkv_proj_hs.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.cocodiff_qkv_proj_hs.restype = ci
        L.cocodiff_a2a_pack.argtypes = [sp, vp, vp, ci, vp]
        L.cocodiff_a2a_unpack.argtypes = [sp, vp, vp, ci, vp]
        L.cocodiff_vmajor_select.argtypes = [i32, i32, i32, i32, vp, vp, f32, vp, vp, vp, vp, i32, vp, sz, vp]
        L.cocodiff_vmajor_select_static.argtypes = [i32, i32, i32, i32, vp, vp, f32, vp, vp, vp, vp, i32, vp]
        L.cocodiff_vmajor_select_static.restype = ci
        L.cocodiff_vmajor_gather.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
        L.cocodiff_vmajor_scatter.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
        L.cocodiff_vmajor_token_metric.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        L.cocodiff_vmajor_topk.argtypes = [i32, i32, vp, i32, i32, vp, vp, vp]
        L.cocodiff_cache_active_count.argtypes = [i32, i32, i32, i32, i32]
        L.cocodiff_cache_active_count.restype = i32
        L.cocodiff_a2a_pack_hs.argtypes = [sp, vp, vp, ci, vp]
        L.cocodiff_a2a_unpack_seq.argtypes = [sp, vp, vp, ci, vp]
        L.cocodiff_vmajor_select_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.cocodiff_vmajor_select_workspace_bytes.restype = sz
        L.cocodiff_rope_table_bytes.argtypes = [rp]
        L.cocodiff_rope_table_bytes.restype = sz
        L.cocodiff_rope_table_fill.argtypes = [rp, vp]
        L.cocodiff_util_copy.argtypes = [vp, vp, sz, vp]
        L.cocodiff_qkv_proj_plan.argtypes = [sp, i32, i32, vp, vp, vp, vp]
        L.cocodiff_qkv_proj_fused.argtypes = [sp, vp, vp, vp, vp, vp, vp, f32, rp, vp, vp, vp, ci, vp, vp, vp, vp]
        L.cocodiff_qkv_proj_fused.restype = ci
        L.cocodiff_qkv_proj_fused_select.argtypes = [sp, vp, vp, vp, vp, vp, vp, f32, rp, vp, vp, vp, ci, vp, vp, vp,
                                                     vp, i32, f32, vp, vp, vp, vp, i32, vp, sz, vp]
        L.cocodiff_qkv_proj_fused_select.restype = ci
        L.cocodiff_qkv_proj_fused_select_workspace_bytes.argtypes = [sp, i32]
        L.cocodiff_qkv_proj_fused_select_workspace_bytes.restype = sz
        L.cocodiff_qkv_proj_plan.restype = ci
        L.cocodiff_version.restype = ctypes.c_char_p
        L.cocodiff_last_error.restype = ctypes.c_char_p
        L.cocodiff_util_mfma_rate.argtypes = [i32, i32, vp, vp]
        L.cocodiff_util_mfma_rate.restype = ctypes.c_int64
        L.cocodiff_a2a_unpack_select.argtypes = [sp, vp, ci, vp, vp, i32, f32, vp, vp, vp, vp, i32, vp, sz, vp]
        L.cocodiff_a2a_unpack_select.restype = ci
        L.cocodiff_a2a_unpack_norm_rope.argtypes = [sp, vp, vp, vp, vp, vp, vp, f32, rp, ci, vp]
        L.cocodiff_a2a_unpack_norm_rope.restype = ci
        L.cocodiff_qkv_proj_pack.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, ci, vp]
        L.cocodiff_qk_norm_rope_pack.argtypes = [sp, vp, vp, vp, vp, ctypes.c_float, rp, vp, vp, ci, vp]
        for name in ("cocodiff_qkv_proj", "cocodiff_qk_norm_rope", "cocodiff_qkv_proj_pack", "cocodiff_qkv_proj_hs", "cocodiff_qkv_proj_fused", "cocodiff_qk_norm_rope_pack", "cocodiff_a2a_pack", "cocodiff_a2a_unpack",
                     "cocodiff_vmajor_select", "cocodiff_vmajor_gather", "cocodiff_vmajor_scatter",
                     "cocodiff_vmajor_token_metric", "cocodiff_vmajor_topk",
                     "cocodiff_a2a_pack_hs", "cocodiff_a2a_unpack_seq", "cocodiff_rope_table_fill", "cocodiff_util_copy"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != OK:
        raise CocodiffError(rc, lib().cocodiff_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device pointer of a tensor (None passes NULL).  Integers pass through (raw pointers)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t or None
    if not t.is_cuda:
        raise ValueError("cocodiff tensors must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("cocodiff tensors must be contiguous")
    return t.data_ptr() or None


def _stream(stream) -> Optional[int]:
    """hipStream_t handle: a torch.cuda.Stream, a raw handle, or None for torch's current stream."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def version() -> str:
    return lib().cocodiff_version().decode()


def qkv_proj(shape: Shape, x, wq, wk, wv, q, k, v, stream=None) -> None:
    _check(lib().cocodiff_qkv_proj(ctypes.byref(shape), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv),
                                   _ptr(q), _ptr(k), _ptr(v), _stream(stream)))


def qk_norm_rope(shape: Shape, q, k, gamma_q, gamma_k, eps: float, rope: Rope, stream=None) -> None:
    _check(lib().cocodiff_qk_norm_rope(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(gamma_q), _ptr(gamma_k),
                                       float(eps), ctypes.byref(rope), _stream(stream)))


def qkv_proj_pack(shape: Shape, x, wq, wk, wv, qbuf, kbuf, vbuf, slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_qkv_proj_pack(ctypes.byref(shape), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv),
                                        _ptr(qbuf), _ptr(kbuf), _ptr(vbuf), int(slot_order), _stream(stream)))


def qkv_proj_hs(shape: Shape, x, wq, wk, wv, q_hs, k_hs, v_hs, stream=None) -> None:
    _check(lib().cocodiff_qkv_proj_hs(ctypes.byref(shape), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv),
                                      _ptr(q_hs), _ptr(k_hs), _ptr(v_hs), _stream(stream)))


def qk_norm_rope_pack(shape: Shape, q, k, gamma_q, gamma_k, eps: float, rope: Rope, qbuf, kbuf,
                      slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_qk_norm_rope_pack(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(gamma_q), _ptr(gamma_k),
                                            float(eps), ctypes.byref(rope), _ptr(qbuf), _ptr(kbuf), int(slot_order),
                                            _stream(stream)))


def a2a_unpack_norm_rope(shape: Shape, qbuf, kbuf, q_hs, k_hs, gamma_q, gamma_k, eps: float, rope: Rope,
                         slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_a2a_unpack_norm_rope(ctypes.byref(shape), _ptr(qbuf), _ptr(kbuf), _ptr(q_hs), _ptr(k_hs),
                                               _ptr(gamma_q), _ptr(gamma_k), float(eps), ctypes.byref(rope),
                                               int(slot_order), _stream(stream)))


def a2a_unpack_select(shape: Shape, vbuf, slot_order: int, v_hs, v_prev, tile_tokens: int, tau: float, flags, active_idx,
                      n_active, compact, cap_tiles: int, workspace, stream=None) -> None:
    _check(lib().cocodiff_a2a_unpack_select(ctypes.byref(shape), _ptr(vbuf), int(slot_order), _ptr(v_hs), _ptr(v_prev),
                                            int(tile_tokens), float(tau), _ptr(flags), _ptr(active_idx), _ptr(n_active),
                                            _ptr(compact), int(cap_tiles), _ptr(workspace),
                                            int(workspace.numel() * workspace.element_size()), _stream(stream)))


def a2a_pack(shape: Shape, x_seq, xbuf, slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_a2a_pack(ctypes.byref(shape), _ptr(x_seq), _ptr(xbuf), int(slot_order), _stream(stream)))


def a2a_unpack(shape: Shape, xbuf, x_hs, slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_a2a_unpack(ctypes.byref(shape), _ptr(xbuf), _ptr(x_hs), int(slot_order), _stream(stream)))


def vmajor_select_workspace_bytes(S: int, N: int, W: int, tile_tokens: int = 16) -> int:
    return int(lib().cocodiff_vmajor_select_workspace_bytes(S, N, W, tile_tokens))


def vmajor_select(S: int, N: int, W: int, tile_tokens: int, v_cur, v_prev, tau: float, flags, active_idx,
                  n_active, compact, cap_tiles: int, workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()
    _check(lib().cocodiff_vmajor_select(S, N, W, tile_tokens, _ptr(v_cur), _ptr(v_prev), float(tau), _ptr(flags),
                                        _ptr(active_idx), _ptr(n_active), _ptr(compact), int(cap_tiles),
                                        _ptr(workspace), int(workspace_bytes), _stream(stream)))


def vmajor_select_static(S: int, N: int, W: int, tile_tokens: int, v_cur, v_prev, tau: float, flags, active_idx,
                         n_active, compact, cap_tiles: int, stream=None) -> None:
    """vmajor_select without a workspace: the flag words live in an array the library owns on the GPU."""
    _check(lib().cocodiff_vmajor_select_static(S, N, W, tile_tokens, _ptr(v_cur), _ptr(v_prev), float(tau), _ptr(flags),
                                               _ptr(active_idx), _ptr(n_active), _ptr(compact), int(cap_tiles),
                                               _stream(stream)))


def vmajor_gather(S: int, N: int, W: int, tile_tokens: int, x, active_idx, n_active, compact, cap_tiles: int, stream=None) -> None:
    _check(lib().cocodiff_vmajor_gather(S, N, W, tile_tokens, _ptr(x), _ptr(active_idx), _ptr(n_active), _ptr(compact),
                                        int(cap_tiles), _stream(stream)))


def vmajor_scatter(S: int, N: int, W: int, tile_tokens: int, compact, active_idx, n_active, cache, cap_tiles: int, stream=None) -> None:
    _check(lib().cocodiff_vmajor_scatter(S, N, W, tile_tokens, _ptr(compact), _ptr(active_idx), _ptr(n_active), _ptr(cache),
                                         int(cap_tiles), _stream(stream)))


def vmajor_token_metric(S: int, N: int, W: int, v_cur, v_prev, metric, stream=None) -> None:
    _check(lib().cocodiff_vmajor_token_metric(S, N, W, _ptr(v_cur), _ptr(v_prev), _ptr(metric), _stream(stream)))


def vmajor_topk(n_seg: int, N: int, metric, n_keep: int, active_idx, n_active, stream=None, global_ids: bool = False) -> None:
    _check(lib().cocodiff_vmajor_topk(int(n_seg), int(N), _ptr(metric), int(n_keep), int(bool(global_ids)),
                                      _ptr(active_idx), _ptr(n_active), _stream(stream)))


def cache_active_count(step: int, n_steps: int, warmup: int, sync_every: int, n_tokens: int) -> int:
    return int(lib().cocodiff_cache_active_count(step, n_steps, warmup, sync_every, n_tokens))


def a2a_pack_hs(shape: Shape, y_hs, xbuf, slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_a2a_pack_hs(ctypes.byref(shape), _ptr(y_hs), _ptr(xbuf), int(slot_order), _stream(stream)))


def a2a_unpack_seq(shape: Shape, xbuf, y_seq, slot_order: int = SEND_MAJOR, stream=None) -> None:
    _check(lib().cocodiff_a2a_unpack_seq(ctypes.byref(shape), _ptr(xbuf), _ptr(y_seq), int(slot_order), _stream(stream)))


def rope_table(grid: Sequence[int], pairs: Sequence[int], theta: float) -> np.ndarray:
    """Host cos/sin table (fp32) in the layout ``Rope.cs`` expects; upload it and pass its device pointer."""
    r = Rope.make(grid, pairs, theta)
    nbytes = int(lib().cocodiff_rope_table_bytes(ctypes.byref(r)))
    if nbytes == 0:
        raise CocodiffError(ERR_SHAPE, lib().cocodiff_last_error().decode())
    out = np.empty(nbytes // 4, dtype=np.float32)
    _check(lib().cocodiff_rope_table_fill(ctypes.byref(r), out.ctypes.data_as(ctypes.c_void_p)))
    return out


def qkv_proj_fused(shape: Shape, x, wq, wk, wv, gamma_q, gamma_k, eps: float, rope: Optional[Rope], qbuf, kbuf, vbuf,
                   slot_order: int, q_hs, k_hs, v_hs, stream=None) -> None:
    _check(lib().cocodiff_qkv_proj_fused(ctypes.byref(shape), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(gamma_q), _ptr(gamma_k),
                                         float(eps), ctypes.byref(rope) if rope is not None else None, _ptr(qbuf), _ptr(kbuf),
                                         _ptr(vbuf), int(slot_order), _ptr(q_hs), _ptr(k_hs), _ptr(v_hs), _stream(stream)))


def qkv_proj_fused_select_workspace_bytes(shape: Shape, tile_tokens: int = 16) -> int:
    return int(lib().cocodiff_qkv_proj_fused_select_workspace_bytes(ctypes.byref(shape), int(tile_tokens)))


def qkv_proj_fused_select(shape: Shape, x, wq, wk, wv, gamma_q, gamma_k, eps: float, rope: Optional[Rope], qbuf, kbuf, vbuf,
                          slot_order: int, q_hs, k_hs, v_hs, v_prev, tile_tokens: int, tau: float, flags, active_idx, n_active,
                          compact, cap_tiles: int, workspace, stream=None) -> None:
    _check(lib().cocodiff_qkv_proj_fused_select(
        ctypes.byref(shape), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(gamma_q), _ptr(gamma_k), float(eps),
        ctypes.byref(rope) if rope is not None else None, _ptr(qbuf), _ptr(kbuf), _ptr(vbuf), int(slot_order), _ptr(q_hs),
        _ptr(k_hs), _ptr(v_hs), _ptr(v_prev), int(tile_tokens), float(tau), _ptr(flags), _ptr(active_idx), _ptr(n_active),
        _ptr(compact), int(cap_tiles), _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream(stream)))


def qkv_proj_plan(shape: Shape, n_tensors: int, whole_heads: bool = False) -> dict:
    """Tile shape and workgroup count the projection takes for this shape and number of weights per launch
    (whole_heads: the choice of qkv_proj_fused)."""
    out = [ctypes.c_int32(0) for _ in range(4)]
    _check(lib().cocodiff_qkv_proj_plan(ctypes.byref(shape), int(n_tensors), int(bool(whole_heads)), *(ctypes.byref(o) for o in out)))
    return {"tile_tokens": out[0].value, "tile_features": out[1].value, "n_tiles": out[2].value, "compute_units": out[3].value}


def util_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().cocodiff_util_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)))


def util_mfma_rate(blocks: int, iters: int, sink, stream=None) -> int:
    """Launch the register-only matrix-core loop; returns the launch's floating-point operation count."""
    flops = int(lib().cocodiff_util_mfma_rate(int(blocks), int(iters), _ptr(sink), _stream(stream)))
    if flops < 0:
        _check(flops)
    return flops
