"""CPU oracle (TEST INFRASTRUCTURE ONLY): the plain definition of every step of the path.

Floating-point steps are the definition written out in fp64 with numpy; the
matrix product uses numpy's fp64 ``matmul`` as a library step.  Index steps call
the explicit loops of ``loops.c``.  Inputs are bf16 bit patterns (uint16), the
very patterns the GPU library receives; they are widened exactly.

Nothing here imports, links or reads the HIP library, and nothing in the
product imports this package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_loops.so")
_lib = None

SEND_MAJOR = 0
RECV_MAJOR = 1


def build_c(force: bool = False) -> str:
    """Compile ``loops.c`` with gcc into ``liboracle_loops.so`` beside it."""
    src = os.path.join(_HERE, "loops.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _SO, src, "-lm"])
    return _SO


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_c())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.oracle_a2a_pack.argtypes = [u16p, u16p, ci, ci, ci, ci, ci, ci, ci]
        lib.oracle_a2a_pack.restype = None
        lib.oracle_a2a_exchange.argtypes = [u16p, u16p, ci, ci, ci, ci]
        lib.oracle_a2a_exchange.restype = None
        lib.oracle_a2a_unpack.argtypes = [u16p, u16p, ci, ci, ci, ci, ci, ci, ci]
        lib.oracle_a2a_unpack.restype = None
        lib.oracle_vmajor_select.argtypes = [ci, ci, ci, ci, u16p, u16p, ctypes.c_float, i32p, i32p, u16p, ci]
        lib.oracle_vmajor_select.restype = ci
        lib.oracle_vmajor_gather.argtypes = [ci, ci, ci, ci, u16p, i32p, ci, u16p, ci]
        lib.oracle_vmajor_gather.restype = None
        lib.oracle_vmajor_scatter.argtypes = [ci, ci, ci, ci, u16p, i32p, ci, u16p, ci]
        lib.oracle_vmajor_scatter.restype = None
        lib.oracle_a2a_pack_hs.argtypes = [u16p, u16p, ci, ci, ci, ci, ci, ci, ci]
        lib.oracle_a2a_pack_hs.restype = None
        lib.oracle_a2a_unpack_seq.argtypes = [u16p, u16p, ci, ci, ci, ci, ci, ci, ci]
        lib.oracle_a2a_unpack_seq.restype = None
        lib.oracle_omp_max_threads.argtypes = []
        lib.oracle_omp_max_threads.restype = ci
        _lib = lib
    return _lib


def omp_max_threads() -> int:
    """Threads the OpenMP index loops of ``loops.c`` run on."""
    return int(_c().oracle_omp_max_threads())


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _i32(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):  # signalling-NaN patterns widen to NaN without a warning
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------------------
# Projection (Section II-B: q_i = h_i W_Q, k_i = h_i W_K, v_i = h_i W_V)
# ---------------------------------------------------------------------------

def qkv_proj(x_bits: np.ndarray, w_bits: np.ndarray) -> np.ndarray:
    """Y[n][o] = sum_k X[n][k] * W[o][k] in fp64; W is stored output-major ([D_out][D_in]), no bias."""
    return np.matmul(widen(x_bits), widen(w_bits).T)


# ---------------------------------------------------------------------------
# Q/K normalisation and rotary embedding (Section II-B; RMSNorm per Section III-C)
# ---------------------------------------------------------------------------

def rms_norm(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm over the last axis (one attention head of one token): x / sqrt(mean(x^2) + eps) * gamma."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gamma


def token_coords(token_ids: np.ndarray, grid: Sequence[int]) -> np.ndarray:
    """Grid coordinates of global token indices; row-major, last axis fastest.  Returns [n][n_axes]."""
    token_ids = np.asarray(token_ids, dtype=np.int64)
    coords = np.empty((token_ids.shape[0], len(grid)), dtype=np.int64)
    rem = token_ids.copy()
    for a in range(len(grid) - 1, -1, -1):
        coords[:, a] = rem % grid[a]
        rem //= grid[a]
    return coords


def rope_rotate(y: np.ndarray, token_ids: np.ndarray, grid: Sequence[int], pairs: Sequence[int],
                theta: float) -> np.ndarray:
    """Axial rotary embedding on [n][H][d] (fp64).

    Adjacent elements (2j, 2j+1) form pair j.  The first pairs[0] pairs belong to grid
    axis 0, the next pairs[1] to axis 1, and so on.  Pair j with local index j' on axis a
    is rotated by the angle coord_a * theta**(-j'/pairs[a]).
    """
    n, H, d = y.shape
    assert sum(pairs) == d // 2 and len(pairs) == len(grid)
    coords = token_coords(token_ids, grid)
    phi = np.empty((n, d // 2), dtype=np.float64)
    j0 = 0
    for a, pa in enumerate(pairs):
        jl = np.arange(pa, dtype=np.float64)
        omega = np.power(float(theta), -jl / float(pa))
        phi[:, j0:j0 + pa] = coords[:, a:a + 1].astype(np.float64) * omega[None, :]
        j0 += pa
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    even = y[..., 0::2]
    odd = y[..., 1::2]
    out = np.empty_like(y)
    out[..., 0::2] = even * c - odd * s
    out[..., 1::2] = even * s + odd * c
    return out


def qk_norm_rope(x_bits: np.ndarray, token_ids: np.ndarray, gamma_bits: np.ndarray, eps: float,
                 grid: Sequence[int], pairs: Sequence[int], theta: float) -> np.ndarray:
    """RMSNorm per (token, head) then axial RoPE at the token's grid position, all in fp64.

    x_bits: [n][H][d] bf16 bits of the rows whose global token indices are ``token_ids``.
    """
    x = widen(x_bits)
    y = rms_norm(x, widen(gamma_bits), float(eps))
    return rope_rotate(y, token_ids, grid, pairs, theta)


# ---------------------------------------------------------------------------
# Ulysses all-to-all #1 as pack / exchange / unpack (Section II-A)
# ---------------------------------------------------------------------------

def a2a_pack(x_bits: np.ndarray, P: int, slot_order: int = SEND_MAJOR, rank_begin: int = 0,
             rank_count: Optional[int] = None, out: Optional[np.ndarray] = None) -> np.ndarray:
    """[N][H][d] -> exchange buffer [P*P][Ns][Hp][d]; only source ranks in the range are written."""
    N, H, d = x_bits.shape
    rank_count = P if rank_count is None else rank_count
    if out is None:
        out = np.zeros((P * P, N // P, H // P, d), dtype=np.uint16)
    _c().oracle_a2a_pack(_u16(x_bits), _u16(out), N, H, d, P, rank_begin, rank_count, slot_order)
    return out


def a2a_exchange(send_major: np.ndarray, N: int, H: int, d: int, P: int) -> np.ndarray:
    """Move every chunk from slot r*P+p to slot p*P+r."""
    out = np.empty_like(send_major)
    _c().oracle_a2a_exchange(_u16(send_major), _u16(out), N, H, d, P)
    return out


def a2a_unpack(xbuf: np.ndarray, N: int, H: int, d: int, P: int, slot_order: int = SEND_MAJOR,
               rank_begin: int = 0, rank_count: Optional[int] = None,
               out: Optional[np.ndarray] = None) -> np.ndarray:
    """Exchange buffer -> head-parallel [H][N][d]; only destination ranks in the range are written."""
    rank_count = P if rank_count is None else rank_count
    if out is None:
        out = np.zeros((H, N, d), dtype=np.uint16)
    _c().oracle_a2a_unpack(_u16(xbuf), _u16(out), N, H, d, P, rank_begin, rank_count, slot_order)
    return out


# ---------------------------------------------------------------------------
# V-Major selection (Section III-D), threshold-per-tile form
# ---------------------------------------------------------------------------

def vmajor_select(v_cur: np.ndarray, v_prev: np.ndarray, tau: float, tile_tokens: int = 16,
                  cap_tiles: Optional[int] = None, want_compact: bool = True
                  ) -> Tuple[np.ndarray, np.ndarray, int, Optional[np.ndarray]]:
    """Returns (flags [NT], idx [n_active] ascending, n_active, compact [S][cap*T][W] or None)."""
    S, N, W = v_cur.shape
    assert v_prev.shape == v_cur.shape and N % tile_tokens == 0
    NT = N // tile_tokens
    cap = NT if cap_tiles is None else cap_tiles
    flags = np.zeros(NT, dtype=np.int32)
    idx = np.full(NT, -1, dtype=np.int32)
    compact = np.zeros((S, cap * tile_tokens, W), dtype=np.uint16) if want_compact else None
    n_active = _c().oracle_vmajor_select(
        S, N, W, tile_tokens, _u16(v_cur), _u16(v_prev), np.float32(tau), _i32(flags), _i32(idx),
        _u16(compact) if want_compact else None, cap)
    return flags, idx[:n_active].copy(), int(n_active), compact


def vmajor_gather(x: np.ndarray, idx: np.ndarray, tile_tokens: int = 16, cap_tiles: Optional[int] = None) -> np.ndarray:
    """Gather the listed tiles of x [S][N][W] into [S][cap*T][W] (Section III-D, extraction of active projections)."""
    S, N, W = x.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    cap = max(len(idx), 1) if cap_tiles is None else cap_tiles
    out = np.zeros((S, cap * tile_tokens, W), dtype=np.uint16)
    _c().oracle_vmajor_gather(S, N, W, tile_tokens, _u16(x), _i32(idx), len(idx), _u16(out), cap)
    return out


def vmajor_scatter(compact: np.ndarray, idx: np.ndarray, cache: np.ndarray, tile_tokens: int = 16) -> np.ndarray:
    """Overwrite the listed tiles of a copy of cache [S][N][W] with compact [S][cap*T][W] (receiver reconstruction)."""
    S, N, W = cache.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    cap = compact.shape[1] // tile_tokens
    out = cache.copy()
    _c().oracle_vmajor_scatter(S, N, W, tile_tokens, _u16(compact), _i32(idx), len(idx), _u16(out), cap)
    return out


# ---------------------------------------------------------------------------
# Ulysses all-to-all #2: head-parallel -> sequence-parallel (Section II-A)
# ---------------------------------------------------------------------------

def a2a_pack_hs(y_hs: np.ndarray, P: int, slot_order: int = SEND_MAJOR, rank_begin: int = 0,
                rank_count: Optional[int] = None, out: Optional[np.ndarray] = None) -> np.ndarray:
    """[H][N][d] -> exchange buffer [P*P][Ns][Hp][d]; only source ranks (head owners) in the range are written."""
    H, N, d = y_hs.shape
    rank_count = P if rank_count is None else rank_count
    if out is None:
        out = np.zeros((P * P, N // P, H // P, d), dtype=np.uint16)
    _c().oracle_a2a_pack_hs(_u16(y_hs), _u16(out), N, H, d, P, rank_begin, rank_count, slot_order)
    return out


def a2a_unpack_seq(xbuf: np.ndarray, N: int, H: int, d: int, P: int, slot_order: int = SEND_MAJOR,
                   rank_begin: int = 0, rank_count: Optional[int] = None,
                   out: Optional[np.ndarray] = None) -> np.ndarray:
    """Exchange buffer -> sequence-parallel [N][H][d]; only destination ranks (token owners) in the range are written."""
    rank_count = P if rank_count is None else rank_count
    if out is None:
        out = np.zeros((N, H, d), dtype=np.uint16)
    _c().oracle_a2a_unpack_seq(_u16(xbuf), _u16(out), N, H, d, P, rank_begin, rank_count, slot_order)
    return out


# ---------------------------------------------------------------------------
# V-Major selection as the paper states it (Section III-D): per-token L1 distance to the cached value
# vector, the fraction r with the smallest distance stays cached, the rest is active; r follows the
# time-varying schedule (warm-up, linear ramp, periodic full update).
# ---------------------------------------------------------------------------

def token_l1_metric(v_cur: np.ndarray, v_prev: np.ndarray) -> np.ndarray:
    """metric[n] = sum over the token's whole value vector (all slabs s, all w) of |v_cur - v_prev|, in fp64."""
    assert v_cur.shape == v_prev.shape
    return np.abs(widen(v_cur) - widen(v_prev)).sum(axis=(0, 2))


def topk_active(metric: np.ndarray, n_active: int) -> np.ndarray:
    """Ascending indices of the n_active tokens with the largest metric; NaN ranks above every number;
    among equal metrics the lower index is taken first."""
    metric = np.asarray(metric)
    n = metric.shape[0]
    n_active = max(0, min(int(n_active), n))
    is_nan = np.isnan(metric)
    value = np.where(is_nan, 0.0, metric)
    order = np.lexsort((np.arange(n), -value, ~is_nan))     # NaN first, then larger metric, then lower index
    return np.sort(order[:n_active]).astype(np.int32)


def cache_ratio(step: int, n_steps: int, warmup: int, sync_every: int) -> float:
    """Cache ratio r of denoising step `step` (1-based, 1..n_steps): 0 during the warm-up steps and on every
    sync_every-th step (full update); otherwise linear from 0 at the warm-up boundary to 1 at the last step."""
    if step <= warmup or (sync_every > 0 and step % sync_every == 0) or n_steps <= warmup:
        return 0.0
    return (step - warmup) / float(n_steps - warmup)


def active_count(step: int, n_steps: int, warmup: int, sync_every: int, n_tokens: int) -> int:
    """Tokens communicated at this step: all but the floor(r * n_tokens) that stay cached."""
    r = cache_ratio(step, n_steps, warmup, sync_every)
    return n_tokens - int(np.floor(r * n_tokens + 1e-9))
