"""Seeded generators for the synthetic DiT-shaped workloads.

Five workloads stand in for the models the paper measures (its weights and its
dataset are not needed: the cost of the path depends on shapes only).  The
shapes follow the paper's evaluation section: a token grid of (H_img/16)^2 for
768/1536/2304-pixel images, 24 attention heads of 128 (the 24-head model of
the evaluation), 12 ranks per node, plus a tiny case and a video-latent case.

Everything here is input generation: random draws, bf16 bit conversion and the
choice of which 16-token tiles differ between two denoising steps.  None of
the method's arithmetic lives here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

SEED_BASE = 2604145610


@dataclass(frozen=True)
class Config:
    name: str
    index: int              # 1-based position in the workload list (used for the seed)
    D: int                  # hidden size = H * d
    H: int                  # attention heads
    d: int                  # per-head dimension
    N: int                  # tokens (product of grid)
    grid: Tuple[int, ...]   # token grid, last axis fastest
    P: int                  # logical ranks
    pairs: Tuple[int, ...]  # rotary dimension pairs per grid axis (sum = d/2)
    changed_frac: float     # fraction of 16-token tiles that differ from the previous step
    tau: float = 1e-3       # selection threshold (fp32)
    eps: float = 1e-6       # RMSNorm epsilon
    theta: float = 10000.0  # rotary base
    tile_tokens: int = 16
    noise_sigma: float = 0.05

    @property
    def Ns(self) -> int:
        return self.N // self.P

    @property
    def Hp(self) -> int:
        return self.H // self.P

    @property
    def NT(self) -> int:
        return self.N // self.tile_tokens

    @property
    def n_changed(self) -> int:
        return int(round(self.changed_frac * self.NT))


CONFIGS: Dict[str, Config] = {
    "C1": Config("C1", 1, D=256, H=4, d=64, N=256, grid=(16, 16), P=2, pairs=(16, 16), changed_frac=0.25),
    "C2": Config("C2", 2, D=3072, H=24, d=128, N=2304, grid=(48, 48), P=12, pairs=(32, 32), changed_frac=0.30),
    "C3": Config("C3", 3, D=3072, H=24, d=128, N=9216, grid=(96, 96), P=12, pairs=(32, 32), changed_frac=0.20),
    "C4": Config("C4", 4, D=3072, H=24, d=128, N=20736, grid=(144, 144), P=12, pairs=(32, 32), changed_frac=0.10),
    "C5": Config("C5", 5, D=3072, H=24, d=128, N=99840, grid=(16, 60, 104), P=24, pairs=(16, 24, 24), changed_frac=0.15),
}


def config_seed(cfg: Config) -> int:
    return SEED_BASE + cfg.index


# ---------------------------------------------------------------------------
# bf16 bit patterns (stored as uint16)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, ((u >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, scale: float = 1.0, shift: float = 0.0,
                 chunk_elems: int = 1 << 24) -> np.ndarray:
    """shift + scale * N(0,1) drawn as float32 in stream order, rounded to bf16 bits."""
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.uint16)
    pos = 0
    while pos < total:
        n = min(chunk_elems, total - pos)
        z = rng.standard_normal(n, dtype=np.float32)
        if scale != 1.0:
            z *= np.float32(scale)
        if shift != 0.0:
            z += np.float32(shift)
        out[pos:pos + n] = f32_to_bf16_bits(z)
        pos += n
    return out.reshape(shape)


# ---------------------------------------------------------------------------
# layer inputs
# ---------------------------------------------------------------------------

def make_layer_inputs(cfg: Config, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Hidden states, projection weights and norm gains of one transformer layer.

    Draw order (fixed): X [N][D] ~ N(0,1); W_Q, W_K, W_V [D_out][D_in] ~ N(0, 1/D)
    (standard deviation D**-0.5); gamma_q, gamma_k [d] = 1 + 0.1 N(0,1).  All are
    float32 draws rounded once to bf16.
    """
    rng = np.random.Generator(np.random.PCG64(config_seed(cfg) if seed is None else seed))
    out = {"X": _normal_bf16(rng, (cfg.N, cfg.D))}
    sd = float(cfg.D) ** -0.5
    for name in ("Wq", "Wk", "Wv"):
        out[name] = _normal_bf16(rng, (cfg.D, cfg.D), scale=sd)
    for name in ("gamma_q", "gamma_k"):
        out[name] = _normal_bf16(rng, (cfg.d,), scale=0.1, shift=1.0)
    return out


def perturb_tiles(v_cur: np.ndarray, token_axis: int, tile_tokens: int, n_changed: int,
                  rng: np.random.Generator, sigma: float = 0.05) -> Tuple[np.ndarray, np.ndarray]:
    """Previous-step V: equal to ``v_cur`` bit for bit except on ``n_changed`` tiles.

    Tiles are ``tile_tokens`` consecutive tokens along ``token_axis``; the changed
    ones are the first ``n_changed`` entries of a seeded permutation of the tile
    ids.  On those tiles N(0, sigma) noise is added in float32 to every element
    and the sum is rounded to bf16.  Returns (v_prev bits, sorted changed tile ids).
    """
    n_tokens = v_cur.shape[token_axis]
    assert n_tokens % tile_tokens == 0
    nt = n_tokens // tile_tokens
    changed = np.sort(rng.permutation(nt)[:n_changed]).astype(np.int32)
    v_prev = v_cur.copy()
    cur_m = np.moveaxis(v_cur, token_axis, 0)
    prev_m = np.moveaxis(v_prev, token_axis, 0)
    for t in changed:
        sl = slice(int(t) * tile_tokens, (int(t) + 1) * tile_tokens)
        block = bf16_bits_to_f32(np.ascontiguousarray(cur_m[sl]))
        noise = rng.standard_normal(block.shape, dtype=np.float32) * np.float32(sigma)
        prev_m[sl] = f32_to_bf16_bits(block + noise)
    return v_prev, changed


def make_v_pair(cfg: Config, seed: Optional[int] = None, layout: str = "hs"):
    """Stand-alone selection workload: (v_cur, v_prev, changed tile ids).

    layout "hs": head-sharded [H][N][d]; layout "seq": [1][N][D].  v_cur ~ N(0,1).
    """
    rng = np.random.Generator(np.random.PCG64((config_seed(cfg) if seed is None else seed) + 7919))
    shape = (cfg.H, cfg.N, cfg.d) if layout == "hs" else (1, cfg.N, cfg.D)
    v_cur = _normal_bf16(rng, shape)
    v_prev, changed = perturb_tiles(v_cur, 1, cfg.tile_tokens, cfg.n_changed, rng, cfg.noise_sigma)
    return v_cur, v_prev, changed


def sample_token_ids(cfg: Config, seed: Optional[int] = None, random_tiles_per_rank: int = 64) -> np.ndarray:
    """Deterministic token subset for float parity at sizes a CPU cannot finish.

    Every rank's first and last 16-token tile plus ``random_tiles_per_rank`` seeded
    random tiles of that rank; returned as sorted unique global token ids.
    """
    rng = np.random.Generator(np.random.PCG64((config_seed(cfg) if seed is None else seed) + 104729))
    tiles_per_rank = cfg.Ns // cfg.tile_tokens
    tiles = []
    for r in range(cfg.P):
        base = r * tiles_per_rank
        pick = {0, tiles_per_rank - 1}
        k = min(random_tiles_per_rank, tiles_per_rank)
        pick.update(int(x) for x in rng.permutation(tiles_per_rank)[:k])
        tiles.extend(base + t for t in sorted(pick))
    tiles = np.asarray(sorted(set(tiles)), dtype=np.int64)
    tok = (tiles[:, None] * cfg.tile_tokens + np.arange(cfg.tile_tokens)[None, :]).reshape(-1)
    return tok
