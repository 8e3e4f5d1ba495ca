"""Pins for the CPU oracle: what the paper prints, closed forms, invariants, brute force.

None of these tests goes through the oracle's own formulas to get its expected
value: brute force is pure-Python arithmetic on tiny inputs (exact rationals for
the projection), special cases reduce to identities or library routines, and
closed forms are numbers worked out by hand.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from synth import CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_layer_inputs, make_v_pair, perturb_tiles

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_shapes.txt")


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            vals[k.strip()] = int(v)
    return vals


def _bits(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _rand_bits(rng, shape, scale=1.0):
    return _bits(rng.standard_normal(shape).astype(np.float32) * scale)


# ---------------------------------------------------------------------------
# shapes: the paper's printed numbers fix D, bytes/element, token counts
# ---------------------------------------------------------------------------

def test_paper_message_and_cache_sizes_fix_the_shapes():
    g = _golden()
    c3 = CONFIGS["C3"]
    assert c3.H == g["heads"] and c3.P == g["ranks_per_node"]
    # one rank's Q+K+V shard, 2 bytes per element, is the paper's "14 MB" message
    msg = c3.Ns * c3.D * 2 * 3
    assert round(msg / 1e6) == g["phase1_message_MB"]
    # head-parallel slab per rank = N * (H/P) * d * 2 bytes; 4 tensors x 60 blocks x batch 4
    slab = c3.N * c3.Hp * c3.d * 2
    total = g["cache_tensors_per_layer"] * g["model_blocks"] * g["cache_batch"] * slab
    assert total == g["cache_per_rank_MB"] * 1024 * 1024
    for name, key in (("C2", "grid_768"), ("C3", "grid_1536"), ("C4", "grid_2304")):
        cfg = CONFIGS[name]
        assert cfg.grid == (g[key], g[key]) and cfg.N == g[key] ** 2
    for cfg in CONFIGS.values():
        assert cfg.D == cfg.H * cfg.d and cfg.N == int(np.prod(cfg.grid))
        assert cfg.N % cfg.P == 0 and cfg.H % cfg.P == 0 and cfg.Ns % cfg.tile_tokens == 0
        assert sum(cfg.pairs) == cfg.d // 2 and len(cfg.pairs) == len(cfg.grid)


def test_bf16_round_trip_and_rne():
    # widening then rounding is the identity on every finite bf16 pattern
    allbits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    f = bf16_bits_to_f32(allbits)
    finite = np.isfinite(f)
    assert np.array_equal(f32_to_bf16_bits(f[finite]), allbits[finite])
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert f32_to_bf16_bits(np.float32([1 + 2.0 ** -8]))[0] == 0x3F80
    assert f32_to_bf16_bits(np.float32([1 + 3 * 2.0 ** -8]))[0] == 0x3F82
    assert f32_to_bf16_bits(np.float32([1 + 2.0 ** -8 + 2.0 ** -20]))[0] == 0x3F81


def test_widen_is_exact(oracle):
    allbits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    w = oracle.widen(allbits)
    # sign, exponent, mantissa decoded by hand for normal numbers
    s = (allbits >> 15).astype(np.int64)
    e = ((allbits >> 7) & 0xFF).astype(np.int64)
    m = (allbits & 0x7F).astype(np.int64)
    normal = (e > 0) & (e < 255)
    expect = (1 - 2 * s[normal]) * (1 + m[normal] / 128.0) * np.exp2((e[normal] - 127).astype(np.float64))
    assert np.array_equal(w[normal], expect)
    sub = e == 0
    assert np.array_equal(w[sub], (1 - 2 * s[sub]) * (m[sub] / 128.0) * 2.0 ** -126)


# ---------------------------------------------------------------------------
# O1 projection
# ---------------------------------------------------------------------------

def test_proj_brute_force_exact_rationals(oracle):
    rng = np.random.default_rng(1)
    n, Di, Do = 5, 12, 7
    x = _rand_bits(rng, (n, Di))
    w = _rand_bits(rng, (Do, Di), 0.3)
    y = oracle.qkv_proj(x, w)
    assert y.shape == (n, Do)
    xf = bf16_bits_to_f32(x)
    wf = bf16_bits_to_f32(w)
    for i in range(n):
        for o in range(Do):
            acc = Fraction(0)
            for k in range(Di):
                acc += Fraction(float(xf[i, k])) * Fraction(float(wf[o, k]))
            assert abs(y[i, o] - float(acc)) <= 1e-14 * max(1.0, abs(float(acc)))


def test_proj_identity_onehot_and_unit_rows(oracle):
    rng = np.random.default_rng(2)
    D = 32
    x = _rand_bits(rng, (9, D))
    eye = _bits(np.eye(D))
    assert np.array_equal(oracle.qkv_proj(x, eye), oracle.widen(x))
    # W rows are one-hot: output column o picks input column perm[o]
    perm = rng.permutation(D)
    w = np.zeros((D, D), dtype=np.float32)
    w[np.arange(D), perm] = 1.0
    assert np.array_equal(oracle.qkv_proj(x, _bits(w)), oracle.widen(x)[:, perm])
    # X rows are unit vectors e_k: output row is column k of W^T = W[:, k]
    wr = _rand_bits(rng, (D, D))
    xe = _bits(np.eye(D)[[3, 17]])
    assert np.array_equal(oracle.qkv_proj(xe, wr), oracle.widen(wr)[:, [3, 17]].T)


def test_proj_small_integers_are_exact(oracle):
    rng = np.random.default_rng(3)
    x = rng.integers(-8, 9, size=(16, 64)).astype(np.float32)
    w = rng.integers(-8, 9, size=(24, 64)).astype(np.float32)
    y = oracle.qkv_proj(_bits(x), _bits(w))
    expect = x.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(y, expect.astype(np.float64))


def test_proj_output_statistics_of_the_workload(oracle):
    cfg = CONFIGS["C1"]
    inp = make_layer_inputs(cfg)
    v = oracle.qkv_proj(inp["X"], inp["Wv"])
    # X ~ N(0,1), W ~ N(0,1/D): outputs have unit variance
    assert abs(v.std() - 1.0) < 0.05 and abs(v.mean()) < 0.02


# ---------------------------------------------------------------------------
# O2 RMSNorm
# ---------------------------------------------------------------------------

def test_rmsnorm_unit_gain_gives_unit_rms(oracle):
    rng = np.random.default_rng(4)
    x = rng.standard_normal((7, 3, 64)) * 5.0
    y = oracle.rms_norm(x, np.ones(64), 1e-6)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-6)


def test_rmsnorm_scale_invariance_constant_rows_and_gain(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 2, 16))
    g = 1.0 + 0.1 * rng.standard_normal(16)
    y = oracle.rms_norm(x, g, 0.0)
    assert np.allclose(oracle.rms_norm(x * 8.0, g, 0.0), y, rtol=1e-14, atol=0)
    # constant row c -> sign(c) * gamma
    c = np.full((1, 1, 16), -3.5)
    assert np.allclose(oracle.rms_norm(c, g, 0.0), -g, rtol=1e-14)
    # eps sits inside the square root, added to the mean square: x = (2,0,0,0), eps = 3 -> 2/sqrt(1+3) = 1
    x4 = np.array([[[2.0, 0.0, 0.0, 0.0]]])
    assert np.allclose(oracle.rms_norm(x4, np.ones(4), 3.0), [[[1.0, 0, 0, 0]]], rtol=1e-15)


def test_rmsnorm_brute_force(oracle):
    rng = np.random.default_rng(6)
    x = rng.standard_normal((3, 2, 8))
    g = rng.standard_normal(8)
    y = oracle.rms_norm(x, g, 1e-6)
    for n in range(3):
        for h in range(2):
            ss = 0.0
            for i in range(8):
                ss += x[n, h, i] ** 2
            denom = math.sqrt(ss / 8 + 1e-6)
            for i in range(8):
                assert abs(y[n, h, i] - x[n, h, i] / denom * g[i]) < 1e-14


# ---------------------------------------------------------------------------
# O2 RoPE
# ---------------------------------------------------------------------------

def test_token_coords_row_major_last_axis_fastest(oracle):
    c = oracle.token_coords(np.array([0, 1, 47, 48, 49, 2303]), (48, 48))
    assert c.tolist() == [[0, 0], [0, 1], [0, 47], [1, 0], [1, 1], [47, 47]]
    c3 = oracle.token_coords(np.array([0, 103, 104, 6239, 6240, 99839]), (16, 60, 104))
    assert c3.tolist() == [[0, 0, 0], [0, 0, 103], [0, 1, 0], [0, 59, 103], [1, 0, 0], [15, 59, 103]]


def test_rope_preserves_norms_and_identity_at_origin(oracle):
    rng = np.random.default_rng(7)
    grid, pairs = (6, 5), (3, 5)
    ids = np.arange(30)
    y = rng.standard_normal((30, 2, 16))
    r = oracle.rope_rotate(y, ids, grid, pairs, 10000.0)
    assert np.allclose((r * r).sum(-1), (y * y).sum(-1), rtol=1e-12)
    # every pair keeps its own norm
    assert np.allclose(r[..., 0::2] ** 2 + r[..., 1::2] ** 2, y[..., 0::2] ** 2 + y[..., 1::2] ** 2, rtol=1e-12)
    assert np.array_equal(r[0], y[0])  # token 0 sits at the origin of every axis


def test_rope_closed_form_angles(oracle):
    # grid 4 x 8, 16 pairs per axis (d = 64), theta = 10000.
    # Local pair j' on an axis with 16 pairs turns by coord * 10000**(-j'/16):
    #   j' = 0 -> coord rad, j' = 4 -> coord * 0.1 rad, j' = 8 -> coord * 0.01 rad, j' = 12 -> coord * 0.001 rad
    grid, pairs = (4, 8), (16, 16)
    tok = np.array([3 * 8 + 5])  # row 3, column 5
    y = np.zeros((1, 1, 64))
    y[0, 0, 0::2] = 1.0  # every pair is (1, 0): rotated to (cos phi, sin phi)
    r = oracle.rope_rotate(y, tok, grid, pairs, 10000.0)[0, 0]
    for jl, w in ((0, 1.0), (4, 0.1), (8, 0.01), (12, 0.001)):
        j = jl  # axis 0 (rows): coordinate 3
        assert abs(r[2 * j] - math.cos(3 * w)) < 1e-12 and abs(r[2 * j + 1] - math.sin(3 * w)) < 1e-12
        j = 16 + jl  # axis 1 (columns): coordinate 5
        assert abs(r[2 * j] - math.cos(5 * w)) < 1e-12 and abs(r[2 * j + 1] - math.sin(5 * w)) < 1e-12
    # a pair (0, 1) is rotated to (-sin phi, cos phi)
    y2 = np.zeros((1, 1, 64))
    y2[0, 0, 1] = 1.0
    r2 = oracle.rope_rotate(y2, tok, grid, pairs, 10000.0)[0, 0]
    assert abs(r2[0] + math.sin(3.0)) < 1e-12 and abs(r2[1] - math.cos(3.0)) < 1e-12


def test_rope_3d_axis_split(oracle):
    # 3 axes (t, h, w) with 2/3/3 pairs; token at (t, h, w) = (1, 2, 3) on a 2x3x4 grid
    grid, pairs = (2, 3, 4), (2, 3, 3)
    tok = np.array([1 * 12 + 2 * 4 + 3])
    y = np.zeros((1, 1, 16))
    y[0, 0, 0::2] = 1.0
    r = oracle.rope_rotate(y, tok, grid, pairs, 10000.0)[0, 0]
    # first pair of each axis turns by exactly the coordinate
    for j, coord in ((0, 1.0), (2, 2.0), (5, 3.0)):
        assert abs(r[2 * j] - math.cos(coord)) < 1e-12 and abs(r[2 * j + 1] - math.sin(coord)) < 1e-12
    # second pair of the t axis (2 pairs): 10000**(-1/2) = 0.01
    assert abs(r[2] - math.cos(0.01)) < 1e-12 and abs(r[3] - math.sin(0.01)) < 1e-12


def test_rope_relative_position_property(oracle):
    rng = np.random.default_rng(8)
    grid, pairs = (8, 8), (4, 4)
    q = rng.standard_normal((1, 1, 16))
    k = rng.standard_normal((1, 1, 16))

    def dot(nq, nk):
        rq = oracle.rope_rotate(q, np.array([nq]), grid, pairs, 10000.0)
        rk = oracle.rope_rotate(k, np.array([nk]), grid, pairs, 10000.0)
        return float((rq * rk).sum())

    # same offset (+2 rows, -1 column) from two different anchors
    a = dot(1 * 8 + 3, 3 * 8 + 2)
    b = dot(4 * 8 + 6, 6 * 8 + 5)
    assert abs(a - b) < 1e-12
    assert abs(a - dot(1 * 8 + 3, 3 * 8 + 3)) > 1e-6  # a different offset gives a different product


def test_rope_axes_are_independent(oracle):
    rng = np.random.default_rng(9)
    grid, pairs = (8, 8), (4, 4)
    y = rng.standard_normal((1, 2, 16))
    a = oracle.rope_rotate(y, np.array([2 * 8 + 5]), grid, pairs, 10000.0)
    b = oracle.rope_rotate(y, np.array([6 * 8 + 5]), grid, pairs, 10000.0)  # other row, same column
    assert np.array_equal(a[..., 8:], b[..., 8:])      # column pairs unchanged
    assert not np.allclose(a[..., :8], b[..., :8])     # row pairs changed


def test_norm_rope_chain_brute_force(oracle):
    rng = np.random.default_rng(10)
    grid, pairs, theta, eps = (3, 4), (2, 2), 10000.0, 1e-6
    H, d = 2, 8
    ids = np.array([0, 5, 7, 11])
    xb = _rand_bits(rng, (4, H, d))
    gb = _bits(1.0 + 0.1 * rng.standard_normal(d))
    out = oracle.qk_norm_rope(xb, ids, gb, eps, grid, pairs, theta)
    xf = bf16_bits_to_f32(xb).astype(np.float64)
    gf = bf16_bits_to_f32(gb).astype(np.float64)
    for t, n in enumerate(ids):
        row, col = divmod(int(n), grid[1])
        for h in range(H):
            ms = sum(float(v) ** 2 for v in xf[t, h]) / d
            y = [float(xf[t, h, i]) / math.sqrt(ms + eps) * float(gf[i]) for i in range(d)]
            for j in range(d // 2):
                coord, jl, pa = (row, j, 2) if j < 2 else (col, j - 2, 2)
                phi = coord * 10000.0 ** (-jl / pa)
                e = y[2 * j] * math.cos(phi) - y[2 * j + 1] * math.sin(phi)
                o = y[2 * j] * math.sin(phi) + y[2 * j + 1] * math.cos(phi)
                assert abs(out[t, h, 2 * j] - e) < 1e-13 and abs(out[t, h, 2 * j + 1] - o) < 1e-13


# ---------------------------------------------------------------------------
# O3 pack / exchange / unpack
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("N,H,d,P", [(32, 4, 8, 2), (48, 6, 8, 3), (16, 4, 8, 1), (64, 4, 16, 4)])
def test_pack_unpack_is_the_head_major_transpose(oracle, N, H, d, P):
    x = np.arange(N * H * d, dtype=np.uint32).astype(np.uint16).reshape(N, H, d)
    want = np.ascontiguousarray(x.transpose(1, 0, 2))
    for order in (0, 1):  # chunk(r->p) in the sender's buffer, or in the receiver's
        buf = oracle.a2a_pack(x, P, order)
        assert np.array_equal(np.sort(buf.reshape(-1)), x.reshape(-1))  # a permutation: every slot once
        y = oracle.a2a_unpack(buf, N, H, d, P, order)
        assert np.array_equal(y, want)
    # the literal exchange between pack and unpack equals the folded addressing
    send = oracle.a2a_pack(x, P, 0)
    recv = oracle.a2a_exchange(send, N, H, d, P)
    assert np.array_equal(recv, oracle.a2a_pack(x, P, 1))
    assert np.array_equal(oracle.a2a_unpack(recv, N, H, d, P, 1), want)


def test_pack_closed_form_source_index_brute_force(oracle):
    N, H, d, P = 48, 6, 8, 3
    Ns, Hp = N // P, H // P
    x = np.arange(N * H * d, dtype=np.uint32).astype(np.uint16).reshape(N, H, d)
    buf = oracle.a2a_pack(x, P, 0).reshape(-1)
    buf_recv = oracle.a2a_pack(x, P, 1).reshape(-1)
    chunk = Ns * Hp * d
    for r in range(P):
        for p in range(P):
            for n in range(Ns):
                for hl in range(Hp):
                    for i in (0, d - 1):
                        src = ((r * Ns + n) * H + p * Hp + hl) * d + i
                        off = (n * Hp + hl) * d + i
                        assert buf[(r * P + p) * chunk + off] == src
                        assert buf_recv[(p * P + r) * chunk + off] == src


def test_pack_single_rank_is_identity_and_unpack_is_numpy_transpose(oracle):
    rng = np.random.default_rng(11)
    x = rng.integers(0, 65536, size=(32, 4, 8)).astype(np.uint16)
    buf = oracle.a2a_pack(x, 1, 0)
    assert np.array_equal(buf.reshape(x.shape), x)
    assert np.array_equal(oracle.a2a_unpack(buf, 32, 4, 8, 1, 0), np.transpose(x, (1, 0, 2)))


def test_per_rank_calls_equal_one_call(oracle):
    rng = np.random.default_rng(12)
    N, H, d, P = 64, 4, 8, 4
    x = rng.integers(0, 65536, size=(N, H, d)).astype(np.uint16)
    for order in (0, 1):
        whole = oracle.a2a_pack(x, P, order)
        parts = np.zeros_like(whole)
        for r in (2, 0, 3, 1):
            oracle.a2a_pack(x, P, order, rank_begin=r, rank_count=1, out=parts)
        assert np.array_equal(parts, whole)
        y_whole = oracle.a2a_unpack(whole, N, H, d, P, order)
        y_parts = np.zeros_like(y_whole)
        oracle.a2a_unpack(whole, N, H, d, P, order, rank_begin=1, rank_count=3, out=y_parts)
        oracle.a2a_unpack(whole, N, H, d, P, order, rank_begin=0, rank_count=1, out=y_parts)
        assert np.array_equal(y_parts, y_whole)


# ---------------------------------------------------------------------------
# O4 selection
# ---------------------------------------------------------------------------

def test_select_finds_exactly_the_generators_tiles(oracle):
    cfg = CONFIGS["C1"]
    for layout in ("hs", "seq"):
        cur, prev, changed = make_v_pair(cfg, layout=layout)
        flags, idx, n_active, compact = oracle.vmajor_select(cur, prev, cfg.tau, cfg.tile_tokens)
        assert n_active == cfg.n_changed == len(changed)
        assert np.array_equal(idx, changed)
        assert np.array_equal(np.nonzero(flags)[0], changed)
        T = cfg.tile_tokens
        for j, t in enumerate(idx):
            assert np.array_equal(compact[:, j * T:(j + 1) * T, :], cur[:, t * T:(t + 1) * T, :])


def test_select_brute_force_mask_and_layout_independence(oracle):
    rng = np.random.default_rng(13)
    H, N, d, T = 3, 64, 8, 16
    cur = _rand_bits(rng, (H, N, d))
    prev, changed = perturb_tiles(cur, 1, T, 2, rng, sigma=0.05)
    tau = 1e-3
    flags, idx, n_active, _ = oracle.vmajor_select(cur, prev, tau, T)
    cf, pf = bf16_bits_to_f32(cur), bf16_bits_to_f32(prev)
    brute = []
    for t in range(N // T):
        m = 0.0
        for h in range(H):
            for n in range(t * T, (t + 1) * T):
                for w in range(d):
                    m = max(m, abs(float(cf[h, n, w]) - float(pf[h, n, w])))
        if m > tau:
            brute.append(t)
    assert idx.tolist() == brute == changed.tolist() and n_active == len(brute)
    # sequence layout [1][N][H*d] of the same values gives the same mask
    cur_seq = np.ascontiguousarray(cur.transpose(1, 0, 2)).reshape(1, N, H * d)
    prev_seq = np.ascontiguousarray(prev.transpose(1, 0, 2)).reshape(1, N, H * d)
    _, idx_seq, _, _ = oracle.vmajor_select(cur_seq, prev_seq, tau, T)
    assert np.array_equal(idx_seq, idx)


def test_select_edge_cases(oracle):
    rng = np.random.default_rng(14)
    S, N, W, T = 2, 80, 8, 16
    NT = N // T
    cur = _rand_bits(rng, (S, N, W))
    tau = 1e-3

    def run(prev, **kw):
        return oracle.vmajor_select(cur, prev, tau, T, **kw)

    # nothing changed
    flags, idx, n, compact = run(cur.copy())
    assert n == 0 and idx.size == 0 and not flags.any()
    # everything changed
    prev = f32_to_bf16_bits(bf16_bits_to_f32(cur) + np.float32(1.0))
    flags, idx, n, compact = run(prev)
    assert n == NT and idx.tolist() == list(range(NT)) and np.array_equal(compact, cur)
    # a single element, last slab / last row of the tile / last column, first and last tile
    for t in (0, NT - 1):
        prev = cur.copy()
        prev[S - 1, t * T + T - 1, W - 1] = _bits([bf16_bits_to_f32(cur[S - 1:, t * T + T - 1, W - 1])[0] + 0.5])[0]
        flags, idx, n, compact = run(prev)
        assert idx.tolist() == [t] and n == 1
        assert np.array_equal(compact[:, :T, :], cur[:, t * T:(t + 1) * T, :])
    # threshold: |diff| = 2^-10 (< 1e-3) inactive, 2^-9 (> 1e-3) active
    base = cur.copy()
    base[0, 20, 3] = _bits([1.0 * 2.0 ** -9])[0]
    cur2 = base
    prev_small = base.copy()
    prev_small[0, 20, 3] = _bits([2.0 ** -9 - 2.0 ** -10])[0]
    prev_big = base.copy()
    prev_big[0, 20, 3] = 0
    assert oracle.vmajor_select(cur2, prev_small, tau, T)[2] == 0
    assert oracle.vmajor_select(cur2, prev_big, tau, T)[1].tolist() == [1]
    # the comparison is NOT(|diff| <= tau): equality is inactive
    assert oracle.vmajor_select(cur2, prev_big, 2.0 ** -9, T)[2] == 0
    # NaN counts as changed; +0 vs -0 does not
    prev_nan = cur.copy()
    prev_nan[1, 70, 0] = 0x7FC0
    assert run(prev_nan)[1].tolist() == [4]
    cz = cur.copy()
    cz[0, 5, 5] = 0x0000
    pz = cz.copy()
    pz[0, 5, 5] = 0x8000
    assert oracle.vmajor_select(cz, pz, tau, T)[2] == 0
    # capacity: the true count is returned, only cap_tiles tiles are gathered
    prev = f32_to_bf16_bits(bf16_bits_to_f32(cur) + np.float32(1.0))
    flags, idx, n, compact = run(prev, cap_tiles=2)
    assert n == NT and compact.shape == (S, 2 * T, W) and np.array_equal(compact, cur[:, :2 * T, :])


def test_select_decides_on_the_exact_difference_not_on_its_fp32_rounding(oracle):
    """|cur - prev| can exceed tau by less than half an fp32 ulp (exponents more than 16 binary orders apart): an fp32
    subtraction rounds such a difference onto tau and would call the tile unchanged.  The definition compares the
    difference itself; exact rational arithmetic on the bit patterns is the judge here."""
    from fractions import Fraction
    S, N, W, T = 1, 64, 8, 16
    NT = N // T

    def frac(bits16):
        return Fraction(float(bf16_bits_to_f32(np.array([bits16], dtype=np.uint16))[0]))

    cases = [  # (cur, prev, tau, active?)
        (2.0 ** -9, -(2.0 ** -40), 2.0 ** -9, True),      # fp32: 2^-9 + 2^-40 rounds to 2^-9 = tau
        (2.0 ** -9, 2.0 ** -40, 2.0 ** -9, False),        # just below tau on the other side
        (-(2.0 ** -9), 2.0 ** -40, 2.0 ** -9, True),      # mirrored signs
        (1.0, -(2.0 ** -30), 1.0, True),
        (1.0, 2.0 ** -30, 1.0, False),
        (1.5, 0.5 - 2.0 ** -8, 1.0, True),                # ordinary: 1 + 2^-8 > 1
        (1.5, 0.5, 1.0, False),                           # exactly tau
    ]
    for t_case, (c, p, tau, want) in enumerate(cases):
        cur = np.zeros((S, N, W), dtype=np.uint16)
        prev = np.zeros((S, N, W), dtype=np.uint16)
        t = t_case % NT
        cur[0, t * T + 5, 3], prev[0, t * T + 5, 3] = _bits([c])[0], _bits([p])[0]
        assert bf16_bits_to_f32(cur[0, t * T + 5, 3:4])[0] == np.float32(c) and bf16_bits_to_f32(prev[0, t * T + 5, 3:4])[0] == np.float32(p)
        exact_active = abs(frac(cur[0, t * T + 5, 3]) - frac(prev[0, t * T + 5, 3])) > Fraction(float(np.float32(tau)))
        assert exact_active == want
        flags, idx, n, _ = oracle.vmajor_select(cur, prev, tau, T)
        assert (n == 1 and idx.tolist() == [t] and flags[t] == 1) if want else (n == 0 and not flags.any()), (c, p, tau)


def test_select_scatter_back_leaves_nothing_active(oracle):
    cfg = CONFIGS["C1"]
    cur, prev, changed = make_v_pair(cfg)
    T = cfg.tile_tokens
    _, idx, n, compact = oracle.vmajor_select(cur, prev, cfg.tau, T)
    rebuilt = prev.copy()
    for j, t in enumerate(idx):
        rebuilt[:, t * T:(t + 1) * T, :] = compact[:, j * T:(j + 1) * T, :]
    assert oracle.vmajor_select(cur, rebuilt, cfg.tau, T)[2] == 0
    assert np.array_equal(rebuilt, cur)


# ---------------------------------------------------------------------------
# V-Major gather / scatter (sender-side extraction, receiver-side reconstruction)
# ---------------------------------------------------------------------------

def test_gather_scatter_brute_force_and_reconstruction(oracle):
    rng = np.random.default_rng(21)
    S, N, W, T = 3, 96, 8, 16
    x = rng.integers(0, 65536, size=(S, N, W)).astype(np.uint16)
    x_prev = rng.integers(0, 65536, size=(S, N, W)).astype(np.uint16)
    idx = np.array([1, 4, 5], dtype=np.int32)
    g = oracle.vmajor_gather(x, idx, T)
    assert g.shape == (S, 3 * T, W)
    for j, t in enumerate(idx):
        for s in range(S):
            for m in range(T):
                for w in range(W):
                    assert g[s, j * T + m, w] == x[s, t * T + m, w]
    rebuilt = oracle.vmajor_scatter(g, idx, x_prev, T)
    for t in range(N // T):
        want = x if t in idx else x_prev
        assert np.array_equal(rebuilt[:, t * T:(t + 1) * T], want[:, t * T:(t + 1) * T])
    # an empty list changes nothing; a small capacity gathers / scatters only the first tiles
    assert np.array_equal(oracle.vmajor_scatter(g, np.zeros(0, np.int32), x_prev, T), x_prev)
    g2 = oracle.vmajor_gather(x, idx, T, cap_tiles=2)
    assert g2.shape == (S, 2 * T, W) and np.array_equal(g2, g[:, :2 * T])
    r2 = oracle.vmajor_scatter(g2, idx, x_prev, T)
    assert np.array_equal(r2[:, 5 * T:6 * T], x_prev[:, 5 * T:6 * T]) and np.array_equal(r2[:, 4 * T:5 * T], x[:, 4 * T:5 * T])


def test_gather_by_selected_tiles_equals_the_selections_own_compaction(oracle):
    cfg = CONFIGS["C1"]
    cur, prev, changed = make_v_pair(cfg)
    _, idx, n, compact = oracle.vmajor_select(cur, prev, cfg.tau, cfg.tile_tokens)
    g = oracle.vmajor_gather(cur, idx, cfg.tile_tokens, cap_tiles=cfg.NT)
    assert np.array_equal(g[:, :n * cfg.tile_tokens], compact[:, :n * cfg.tile_tokens])
    # sender gathers, receiver scatters into its cache: the cache becomes the current tensor
    assert np.array_equal(oracle.vmajor_scatter(g, idx, prev, cfg.tile_tokens), cur)


# ---------------------------------------------------------------------------
# second all-to-all: head-parallel -> sequence-parallel
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("N,H,d,P", [(32, 4, 8, 2), (48, 6, 8, 3), (16, 4, 8, 1), (64, 4, 16, 4)])
def test_second_all_to_all_is_the_inverse_transpose(oracle, N, H, d, P):
    y = np.arange(N * H * d, dtype=np.uint32).astype(np.uint16).reshape(H, N, d)
    want = np.ascontiguousarray(y.transpose(1, 0, 2))
    for order in (0, 1):
        buf = oracle.a2a_pack_hs(y, P, order)
        assert np.array_equal(np.sort(buf.reshape(-1)), y.reshape(-1))
        assert np.array_equal(oracle.a2a_unpack_seq(buf, N, H, d, P, order), want)
    # literal round trip: first all-to-all, then the second, gives the tensor back
    x = np.random.default_rng(3).integers(0, 65536, size=(N, H, d)).astype(np.uint16)
    hs = oracle.a2a_unpack(oracle.a2a_pack(x, P, 1), N, H, d, P, 1)
    back = oracle.a2a_unpack_seq(oracle.a2a_pack_hs(hs, P, 0), N, H, d, P, 0)
    assert np.array_equal(back, x)


def test_second_all_to_all_chunk_contents_brute_force(oracle):
    N, H, d, P = 48, 6, 8, 3
    Ns, Hp = N // P, H // P
    y = np.arange(N * H * d, dtype=np.uint32).astype(np.uint16).reshape(H, N, d)
    send = oracle.a2a_pack_hs(y, P, 0).reshape(-1)
    recv = oracle.a2a_pack_hs(y, P, 1).reshape(-1)
    chunk = Ns * Hp * d
    for p in range(P):            # sender: owner of heads p*Hp ..
        for r in range(P):        # receiver: owner of tokens r*Ns ..
            for n in range(Ns):
                for hl in range(Hp):
                    for i in (0, d - 1):
                        src = ((p * Hp + hl) * N + r * Ns + n) * d + i
                        off = (n * Hp + hl) * d + i
                        assert send[(p * P + r) * chunk + off] == src
                        assert recv[(r * P + p) * chunk + off] == src
    # per-rank calls fill the same buffer as one call
    whole = oracle.a2a_pack_hs(y, P, 1)
    parts = np.zeros_like(whole)
    for p in (2, 0, 1):
        oracle.a2a_pack_hs(y, P, 1, rank_begin=p, rank_count=1, out=parts)
    assert np.array_equal(parts, whole)
    out = np.zeros((N, H, d), dtype=np.uint16)
    oracle.a2a_unpack_seq(whole, N, H, d, P, 1, rank_begin=1, rank_count=2, out=out)
    assert not out[:Ns].any()
    oracle.a2a_unpack_seq(whole, N, H, d, P, 1, rank_begin=0, rank_count=1, out=out)
    assert np.array_equal(out, y.transpose(1, 0, 2))


# ---------------------------------------------------------------------------
# the paper's own selection rule: per-token L1 distance, top (1 - r) fraction, cache schedule
# ---------------------------------------------------------------------------

def test_token_l1_metric_brute_force_and_closed_form(oracle):
    rng = np.random.default_rng(31)
    S, N, W = 3, 10, 8
    cur = _rand_bits(rng, (S, N, W))
    prev = _rand_bits(rng, (S, N, W))
    m = oracle.token_l1_metric(cur, prev)
    cf, pf = bf16_bits_to_f32(cur).astype(np.float64), bf16_bits_to_f32(prev).astype(np.float64)
    for n in range(N):
        acc = 0.0
        for s in range(S):
            for w in range(W):
                acc += abs(cf[s, n, w] - pf[s, n, w])
        assert abs(m[n] - acc) < 1e-12
    # closed form: every element of token 4 moved by exactly 0.5 -> S*W*0.5; untouched tokens -> 0
    prev2 = cur.copy()
    prev2[:, 4, :] = f32_to_bf16_bits(bf16_bits_to_f32(np.ascontiguousarray(cur[:, 4, :])) * 0 + 0.5)
    cur2 = cur.copy()
    cur2[:, 4, :] = f32_to_bf16_bits(np.ones((S, W), dtype=np.float32))
    m2 = oracle.token_l1_metric(cur2, prev2)
    assert m2[4] == S * W * 0.5 and np.count_nonzero(m2) == 1
    # layout independence: the same values as one slab [1][N][S*W]
    cs = np.ascontiguousarray(cur.transpose(1, 0, 2)).reshape(1, N, S * W)
    ps = np.ascontiguousarray(prev.transpose(1, 0, 2)).reshape(1, N, S * W)
    assert np.allclose(oracle.token_l1_metric(cs, ps), m, rtol=1e-14)


def test_topk_active_rules(oracle):
    m = np.array([0.5, 3.0, 3.0, 0.0, 7.0, 3.0, 1.0])
    assert oracle.topk_active(m, 0).tolist() == []
    assert oracle.topk_active(m, 1).tolist() == [4]
    assert oracle.topk_active(m, 2).tolist() == [1, 4]          # tie at 3.0: lower index first
    assert oracle.topk_active(m, 3).tolist() == [1, 2, 4]
    assert oracle.topk_active(m, 4).tolist() == [1, 2, 4, 5]
    assert oracle.topk_active(m, 7).tolist() == list(range(7))
    assert oracle.topk_active(m, 99).tolist() == list(range(7))
    mn = np.array([1.0, np.nan, np.inf, 2.0])
    assert oracle.topk_active(mn, 1).tolist() == [1]            # NaN counts as the largest change
    assert oracle.topk_active(mn, 2).tolist() == [1, 2]
    # brute force on random data with many ties
    rng = np.random.default_rng(32)
    m = rng.integers(0, 5, size=200).astype(np.float64)
    for k in (0, 1, 17, 100, 199, 200):
        pairs = sorted(((-m[i], i) for i in range(200)))[:k]
        assert oracle.topk_active(m, k).tolist() == sorted(i for _, i in pairs)


def test_cache_schedule_matches_the_papers_setup(oracle):
    # evaluation setup: 50 denoising steps, 5 warm-up steps, full update every 10 steps
    T, warm, sync = 50, 5, 10
    r = [oracle.cache_ratio(t, T, warm, sync) for t in range(1, T + 1)]
    assert all(x == 0.0 for x in r[:5])                        # warm-up: full exchange
    assert all(r[t - 1] == 0.0 for t in (10, 20, 30, 40, 50))  # periodic full update
    assert r[5] == pytest.approx(1 / 45) and r[48] == pytest.approx(44 / 45)   # linear from 0 towards 1
    body = [r[t - 1] for t in range(6, 50) if t % 10]
    assert all(b > a for a, b in zip(body, body[1:]))
    assert oracle.active_count(3, T, warm, sync, 9216) == 9216
    assert oracle.active_count(20, T, warm, sync, 9216) == 9216
    assert oracle.active_count(49, T, warm, sync, 9216) == 9216 - (9216 * 44) // 45
    assert oracle.active_count(28, T, warm, sync, 900) == 900 - int(900 * 23 / 45)
