"""GPU parity: every entry point of libcocodiff.so, through the C ABI, against the CPU oracle.

Integer/byte work (pack, unpack, select) must match bit for bit.  Float work (projection,
norm, RoPE) must satisfy max abs error <= 2e-2 and max |err| / max(|oracle|, 1) <= 1e-2 against
the oracle's unrounded fp64 result.  All inputs are seeded and synthetic (see ``synth``).
"""
import sys

import numpy as np
import pytest

import paper_2604_14561_amd as cd
from synth import (CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_layer_inputs, make_v_pair, perturb_tiles,
                   sample_token_ids)
from parity_util import assert_float_parity, dev_empty, to_dev, to_host_bits

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _sync():
    import torch
    torch.cuda.synchronize()


def _shape(cfg, rank_begin=0, rank_count=None):
    return cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, rank_begin, rank_count)


def _rope(cfg):
    table = to_dev(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta))
    return cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr()), table


# ---------------------------------------------------------------------------
# pack / unpack: bit-exact, every byte, every workload, both slot orders
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_pack_unpack_bit_exact(oracle, name):
    cfg = CONFIGS[name]
    say(f"pack/unpack {name} N={cfg.N} D={cfg.D} P={cfg.P}")
    rng = np.random.default_rng(100 + cfg.index)
    x = rng.integers(0, 65536, size=(cfg.N, cfg.H, cfg.d), dtype=np.uint16)
    want_hs = np.ascontiguousarray(x.transpose(1, 0, 2))
    xd = to_dev(x)
    for order in (cd.SEND_MAJOR, cd.RECV_MAJOR):
        buf = dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d))
        buf.fill_(-1)
        cd.a2a_pack(_shape(cfg), xd, buf, order)
        hs = dev_empty((cfg.H, cfg.N, cfg.d))
        hs.fill_(-1)
        cd.a2a_unpack(_shape(cfg), buf, hs, order)
        _sync()
        want_buf = oracle.a2a_pack(x, cfg.P, order)
        assert np.array_equal(to_host_bits(buf), want_buf), f"pack {name} order {order}"
        got_hs = to_host_bits(hs)
        assert np.array_equal(got_hs, oracle.a2a_unpack(want_buf, cfg.N, cfg.H, cfg.d, cfg.P, order))
        assert np.array_equal(got_hs, want_hs)   # the whole all-to-all: Y[h][n][i] = X[n][h][i]
        del buf, hs


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_per_rank_calls_equal_one_call(oracle, name):
    cfg = CONFIGS[name]
    rng = np.random.default_rng(200 + cfg.index)
    x = rng.integers(0, 65536, size=(cfg.N, cfg.H, cfg.d), dtype=np.uint16)
    xd = to_dev(x)
    for order in (cd.SEND_MAJOR, cd.RECV_MAJOR):
        buf = dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d))
        buf.fill_(-1)
        for r in reversed(range(cfg.P)):            # one source rank at a time, back to back
            cd.a2a_pack(_shape(cfg, r, 1), xd, buf, order)
        _sync()
        want_buf = oracle.a2a_pack(x, cfg.P, order)
        assert np.array_equal(to_host_bits(buf), want_buf)
        hs = dev_empty((cfg.H, cfg.N, cfg.d))
        hs.fill_(-1)
        split = cfg.P // 2
        cd.a2a_unpack(_shape(cfg, split, cfg.P - split), buf, hs, order)
        _sync()
        part = to_host_bits(hs)
        assert np.all(part[:split * cfg.Hp] == 0xFFFF)   # heads of ranks outside the range are untouched
        cd.a2a_unpack(_shape(cfg, 0, split), buf, hs, order)
        _sync()
        assert np.array_equal(to_host_bits(hs), x.transpose(1, 0, 2))


@pytest.mark.parametrize("order", [0, 1])
def test_pack_rank_ranges_of_several_ranks(oracle, order):
    """A range of several sender ranks that starts past rank 0: its chunks equal the oracle's, every other chunk stays
    as it was -- for the first all-to-all's pack (senders own tokens) and the second's (senders own heads)."""
    cfg = CONFIGS["C2"]
    P, first, count = cfg.P, 3, 4
    rng = np.random.default_rng(31 + order)
    x = rng.integers(0, 65535, size=(cfg.N, cfg.H, cfg.d), dtype=np.uint16)      # 0xFFFF is the fill value
    y = np.ascontiguousarray(x.transpose(1, 0, 2))
    # chunk slot of (sender s, receiver t)
    slot = (lambda s_, t_: t_ * P + s_) if order == cd.RECV_MAJOR else (lambda s_, t_: s_ * P + t_)
    sent = np.zeros(P * P, dtype=bool)
    for s_ in range(first, first + count):
        for t_ in range(P):
            sent[slot(s_, t_)] = True
    for call, src, want in ((cd.a2a_pack, x, oracle.a2a_pack(x, P, order)), (cd.a2a_pack_hs, y, oracle.a2a_pack_hs(y, P, order))):
        buf = dev_empty((P * P, cfg.Ns, cfg.Hp, cfg.d))
        buf.fill_(-1)
        call(_shape(cfg, first, count), to_dev(src), buf, order)
        _sync()
        got = to_host_bits(buf).reshape(P * P, -1)
        want = want.reshape(P * P, -1)
        assert np.array_equal(got[sent], want[sent]), call.__name__
        assert np.all(got[~sent] == 0xFFFF), f"{call.__name__}: chunks of other senders were written"


@pytest.mark.parametrize("N,H,d,P", [(48, 3, 8, 3), (16, 1, 8, 1), (80, 5, 24, 5), (272, 2, 200, 1), (32, 4, 512, 2)])
def test_pack_unpack_odd_shapes(oracle, N, H, d, P):
    rng = np.random.default_rng(N + H + d)
    x = rng.integers(0, 65536, size=(N, H, d), dtype=np.uint16)
    s = cd.Shape.make(N, H * d, H, d, P)
    buf = dev_empty((P * P, N // P, H // P, d))
    hs = dev_empty((H, N, d))
    cd.a2a_pack(s, to_dev(x), buf, cd.RECV_MAJOR)
    cd.a2a_unpack(s, buf, hs, cd.RECV_MAJOR)
    _sync()
    assert np.array_equal(to_host_bits(buf), oracle.a2a_pack(x, P, 1))
    assert np.array_equal(to_host_bits(hs), x.transpose(1, 0, 2))


# ---------------------------------------------------------------------------
# select: bit-exact flags, index list, count and gathered tiles
# ---------------------------------------------------------------------------

def _run_select(cur, prev, tau, T, cap=None, want_flags=True, want_compact=True):
    import torch
    S, N, W = cur.shape
    NT = N // T
    cap = NT if cap is None else cap
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(S, N, W, T), 16), dtype=torch.uint8, device="cuda:0")
    flags = dev_empty((NT,), "i32") if want_flags else None
    idx = dev_empty((NT,), "i32")
    idx.fill_(-7)
    n_act = dev_empty((1,), "i32")
    compact = dev_empty((S, cap * T, W)) if want_compact else None
    if compact is not None:
        compact.fill_(-1)
    cd.vmajor_select(S, N, W, T, to_dev(cur), to_dev(prev), tau, flags, idx, n_act, compact, cap, ws)
    _sync()
    n = int(n_act.cpu()[0])
    return (flags.cpu().numpy() if want_flags else None, idx.cpu().numpy(), n,
            to_host_bits(compact) if want_compact else None)


def _check_select(oracle, cur, prev, tau, T, cap=None):
    flags, idx, n, compact = _run_select(cur, prev, tau, T, cap)
    o_flags, o_idx, o_n, o_compact = oracle.vmajor_select(cur, prev, tau, T, cap_tiles=cap)
    assert n == o_n
    assert np.array_equal(flags, o_flags)
    assert np.array_equal(idx[:n], o_idx)
    k = min(n, o_compact.shape[1] // T)
    assert np.array_equal(compact[:, :k * T, :], o_compact[:, :k * T, :])
    return o_idx, n


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_select_bit_exact(oracle, name):
    cfg = CONFIGS[name]
    say(f"select {name} head-sharded [{cfg.H}][{cfg.N}][{cfg.d}], {cfg.n_changed} of {cfg.NT} tiles changed")
    cur, prev, changed = make_v_pair(cfg, layout="hs")
    idx, n = _check_select(oracle, cur, prev, cfg.tau, cfg.tile_tokens)
    assert n == cfg.n_changed and np.array_equal(idx, changed)   # the generator's own record of what it changed


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_select_sequence_layout_gives_the_same_tiles(oracle, name):
    cfg = CONFIGS[name]
    cur, prev, changed = make_v_pair(cfg, layout="seq")
    idx, n = _check_select(oracle, cur, prev, cfg.tau, cfg.tile_tokens)
    assert np.array_equal(idx, changed)


def test_select_edge_cases(oracle):
    rng = np.random.default_rng(77)
    S, N, W, T = 3, 1280, 40, 16            # 80 tiles; a (tile, slab) segment is 80 vectors: a ragged piece
    NT = N // T
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    tau = 1e-3
    # nothing changed / everything changed
    assert _check_select(oracle, cur, cur.copy(), tau, T)[1] == 0
    allc = f32_to_bf16_bits(bf16_bits_to_f32(cur) + np.float32(1.0))
    assert _check_select(oracle, cur, allc, tau, T)[1] == NT
    # capacity smaller than the active count: the count is the true one, cap tiles are gathered
    flags, idx, n, compact = _run_select(cur, allc, tau, T, cap=5)
    assert n == NT and np.array_equal(compact, cur[:, :5 * T, :])
    # single elements in corners of first / last tile
    for t, s, m, w in ((0, 0, 0, 0), (NT - 1, S - 1, T - 1, W - 1), (37, 1, 7, 39)):
        prev = cur.copy()
        prev[s, t * T + m, w] ^= 0x4000
        idx, n = _check_select(oracle, cur, prev, tau, T)
        assert idx.tolist() == [t]
    # threshold: 2^-10 below tau, 2^-9 above; equality with tau is inactive; NaN active; -0 vs +0 inactive
    base = cur.copy()
    base[0, 20, 3] = f32_to_bf16_bits(np.float32([2.0 ** -9]))[0]
    p_small = base.copy()
    p_small[0, 20, 3] = f32_to_bf16_bits(np.float32([2.0 ** -10]))[0]
    p_big = base.copy()
    p_big[0, 20, 3] = 0
    assert _check_select(oracle, base, p_small, tau, T)[1] == 0
    assert _check_select(oracle, base, p_big, tau, T)[0].tolist() == [1]
    assert _check_select(oracle, base, p_big, 2.0 ** -9, T)[1] == 0
    p_nan = cur.copy()
    p_nan[2, 1279, 39] = 0x7FC0
    assert _check_select(oracle, cur, p_nan, tau, T)[0].tolist() == [NT - 1]
    cz, pz = cur.copy(), cur.copy()
    cz[1, 5, 5], pz[1, 5, 5] = 0x0000, 0x8000
    assert _check_select(oracle, cz, pz, tau, T)[1] == 0
    # differences that an fp32 subtraction rounds onto tau are still decided as what they are (double difference)
    for c_val, p_val, tau_c, want_active in ((2.0 ** -9, -(2.0 ** -40), 2.0 ** -9, True), (2.0 ** -9, 2.0 ** -40, 2.0 ** -9, False),
                                             (-(2.0 ** -9), 2.0 ** -40, 2.0 ** -9, True), (1.0, -(2.0 ** -30), 1.0, True),
                                             (1.0, 2.0 ** -30, 1.0, False), (1.5, 0.5, 1.0, False)):
        cc, pp = np.zeros((S, N, W), dtype=np.uint16), np.zeros((S, N, W), dtype=np.uint16)
        cc[1, 16 * 33 + 9, 17] = f32_to_bf16_bits(np.float32([c_val]))[0]
        pp[1, 16 * 33 + 9, 17] = f32_to_bf16_bits(np.float32([p_val]))[0]
        assert _check_select(oracle, cc, pp, tau_c, T)[0].tolist() == ([33] if want_active else []), (c_val, p_val)
    # tau = 0: every equal element sits on the threshold (the double re-compare runs everywhere); only real changes count
    prev0, changed0 = perturb_tiles(cur, 1, T, 5, rng)
    assert np.array_equal(_check_select(oracle, cur, prev0, 0.0, T)[0], changed0)
    # index-only call (no flags, no gathered data)
    prev, changed = perturb_tiles(cur, 1, T, 9, rng)
    _, idx, n, _ = _run_select(cur, prev, tau, T, want_flags=False, want_compact=False)
    assert n == 9 and np.array_equal(idx[:n], changed)


def test_select_unusual_thresholds(oracle):
    """tau = 0, a negative tau, an infinite tau and a NaN tau: the same answers as the definition
    NOT(|cur - prev| <= tau) gives on the CPU (every tile with a difference / every tile / none / every tile)."""
    rng = np.random.default_rng(81)
    S, N, W, T = 2, 640, 64, 16
    NT = N // T
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    prev, changed = perturb_tiles(cur, 1, T, 6, rng)
    assert np.array_equal(_check_select(oracle, cur, prev, 0.0, T)[0], changed)
    assert _check_select(oracle, cur, prev, -1.0, T)[1] == NT
    assert _check_select(oracle, cur, prev, float("inf"), T)[1] == 0
    assert _check_select(oracle, cur, prev, float("nan"), T)[1] == NT
    # denormal differences against tau = 0 and against the smallest normal number
    tiny = np.zeros((S, N, W), dtype=np.uint16)
    tiny_prev = tiny.copy()
    tiny_prev[1, 16 * 7 + 3, 5] = 0x0001                     # the smallest bf16 denormal, 2^-133
    assert _check_select(oracle, tiny, tiny_prev, 0.0, T)[0].tolist() == [7]
    assert _check_select(oracle, tiny, tiny_prev, 2.0 ** -126, T)[1] == 0


def test_select_static_and_workspace_forms_agree_at_full_size(oracle):
    """The largest workload through both forms of the selection (caller workspace / library-owned flag words)."""
    import torch
    cfg = CONFIGS["C5"]
    cur, prev, changed = make_v_pair(cfg, layout="hs")
    S, N, W, T, NT = cfg.H, cfg.N, cfg.d, cfg.tile_tokens, cfg.NT
    cur_d, prev_d = to_dev(cur), to_dev(prev)
    res = []
    for static in (False, True):
        idx, n_act = dev_empty((NT,), "i32"), dev_empty((1,), "i32")
        idx.fill_(-1)
        if static:
            cd.vmajor_select_static(S, N, W, T, cur_d, prev_d, cfg.tau, None, idx, n_act, None, 0)
        else:
            ws = torch.empty(cd.vmajor_select_workspace_bytes(S, N, W, T), dtype=torch.uint8, device="cuda:0")
            cd.vmajor_select(S, N, W, T, cur_d, prev_d, cfg.tau, None, idx, n_act, None, 0, ws)
        _sync()
        res.append((int(n_act.cpu()[0]), idx.cpu().numpy()))
    assert res[0][0] == res[1][0] == cfg.n_changed
    assert np.array_equal(res[0][1], res[1][1]) and np.array_equal(res[0][1][:cfg.n_changed], changed)


def test_select_more_than_one_scan_round(oracle):
    # 2500 tiles: the scan workgroup walks them 1024 at a time
    rng = np.random.default_rng(78)
    S, N, W, T = 1, 2500 * 4, 8, 4
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    prev, changed = perturb_tiles(cur, 1, T, 700, rng, sigma=0.5)
    idx, n = _check_select(oracle, cur, prev, 1e-3, T)
    assert n == len(idx)


def test_select_large_tiles(oracle):
    # a tile of 16 x 3200 values per slab: 6400 vectors per (tile, slab) segment, two slabs
    rng = np.random.default_rng(79)
    S, N, W, T = 2, 160, 3200, 16
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    prev, changed = perturb_tiles(cur, 1, T, 4, rng)
    idx, n = _check_select(oracle, cur, prev, 1e-3, T)
    assert np.array_equal(idx, changed)


def test_select_repeated_calls_reuse_the_workspace(oracle):
    # the status words of one call must not leak into the next: same buffers, different inputs
    import torch
    rng = np.random.default_rng(80)
    S, N, W, T = 4, 4096, 64, 16
    NT = N // T
    ws = torch.empty(cd.vmajor_select_workspace_bytes(S, N, W, T), dtype=torch.uint8, device="cuda:0")
    idx, n_act = dev_empty((NT,), "i32"), dev_empty((1,), "i32")
    compact = dev_empty((S, NT * T, W))
    cur = f32_to_bf16_bits(rng.standard_normal((S, N, W)).astype(np.float32))
    cur_d = to_dev(cur)
    for k in (200, 3, 0, NT, 57):
        prev, changed = perturb_tiles(cur, 1, T, k, rng, sigma=0.5)
        cd.vmajor_select(S, N, W, T, cur_d, to_dev(prev), 1e-3, None, idx, n_act, compact, NT, ws)
        _sync()
        n = int(n_act.cpu()[0])
        assert n == k and np.array_equal(idx.cpu().numpy()[:n], changed)
        got = to_host_bits(compact)
        for j, t in enumerate(changed):
            assert np.array_equal(got[:, j * T:(j + 1) * T], cur[:, t * T:(t + 1) * T])


# ---------------------------------------------------------------------------
# norm + RoPE
# ---------------------------------------------------------------------------

def _norm_rope_case(oracle, cfg, token_ids=None, seed=0):
    rng = np.random.default_rng(300 + cfg.index + seed)
    scale = np.float32(1.7)
    q = f32_to_bf16_bits(rng.standard_normal((cfg.N, cfg.H, cfg.d), dtype=np.float32) * scale)
    k = f32_to_bf16_bits(rng.standard_normal((cfg.N, cfg.H, cfg.d), dtype=np.float32))
    gq = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(cfg.d)).astype(np.float32))
    gk = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(cfg.d)).astype(np.float32))
    rope, table = _rope(cfg)
    qd, kd = to_dev(q), to_dev(k)
    cd.qk_norm_rope(_shape(cfg), qd, kd, to_dev(gq), to_dev(gk), cfg.eps, rope)
    _sync()
    ids = np.arange(cfg.N) if token_ids is None else token_ids
    gq_out, gk_out = to_host_bits(qd)[ids], to_host_bits(kd)[ids]
    oq = oracle.qk_norm_rope(q[ids], ids, gq, cfg.eps, cfg.grid, cfg.pairs, cfg.theta)
    ok = oracle.qk_norm_rope(k[ids], ids, gk, cfg.eps, cfg.grid, cfg.pairs, cfg.theta)
    e1 = assert_float_parity(gq_out, oq, f"norm_rope Q {cfg.name}")
    e2 = assert_float_parity(gk_out, ok, f"norm_rope K {cfg.name}")
    say(f"norm_rope {cfg.name}: {len(ids)} tokens, Q abs/rel {e1[0]:.3g}/{e1[1]:.3g}, K {e2[0]:.3g}/{e2[1]:.3g}")


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_norm_rope_full(oracle, name):
    _norm_rope_case(oracle, CONFIGS[name])


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_norm_rope_sampled_tokens_at_full_size(oracle, name):
    cfg = CONFIGS[name]
    _norm_rope_case(oracle, cfg, sample_token_ids(cfg, random_tiles_per_rank=8))


def test_norm_rope_rank_range_and_single_tensor(oracle):
    cfg = CONFIGS["C1"]
    rng = np.random.default_rng(5)
    q = f32_to_bf16_bits(rng.standard_normal((cfg.N, cfg.H, cfg.d), dtype=np.float32))
    g = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(cfg.d)).astype(np.float32))
    rope, table = _rope(cfg)
    kd = to_dev(q)
    cd.qk_norm_rope(_shape(cfg, 1, 1), None, kd, None, to_dev(g), cfg.eps, rope)   # K only, rank 1 only
    _sync()
    out = to_host_bits(kd)
    assert np.array_equal(out[:cfg.Ns], q[:cfg.Ns])                      # rank 0's rows untouched
    ids = np.arange(cfg.Ns, cfg.N)                                       # global positions of rank 1's tokens
    assert_float_parity(out[ids], oracle.qk_norm_rope(q[ids], ids, g, cfg.eps, cfg.grid, cfg.pairs, cfg.theta))


@pytest.mark.parametrize("N,H,d,grid,pairs", [
    (64, 2, 32, (8, 8), (8, 8)),          # D/8 = 8: eight short tokens per wavefront
    (32, 1, 8, (32,), (4,)),              # one vector per head, one axis
    (48, 8, 64, (2, 4, 6), (10, 11, 11)),  # D/8 = 64; pair split not a multiple of 4
    (96, 16, 256, (12, 8), (64, 64)),     # d/8 = 32: reduction crosses 16-lane rows; D/8 = 512 = 8 steps
    (32, 10, 512, (4, 8), (128, 128)),    # d/8 = 64; D/8 = 640 = 10 steps (generic step loop)
])
def test_norm_rope_other_shapes(oracle, N, H, d, grid, pairs):
    rng = np.random.default_rng(N + d)
    x = f32_to_bf16_bits(rng.standard_normal((N, H, d), dtype=np.float32) * np.float32(3.0))
    g = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    table = to_dev(cd.rope_table(grid, pairs, 10000.0))
    rope = cd.Rope.make(grid, pairs, 10000.0, table.data_ptr())
    xd = to_dev(x)
    cd.qk_norm_rope(cd.Shape.make(N, H * d, H, d, 1), xd, None, to_dev(g), None, 1e-6, rope)
    _sync()
    assert_float_parity(to_host_bits(xd), oracle.qk_norm_rope(x, np.arange(N), g, 1e-6, grid, pairs, 10000.0))


# ---------------------------------------------------------------------------
# projection
# ---------------------------------------------------------------------------

def _proj(cfg_shape, x, wq, wk, wv, N, D):
    xd = to_dev(x)
    outs = []
    for w in (wq, wk, wv):
        if w is None:
            outs.append(None)
        else:
            o = dev_empty((N, D))
            o.fill_(-1)
            outs.append(o)
    cd.qkv_proj(cfg_shape, xd, *(None if w is None else to_dev(w) for w in (wq, wk, wv)), *outs)
    _sync()
    return [None if o is None else to_host_bits(o) for o in outs]


def test_proj_c1_full_all_three(oracle):
    cfg = CONFIGS["C1"]
    inp = make_layer_inputs(cfg)
    q, k, v = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    for got, w in ((q, "Wq"), (k, "Wk"), (v, "Wv")):
        e = assert_float_parity(got, oracle.qkv_proj(inp["X"], inp[w]), f"proj {w}")
        say(f"proj C1 {w}: abs {e[0]:.3g} rel {e[1]:.3g}")


def test_proj_identity_and_small_integers_are_bit_exact(oracle):
    rng = np.random.default_rng(9)
    N, H, d = 272, 5, 64          # 272 tokens: a ragged second token tile; 320 features: a ragged feature tile
    D = H * d
    s = cd.Shape.make(N, D, H, d, 1)
    x = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
    eye = f32_to_bf16_bits(np.eye(D, dtype=np.float32))
    (q,) = [o for o in _proj(s, x, eye, None, None, N, D) if o is not None]
    assert np.array_equal(q, x)
    xi = rng.integers(-8, 9, size=(N, D)).astype(np.float32)
    wi = rng.integers(-8, 9, size=(D, D)).astype(np.float32)
    _, k, _ = _proj(s, f32_to_bf16_bits(xi), None, f32_to_bf16_bits(wi), None, N, D)
    exact = oracle.qkv_proj(f32_to_bf16_bits(xi), f32_to_bf16_bits(wi))
    # |sum| <= 320*64 = 20480 is not always a bf16 value: compare with the exact sum rounded once
    assert np.array_equal(k, f32_to_bf16_bits(exact.astype(np.float32)))


@pytest.mark.parametrize("N,H,d,P", [(16, 1, 8, 1), (48, 3, 40, 3), (528, 9, 64, 1), (256, 2, 264, 2)])
def test_proj_odd_shapes(oracle, N, H, d, P):
    # K = H*d not a multiple of 64 exercises the zero-filled K tail; N, D off the 256 tile grid
    rng = np.random.default_rng(N * 7 + d)
    D = H * d
    x = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
    ws = [f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5)) for _ in range(3)]
    q, k, v = _proj(cd.Shape.make(N, D, H, d, P), x, ws[0], ws[1], ws[2], N, D)
    for got, w in zip((q, k, v), ws):
        assert_float_parity(got, oracle.qkv_proj(x, w), f"proj odd {N}x{D}")


def test_proj_v_first_subsets_and_rank_ranges(oracle):
    cfg = CONFIGS["C1"]
    inp = make_layer_inputs(cfg)
    xd = to_dev(inp["X"])
    wq, wk, wv = to_dev(inp["Wq"]), to_dev(inp["Wk"]), to_dev(inp["Wv"])
    q, k, v = (dev_empty((cfg.N, cfg.D)) for _ in range(3))
    for t in (q, k, v):
        t.fill_(-1)
    cd.qkv_proj(_shape(cfg), xd, None, None, wv, None, None, v)        # V first
    for r in range(cfg.P):                                            # then Q and K, one rank at a time
        cd.qkv_proj(_shape(cfg, r, 1), xd, wq, wk, None, q, k, None)
    _sync()
    q1, k1, v1 = to_host_bits(q), to_host_bits(k), to_host_bits(v)
    q2, k2, v2 = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    # a rank-range call leaves the other ranks' rows alone
    q.fill_(-1)
    cd.qkv_proj(_shape(cfg, 1, 1), xd, wq, None, None, q, None, None)
    _sync()
    part = to_host_bits(q)
    assert np.all(part[:cfg.Ns] == 0xFFFF) and np.array_equal(part[cfg.Ns:], q2[cfg.Ns:])


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_proj_full(oracle, name):
    cfg = CONFIGS[name]
    say(f"proj {name}: every row against the fp64 product")
    inp = make_layer_inputs(cfg)
    q, k, v = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    for got, w in ((q, "Wq"), (k, "Wk"), (v, "Wv")):
        e = assert_float_parity(got, oracle.qkv_proj(inp["X"], inp[w]), f"proj {name} {w}")
        say(f"proj {name} {w}: abs {e[0]:.3g} rel {e[1]:.3g}")


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_proj_sampled_rows_at_full_size(oracle, name):
    cfg = CONFIGS[name]
    say(f"proj {name}: generating inputs")
    inp = make_layer_inputs(cfg)
    ids = sample_token_ids(cfg, random_tiles_per_rank=(6 if name != "C5" else 2))
    q, k, v = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    for got, w in ((q, "Wq"), (k, "Wk"), (v, "Wv")):
        e = assert_float_parity(got[ids], oracle.qkv_proj(inp["X"][ids], inp[w]), f"proj {name} {w}")
        say(f"proj {name} {w}: {len(ids)} sampled rows, abs {e[0]:.3g} rel {e[1]:.3g}")


def test_proj_ragged_edges_of_the_288_token_tile(oracle):
    """9200 tokens x 3008 features, one weight: 512 tiles of 288 x 192 are two rounds of the compute units where 432
    square tiles are 1.69, so the host picks the 288 x 192 tile; its last token tile has 272 of 288 rows and its last
    feature tile 128 of 192 columns.  Rows around both edges against the oracle, and nothing written past the end."""
    import torch
    N, H, d = 9200, 47, 64
    D = H * d
    rng = np.random.default_rng(2881)
    x = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
    w = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    out = torch.full((N + 16, D), -1, dtype=torch.int16, device="cuda:0")
    say("proj 9200 x 3008: launch")
    cd.qkv_proj(cd.Shape.make(N, D, H, d, 1), to_dev(x), None, None, to_dev(w), None, None, out[:N])
    _sync()
    got = to_host_bits(out)
    assert np.all(got[N:] == 0xFFFF), "rows past the last token were written"
    ids = np.concatenate([np.arange(0, 8), np.arange(280, 296), np.arange(8920, 8936), np.arange(N - 24, N),
                          rng.choice(N, size=64, replace=False)])
    e = assert_float_parity(got[ids], oracle.qkv_proj(x[ids], w), "proj 288-token tile")
    say(f"proj 9200 x 3008: {len(ids)} rows, abs {e[0]:.3g} rel {e[1]:.3g}")
    # the same through the exchange-buffer epilogue: identical bits after a pack of the plain result
    sh = cd.Shape.make(N, D, H, d, 1)
    buf_direct = torch.full((N * D + 64,), -1, dtype=torch.int16, device="cuda:0")
    buf_packed = dev_empty((N * D,))
    cd.qkv_proj_pack(sh, to_dev(x), None, None, to_dev(w), None, None, buf_direct[:N * D], cd.RECV_MAJOR)
    cd.a2a_pack(sh, out[:N], buf_packed, cd.RECV_MAJOR)
    _sync()
    assert torch.equal(buf_direct[:N * D], buf_packed) and bool((buf_direct[N * D:] == -1).all().cpu())


def test_proj_ragged_edges_of_the_256_token_tile(oracle):
    """20720 tokens x 3008 features, one weight: 972 tiles of 256 x 256 are four rounds of the compute units, fewer
    tile-rounds x area than the other shapes, so the host takes the 256 x 256 tile (asserted through the plan query)
    -- the tile the two largest workloads run on, there on exact multiples of 256.  Here its last token tile has 240
    of 256 rows and its last feature tile 192 of 256 columns.  Rows around both edges and random rows against the
    oracle, every feature; nothing written past the end; both epilogues."""
    import torch
    N, H, d = 20720, 47, 64
    D = H * d
    sh = cd.Shape.make(N, D, H, d, 1)
    plan = cd.qkv_proj_plan(sh, 1)
    say(f"proj 20720 x 3008: plan {plan}")
    assert (plan["tile_tokens"], plan["tile_features"]) == (256, 256), plan
    rng = np.random.default_rng(2561)
    x = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
    w = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    out = torch.full((N + 16, D), -1, dtype=torch.int16, device="cuda:0")
    xd, wd = to_dev(x), to_dev(w)
    say("proj 20720 x 3008: launch")
    cd.qkv_proj(sh, xd, None, None, wd, None, None, out[:N])
    _sync()
    got = to_host_bits(out)
    assert np.all(got[N:] == 0xFFFF), "rows past the last token were written"
    ids = np.concatenate([np.arange(0, 8), np.arange(248, 264), np.arange(20472, 20488), np.arange(N - 24, N),
                          rng.choice(N, size=96, replace=False)])
    e = assert_float_parity(got[ids], oracle.qkv_proj(x[ids], w), "proj 256-token tile")
    say(f"proj 20720 x 3008: {len(ids)} rows x {D} features, abs {e[0]:.3g} rel {e[1]:.3g}")
    # the exchange-buffer epilogue: identical bits after a pack of the plain result, nothing past the end
    buf_direct = torch.full((N * D + 64,), -1, dtype=torch.int16, device="cuda:0")
    buf_packed = dev_empty((N * D,))
    cd.qkv_proj_pack(sh, xd, None, None, wd, None, None, buf_direct[:N * D], cd.RECV_MAJOR)
    cd.a2a_pack(sh, out[:N], buf_packed, cd.RECV_MAJOR)
    _sync()
    assert torch.equal(buf_direct[:N * D], buf_packed) and bool((buf_direct[N * D:] == -1).all().cpu())


# ---------------------------------------------------------------------------
# the whole path, two streams (V first), against the oracle chain
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_chain_v_first_two_streams(oracle, name):
    import torch
    cfg = CONFIGS[name]
    inp = make_layer_inputs(cfg)
    dev = {k_: to_dev(v_) for k_, v_ in inp.items()}
    rope, table = _rope(cfg)
    sh = _shape(cfg)
    q, k, v = (dev_empty((cfg.N, cfg.D)) for _ in range(3))
    bq, bk, bv = (dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d)) for _ in range(3))
    hq, hk, hv = (dev_empty((cfg.H, cfg.N, cfg.d)) for _ in range(3))
    sv, sqk = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    # stream V: projection of V alone, pack, unpack
    cd.qkv_proj(sh, dev["X"], None, None, dev["Wv"], None, None, v, stream=sv)
    cd.a2a_pack(sh, v, bv, cd.RECV_MAJOR, stream=sv)
    cd.a2a_unpack(sh, bv, hv, cd.RECV_MAJOR, stream=sv)
    # stream QK: projection of Q and K, norm + RoPE, pack, unpack
    cd.qkv_proj(sh, dev["X"], dev["Wq"], dev["Wk"], None, q, k, None, stream=sqk)
    cd.qk_norm_rope(sh, q, k, dev["gamma_q"], dev["gamma_k"], cfg.eps, rope, stream=sqk)
    for src, buf, dst in ((q, bq, hq), (k, bk, hk)):
        cd.a2a_pack(sh, src, buf, cd.RECV_MAJOR, stream=sqk)
        cd.a2a_unpack(sh, buf, dst, cd.RECV_MAJOR, stream=sqk)
    torch.cuda.synchronize()

    ids = np.arange(cfg.N)
    # the layout change itself is bit-exact on the GPU's own upstream output
    for seq, hs in ((q, hq), (k, hk), (v, hv)):
        assert np.array_equal(to_host_bits(hs), to_host_bits(seq).reshape(cfg.N, cfg.H, cfg.d).transpose(1, 0, 2))
    # End to end against the unrounded fp64 chain.  The GPU rounds to bf16 twice on the Q/K path (after
    # the projection and after norm + RoPE); a relative error 2^-9 in the projection moves a normalised
    # element by at most 2 * 2^-9 of its size (itself and the row's RMS), the rotation adds the two
    # elements of a pair, and the last rounding adds 2^-9 of the result:
    #   |err| <= 2^-8 * sqrt(2) * |pair| + 2^-9 * |o| + 1e-3     (|pair| = norm of the rotary pair)
    o_v = oracle.qkv_proj(inp["X"], inp["Wv"]).reshape(cfg.N, cfg.H, cfg.d)
    assert_float_parity(to_host_bits(hv), o_v.transpose(1, 0, 2), "chain V")
    for name_t, w, g, got in (("Q", "Wq", "gamma_q", hq), ("K", "Wk", "gamma_k", hk)):
        o = oracle.rope_rotate(oracle.rms_norm(oracle.qkv_proj(inp["X"], inp[w]).reshape(cfg.N, cfg.H, cfg.d),
                                               oracle.widen(inp[g]), cfg.eps), ids, cfg.grid, cfg.pairs, cfg.theta)
        pair = np.sqrt(o[..., 0::2] ** 2 + o[..., 1::2] ** 2)
        bound = 2.0 ** -8 * np.sqrt(2.0) * np.repeat(pair, 2, axis=-1) + 2.0 ** -9 * np.abs(o) + 1e-3
        err = np.abs(oracle.widen(to_host_bits(got)) - o.transpose(1, 0, 2))
        ratio = float((err / bound.transpose(1, 0, 2)).max())
        rel = float((err / np.maximum(np.abs(o.transpose(1, 0, 2)), 1.0)).max())
        say(f"chain {name} {name_t}: max abs err {err.max():.3g}, max rel (floored) {rel:.3g}, worst err/bound {ratio:.3g}")
        assert ratio <= 1.0

    # V-Major selection on the GPU's own head-parallel V against a perturbed previous step
    v_cur = to_host_bits(hv)
    rng = np.random.default_rng(400 + cfg.index)
    v_prev, changed = perturb_tiles(v_cur, 1, cfg.tile_tokens, cfg.n_changed, rng, cfg.noise_sigma)
    idx, n = _check_select(oracle, v_cur, v_prev, cfg.tau, cfg.tile_tokens)
    assert np.array_equal(idx, changed)


def test_two_runs_are_bit_identical(oracle):
    cfg = CONFIGS["C2"]
    inp = make_layer_inputs(cfg)
    a = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    b = _proj(_shape(cfg), inp["X"], inp["Wq"], inp["Wk"], inp["Wv"], cfg.N, cfg.D)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    cur, prev, _ = make_v_pair(cfg)
    r1 = _run_select(cur, prev, cfg.tau, cfg.tile_tokens)
    r2 = _run_select(cur, prev, cfg.tau, cfg.tile_tokens)
    assert r1[2] == r2[2] and np.array_equal(r1[1][:r1[2]], r2[1][:r2[2]]) and np.array_equal(r1[0], r2[0])
    assert np.array_equal(r1[3][:, :r1[2] * cfg.tile_tokens], r2[3][:, :r2[2] * cfg.tile_tokens])


# ---------------------------------------------------------------------------
# no entry point writes outside its outputs
# ---------------------------------------------------------------------------

def test_outputs_are_written_inside_their_bounds_only(oracle):
    """Every output sits between two guard bands inside one larger allocation; after the calls the bands still hold
    their fill pattern.  Shapes off the tile grid (528 tokens, D = 512) and the tiny workload."""
    import torch
    GUARD = 4096                                       # int16 elements on either side

    class Guarded:
        def __init__(self, n_elems, dtype=torch.int16):
            self.raw = torch.full((n_elems + 2 * GUARD,), 0x5A5A if dtype == torch.int16 else 0x5A5A5A5A, dtype=dtype, device="cuda:0")
            self.t = self.raw[GUARD:GUARD + n_elems]
            self.fill = int(self.raw[0].cpu())

        def intact(self):
            r = self.raw.cpu().numpy()
            return bool(np.all(r[:GUARD] == self.fill) and np.all(r[-GUARD:] == self.fill))

    for N, H, d, P, grid, pairs in ((528, 8, 64, 1, (22, 24), (16, 16)), (256, 4, 64, 2, (16, 16), (16, 16))):
        D, T = H * d, 16
        NT = N // T
        sh = cd.Shape.make(N, D, H, d, P)
        rng = np.random.default_rng(N)
        x = to_dev(f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32)))
        w = to_dev(f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5)))
        g = to_dev(f32_to_bf16_bits(np.ones(d, dtype=np.float32)))
        table = torch.from_numpy(cd.rope_table(grid, pairs, 10000.0)).to("cuda:0")
        rope = cd.Rope.make(grid, pairs, 10000.0, table.data_ptr())
        outs = {k_: Guarded(N * D) for k_ in ("q", "k", "v", "bq", "bk", "bv", "hq", "hk", "hv", "compact", "seq2")}
        ints = {k_: Guarded(n_, torch.int32) for k_, n_ in (("flags", NT), ("idx", NT), ("n", 1), ("tok_idx", N), ("tok_n", P))}
        metric = Guarded(N, torch.float32)
        ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")
        o = {k_: v_.t for k_, v_ in outs.items()}
        i_ = {k_: v_.t for k_, v_ in ints.items()}
        cd.qkv_proj(sh, x, w, w, w, o["q"], o["k"], o["v"])
        cd.qk_norm_rope(sh, o["q"], o["k"], g, g, 1e-6, rope)
        cd.a2a_pack(sh, o["v"], o["bv"], cd.RECV_MAJOR)
        cd.a2a_unpack(sh, o["bv"], o["hv"], cd.RECV_MAJOR)
        cd.qkv_proj_pack(sh, x, w, w, None, o["bq"], o["bk"], None, cd.RECV_MAJOR)
        cd.a2a_unpack_norm_rope(sh, o["bq"], o["bk"], o["hq"], o["hk"], g, g, 1e-6, rope, cd.RECV_MAJOR)
        cd.qk_norm_rope_pack(sh, o["q"], o["k"], g, g, 1e-6, rope, o["bq"], o["bk"], cd.SEND_MAJOR)
        prev = o["hq"]                                  # any tensor of the right shape: most tiles differ
        cd.vmajor_select(H, N, d, T, o["hv"], prev, 1e-3, i_["flags"], i_["idx"], i_["n"], o["compact"], NT, ws)
        cd.a2a_unpack_select(sh, o["bv"], cd.RECV_MAJOR, o["hv"], prev, T, 1e-3, i_["flags"], i_["idx"], i_["n"], o["compact"], NT, ws)
        cd.vmajor_gather(H, N, d, T, o["hv"], i_["idx"], i_["n"], o["compact"], NT)
        cd.vmajor_scatter(H, N, d, T, o["compact"], i_["idx"], i_["n"], o["hk"], NT)
        cd.a2a_pack_hs(sh, o["hv"], o["bv"], cd.SEND_MAJOR)
        cd.a2a_unpack_seq(sh, o["bv"], o["seq2"], cd.SEND_MAJOR)
        cd.vmajor_token_metric(H, N, d, o["hv"], prev, metric.t)
        cd.vmajor_topk(P, N // P, metric.t, (N // P) // 3, i_["tok_idx"], i_["tok_n"], global_ids=True)
        _sync()
        for name, gd in list(outs.items()) + list(ints.items()) + [("metric", metric)]:
            assert gd.intact(), (N, name)
