"""GPU parity for the rows after the hot path: V-Major gather / scatter (Section III-D, sender-side extraction
and receiver-side reconstruction) and the second all-to-all (Section II-A).  All byte work: bit-exact."""
import numpy as np
import pytest

import paper_2604_14561_amd as cd
from parity_util import assert_float_parity, dev_empty, to_dev, to_host_bits
from synth import CONFIGS, make_v_pair

gpu = pytest.mark.gpu


def _sync():
    import torch
    torch.cuda.synchronize()


def _shape(cfg, rank_begin=0, rank_count=None):
    return cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, rank_begin, rank_count)


@gpu
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_second_all_to_all_bit_exact_and_round_trip(oracle, name):
    cfg = CONFIGS[name]
    print(f"second all-to-all {name}", flush=True)
    rng = np.random.default_rng(500 + cfg.index)
    y = rng.integers(0, 65536, size=(cfg.H, cfg.N, cfg.d), dtype=np.uint16)
    yd = to_dev(y)
    for order in (cd.SEND_MAJOR, cd.RECV_MAJOR):
        buf = dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d))
        buf.fill_(-1)
        seq = dev_empty((cfg.N, cfg.H, cfg.d))
        seq.fill_(-1)
        cd.a2a_pack_hs(_shape(cfg), yd, buf, order)
        cd.a2a_unpack_seq(_shape(cfg), buf, seq, order)
        _sync()
        want_buf = oracle.a2a_pack_hs(y, cfg.P, order)
        assert np.array_equal(to_host_bits(buf), want_buf)
        got = to_host_bits(seq)
        assert np.array_equal(got, oracle.a2a_unpack_seq(want_buf, cfg.N, cfg.H, cfg.d, cfg.P, order))
        assert np.array_equal(got, y.transpose(1, 0, 2))
        del buf
    # literal round trip: first all-to-all on what came back gives the head-parallel tensor again
    buf = dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d))
    hs = dev_empty((cfg.H, cfg.N, cfg.d))
    cd.a2a_pack(_shape(cfg), seq, buf, cd.RECV_MAJOR)
    cd.a2a_unpack(_shape(cfg), buf, hs, cd.RECV_MAJOR)
    _sync()
    assert np.array_equal(to_host_bits(hs), y)


@gpu
def test_second_all_to_all_rank_ranges(oracle):
    cfg = CONFIGS["C2"]
    rng = np.random.default_rng(7)
    y = rng.integers(0, 65536, size=(cfg.H, cfg.N, cfg.d), dtype=np.uint16)
    yd = to_dev(y)
    buf = dev_empty((cfg.P * cfg.P, cfg.Ns, cfg.Hp, cfg.d))
    buf.fill_(-1)
    for p in reversed(range(cfg.P)):            # one head owner at a time
        cd.a2a_pack_hs(_shape(cfg, p, 1), yd, buf, cd.SEND_MAJOR)
    _sync()
    assert np.array_equal(to_host_bits(buf), oracle.a2a_pack_hs(y, cfg.P, 0))
    seq = dev_empty((cfg.N, cfg.H, cfg.d))
    seq.fill_(-1)
    cd.a2a_unpack_seq(_shape(cfg, 3, 4), buf, seq, cd.SEND_MAJOR)
    _sync()
    got = to_host_bits(seq)
    assert np.all(got[:3 * cfg.Ns] == 0xFFFF) and np.all(got[7 * cfg.Ns:] == 0xFFFF)
    assert np.array_equal(got[3 * cfg.Ns:7 * cfg.Ns], y.transpose(1, 0, 2)[3 * cfg.Ns:7 * cfg.Ns])


@gpu
@pytest.mark.parametrize("name", ["C1", "C3", "C4", "C5"])
def test_gather_and_scatter_close_the_selection_loop(oracle, name):
    import torch
    cfg = CONFIGS[name]
    print(f"gather/scatter {name}", flush=True)
    T, NT = cfg.tile_tokens, cfg.NT
    cur, prev, changed = make_v_pair(cfg, layout="hs")
    cur_d, prev_d = to_dev(cur), to_dev(prev)
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(cfg.H, cfg.N, cfg.d, T), 16), dtype=torch.uint8, device="cuda:0")
    idx, n_act = dev_empty((NT,), "i32"), dev_empty((1,), "i32")
    cd.vmajor_select(cfg.H, cfg.N, cfg.d, T, cur_d, prev_d, cfg.tau, None, idx, n_act, None, 0, ws)
    # sender: gather the active tiles of another tensor (stands for Q or K) by V's list, without reading it on the host
    rng = np.random.default_rng(600 + cfg.index)
    q = rng.integers(0, 65536, size=(cfg.H, cfg.N, cfg.d), dtype=np.uint16)
    cap = cfg.n_changed + 3
    q_act = dev_empty((cfg.H, cap * T, cfg.d))
    q_act.fill_(-1)
    cd.vmajor_gather(cfg.H, cfg.N, cfg.d, T, to_dev(q), idx, n_act, q_act, cap)
    # receiver: overwrite its cached copy
    q_cache = rng.integers(0, 65536, size=(cfg.H, cfg.N, cfg.d), dtype=np.uint16)
    cache_d = to_dev(q_cache)
    cd.vmajor_scatter(cfg.H, cfg.N, cfg.d, T, q_act, idx, n_act, cache_d, cap)
    # and V itself: gather + scatter into the previous step's V must rebuild the current V
    v_act = dev_empty((cfg.H, cap * T, cfg.d))
    cd.vmajor_gather(cfg.H, cfg.N, cfg.d, T, cur_d, idx, n_act, v_act, cap)
    cd.vmajor_scatter(cfg.H, cfg.N, cfg.d, T, v_act, idx, n_act, prev_d, cap)
    _sync()
    n = int(n_act.cpu()[0])
    assert n == cfg.n_changed
    want_act = oracle.vmajor_gather(q, changed, T, cap_tiles=cap)
    got_act = to_host_bits(q_act)
    assert np.array_equal(got_act[:, :n * T], want_act[:, :n * T])
    assert np.all(got_act[:, n * T:] == 0xFFFF)                       # rows beyond the list are not written
    assert np.array_equal(to_host_bits(cache_d), oracle.vmajor_scatter(want_act, changed, q_cache, T))
    assert np.array_equal(to_host_bits(prev_d), cur)


@gpu
def test_gather_scatter_edge_cases(oracle):
    rng = np.random.default_rng(9)
    S, N, W, T = 3, 1280, 40, 16
    NT = N // T
    x = rng.integers(0, 65536, size=(S, N, W), dtype=np.uint16)
    cache = rng.integers(0, 65536, size=(S, N, W), dtype=np.uint16)

    def run(idx_list, n, cap):
        idx = np.full(NT, -5, dtype=np.int32)
        idx[:len(idx_list)] = idx_list
        idx_d, n_d = to_dev(idx), to_dev(np.array([n], dtype=np.int32))
        comp = dev_empty((S, cap * T, W))
        comp.fill_(-1)
        cd.vmajor_gather(S, N, W, T, to_dev(x), idx_d, n_d, comp, cap)
        c_d = to_dev(cache)
        cd.vmajor_scatter(S, N, W, T, comp, idx_d, n_d, c_d, cap)
        _sync()
        return to_host_bits(comp), to_host_bits(c_d)

    # empty list: nothing moves
    comp, c = run([], 0, 4)
    assert np.all(comp == 0xFFFF) and np.array_equal(c, cache)
    # capacity smaller than the list: only the first cap tiles move
    lst = [0, 7, 79, 33]
    comp, c = run(lst, 4, 2)
    want = oracle.vmajor_gather(x, np.array(lst, np.int32), T, cap_tiles=2)
    assert np.array_equal(comp, want)
    assert np.array_equal(c, oracle.vmajor_scatter(want, np.array(lst, np.int32), cache, T))
    # full list in arbitrary order, first and last tile included
    lst = [79, 0, 41]
    comp, c = run(lst, 3, 3)
    want = oracle.vmajor_gather(x, np.array(lst, np.int32), T, cap_tiles=3)
    assert np.array_equal(comp, want) and np.array_equal(c, oracle.vmajor_scatter(want, np.array(lst, np.int32), cache, T))
    # an entry outside the tile range is skipped, not dereferenced
    comp, c = run([5, 4000, -1, 6], 4, 4)
    assert np.array_equal(comp[:, :T], x[:, 5 * T:6 * T]) and np.array_equal(comp[:, 3 * T:4 * T], x[:, 6 * T:7 * T])
    assert np.all(comp[:, T:3 * T] == 0xFFFF)


@gpu
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_token_metric_and_topk(oracle, name):
    import torch
    cfg = CONFIGS[name]
    print(f"token metric / top-k {name}", flush=True)
    cur, prev, changed = make_v_pair(cfg, layout="hs")
    # make the metric non-trivial everywhere: a second, smaller perturbation on every token of some random tiles
    from synth import perturb_tiles
    prev, _ = perturb_tiles(prev, 1, 1, cfg.N // 3, np.random.default_rng(cfg.index), sigma=0.01)
    N = cfg.N
    metric = torch.empty(N, dtype=torch.float32, device="cuda:0")
    cd.vmajor_token_metric(cfg.H, N, cfg.d, to_dev(cur), to_dev(prev), metric)
    _sync()
    got = metric.cpu().numpy()
    want = oracle.token_l1_metric(cur, prev)
    # fp32 accumulation of 3072 non-negative terms against the fp64 sum
    assert np.all(np.abs(got - want) <= 1e-4 * np.maximum(want, 1e-3)), float(np.max(np.abs(got - want)))
    # the integer decision is taken on the metric the GPU produced (fp32), on both sides
    idx, n_act = dev_empty((N,), "i32"), dev_empty((1,), "i32")
    for step in (3, 6, 20, 27, 49):
        k = cd.cache_active_count(step, 50, 5, 10, N)
        assert k == oracle.active_count(step, 50, 5, 10, N)
        idx.fill_(-1)
        cd.vmajor_topk(1, N, metric, k, idx, n_act)
        _sync()
        assert int(n_act.cpu()[0]) == k
        got_list = idx.cpu().numpy()[:k]
        assert np.array_equal(got_list, oracle.topk_active(got, k))
        # ... and against the oracle's own set from the same INPUTS (fp64 metric): the two sets may differ only in
        # tokens whose fp64 metric lies within the fp32 accumulation error of the cut (the smallest active metric)
        want_list = oracle.topk_active(want, k)
        if 0 < k < N:
            cut = np.sort(want)[N - k]
            differ = np.setxor1d(got_list, want_list)
            assert np.all(np.abs(want[differ] - cut) <= 2e-4 * max(cut, 1e-3)), (step, len(differ))
            assert len(differ) <= 0.01 * N, (step, len(differ))
        else:
            assert np.array_equal(got_list, want_list)
    # one segment per logical rank: each rank ranks its own N/P tokens, ids local to the rank
    P, Ns = cfg.P, cfg.N // cfg.P
    n_act = dev_empty((P,), "i32")
    for step in (6, 27, 50):
        k = cd.cache_active_count(step, 50, 5, 10, Ns)
        idx.fill_(-1)
        cd.vmajor_topk(P, Ns, metric, k, idx, n_act)
        _sync()
        assert np.all(n_act.cpu().numpy() == k)
        rows = idx.cpu().numpy().reshape(P, Ns)
        for r in range(P):
            assert np.array_equal(rows[r, :k], oracle.topk_active(got[r * Ns:(r + 1) * Ns], k)), (step, r)
            assert np.all(rows[r, k:] == -1)


@gpu
def test_topk_ties_nan_and_extremes(oracle):
    import torch
    rng = np.random.default_rng(44)
    N = 5000
    m = rng.integers(0, 6, size=N).astype(np.float32)          # heavy ties
    m[17] = np.nan
    m[4000] = np.inf
    m[3] = -0.0
    md = torch.from_numpy(m).to("cuda:0")
    idx, n_act = dev_empty((N,), "i32"), dev_empty((1,), "i32")
    for k in (0, 1, 2, 3, 777, 2500, N - 1, N):
        cd.vmajor_topk(1, N, md, k, idx, n_act)
        _sync()
        assert int(n_act.cpu()[0]) == k
        assert np.array_equal(idx.cpu().numpy()[:k], oracle.topk_active(m.astype(np.float64), k)), k
    # a segment too long for the LDS key cache: the variant that reads the metric again on every pass
    NL = 40000
    ml = rng.integers(0, 1000, size=NL).astype(np.float32) * 0.25
    mld = torch.from_numpy(ml).to("cuda:0")
    idx_l, n_l = dev_empty((NL,), "i32"), dev_empty((1,), "i32")
    for k in (1, 9999, NL - 1, NL):
        cd.vmajor_topk(1, NL, mld, k, idx_l, n_l)
        _sync()
        assert np.array_equal(idx_l.cpu().numpy()[:k], oracle.topk_active(ml.astype(np.float64), k)), k
    # token-granular gather by the list: tile_tokens = 1
    S, W = 2, 16
    x = rng.integers(0, 65536, size=(S, N, W), dtype=np.uint16)
    k = 123
    cd.vmajor_topk(1, N, md, k, idx, n_act)
    comp = dev_empty((S, k, W))
    cd.vmajor_gather(S, N, W, 1, to_dev(x), idx, n_act, comp, k)
    _sync()
    assert np.array_equal(to_host_bits(comp), x[:, oracle.topk_active(m.astype(np.float64), k), :])


# ---------------------------------------------------------------------------
# fusions: projection -> exchange buffer, norm + RoPE -> exchange buffer
# ---------------------------------------------------------------------------

@gpu
@pytest.mark.parametrize("name,order", [("C1", 0), ("C1", 1), ("C2", 1), ("C3", 1), ("C4", 0), ("C5", 0)])
def test_proj_pack_equals_proj_then_pack(oracle, name, order):
    cfg = CONFIGS[name]
    print(f"proj_pack {name} order {order}", flush=True)
    from synth import make_layer_inputs, sample_token_ids
    inp = make_layer_inputs(cfg)
    sh = cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P)
    X, Wq, Wv = to_dev(inp["X"]), to_dev(inp["Wq"]), to_dev(inp["Wv"])
    q, v = dev_empty((cfg.N, cfg.D)), dev_empty((cfg.N, cfg.D))
    bq, bv, fq, fv = (dev_empty((cfg.N * cfg.D,)) for _ in range(4))
    cd.qkv_proj(sh, X, Wq, None, Wv, q, None, v)
    cd.a2a_pack(sh, q, bq, order)
    cd.a2a_pack(sh, v, bv, order)
    for t in (fq, fv):
        t.fill_(-1)
    cd.qkv_proj_pack(sh, X, Wq, None, Wv, fq, None, fv, order)
    _sync()
    assert np.array_equal(to_host_bits(fq), to_host_bits(bq)) and np.array_equal(to_host_bits(fv), to_host_bits(bv))
    # and against the oracle: pack(round_bf16(fp64 projection)) on sampled tokens, within the float tolerance
    ids = np.arange(cfg.N) if name in ("C1", "C2") else sample_token_ids(cfg, random_tiles_per_rank=2)
    hs = dev_empty((cfg.H, cfg.N, cfg.d))
    cd.a2a_unpack(sh, fv, hs, order)
    _sync()
    got = to_host_bits(hs).transpose(1, 0, 2).reshape(cfg.N, cfg.D)[ids]
    assert_float_parity(got, oracle.qkv_proj(inp["X"][ids], inp["Wv"]), f"proj_pack {name}")
    # a rank range writes only that range's chunks
    fq.fill_(-1)
    r0 = cfg.P - 1
    cd.qkv_proj_pack(cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, r0, 1), X, Wq, None, None, fq, None, None, order)
    _sync()
    part, full = to_host_bits(fq).reshape(cfg.P, cfg.P, -1), to_host_bits(bq).reshape(cfg.P, cfg.P, -1)
    mine = np.zeros((cfg.P, cfg.P), dtype=bool)
    if order == cd.SEND_MAJOR:
        mine[r0, :] = True
    else:
        mine[:, r0] = True
    assert np.array_equal(part[mine], full[mine]) and np.all(part[~mine] == 0xFFFF)


@gpu
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_proj_hs_equals_proj_pack_unpack(oracle, name):
    """The projection with the head-parallel epilogue against projection -> pack -> unpack (bit-identical), against the
    oracle on sampled tokens, and on a rank range (only that range's token rows of every head are written)."""
    cfg = CONFIGS[name]
    print(f"proj_hs {name}", flush=True)
    from synth import make_layer_inputs, sample_token_ids
    inp = make_layer_inputs(cfg)
    N, D, H, d, P = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P
    sh = cd.Shape.make(N, D, H, d, P)
    X, Wk, Wv = to_dev(inp["X"]), to_dev(inp["Wk"]), to_dev(inp["Wv"])
    k, v = dev_empty((N, D)), dev_empty((N, D))
    buf = dev_empty((N * D,))
    hk, hv, fk, fv = (dev_empty((H, N, d)) for _ in range(4))
    cd.qkv_proj(sh, X, None, Wk, Wv, None, k, v)
    for src, dst in ((k, hk), (v, hv)):
        cd.a2a_pack(sh, src, buf, cd.RECV_MAJOR)
        cd.a2a_unpack(sh, buf, dst, cd.RECV_MAJOR)
    for t in (fk, fv):
        t.fill_(-1)
    cd.qkv_proj_hs(sh, X, None, Wk, Wv, None, fk, fv)
    _sync()
    assert np.array_equal(to_host_bits(fk), to_host_bits(hk)) and np.array_equal(to_host_bits(fv), to_host_bits(hv))
    ids = np.arange(N) if name in ("C1", "C2") else sample_token_ids(cfg, random_tiles_per_rank=2)
    got = to_host_bits(fv).transpose(1, 0, 2).reshape(N, D)[ids]
    assert_float_parity(got, oracle.qkv_proj(inp["X"][ids], inp["Wv"]), f"proj_hs {name}")
    # one rank alone: its tokens' rows in every head, nothing else
    fk.fill_(-1)
    r0 = P // 2
    cd.qkv_proj_hs(cd.Shape.make(N, D, H, d, P, r0, 1), X, None, Wk, None, None, fk, None)
    _sync()
    part, full = to_host_bits(fk), to_host_bits(hk)
    rows = slice(r0 * cfg.Ns, (r0 + 1) * cfg.Ns)
    assert np.array_equal(part[:, rows], full[:, rows])
    assert np.all(part[:, :r0 * cfg.Ns] == 0xFFFF) and np.all(part[:, (r0 + 1) * cfg.Ns:] == 0xFFFF)


@gpu
def test_proj_hs_off_grid_shapes_and_bounds(oracle):
    """Shapes off the tile grid (ragged token and feature tiles, K not a multiple of 64 on the general kernel), with
    guard bands around the head-parallel output."""
    import torch
    from synth import f32_to_bf16_bits
    for N, H, d, P in ((272, 5, 64, 1), (528, 9, 64, 1), (48, 3, 40, 3), (9200, 47, 64, 1)):
        D = H * d
        rng = np.random.default_rng(N + d)
        x = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
        w = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
        sh = cd.Shape.make(N, D, H, d, P)
        G = 4096
        raw = torch.full((N * D + 2 * G,), 0x5A5A, dtype=torch.int16, device="cuda:0")
        out_hs = raw[G:G + N * D]
        seq = dev_empty((N, D))
        xd, wd = to_dev(x), to_dev(w)
        cd.qkv_proj_hs(sh, xd, wd, None, None, out_hs, None, None)
        cd.qkv_proj(sh, xd, wd, None, None, seq, None, None)
        _sync()
        r = raw.cpu().numpy()
        assert np.all(r[:G] == 0x5A5A) and np.all(r[-G:] == 0x5A5A), (N, D)
        want = to_host_bits(seq).reshape(N, H, d).transpose(1, 0, 2)
        assert np.array_equal(to_host_bits(out_hs).reshape(H, N, d), want), (N, D)
        ids = np.concatenate([np.arange(0, 8), np.arange(N - 8, N)])
        assert_float_parity(to_host_bits(seq)[ids], oracle.qkv_proj(x[ids], w), f"proj {N}x{D}")


# ---------------------------------------------------------------------------
# the sender's whole share in the projection kernel: norm + RoPE on the accumulators, both destinations
# ---------------------------------------------------------------------------

def _fused_case(oracle, N, D, H, d, P, grid, pairs, inp, ids, rank=None, what=""):
    """Runs cocodiff_qkv_proj_fused (Q, K, V in one launch, both destinations) and checks: V bit-identical to the plain
    projection; both destinations of every tensor hold the same bits; Q and K against the fp64 chain
    projection -> RMSNorm -> RoPE within the float tolerance (one rounding: the tolerance of a single stage holds end to
    end), and close to the twice-rounded stand-alone chain."""
    import torch
    from parity_util import widen_bits
    sh = cd.Shape.make(N, D, H, d, P) if rank is None else cd.Shape.make(N, D, H, d, P, rank, 1)
    full = cd.Shape.make(N, D, H, d, P)
    table = torch.from_numpy(cd.rope_table(grid, pairs, 10000.0)).to("cuda:0")
    rope = cd.Rope.make(grid, pairs, 10000.0, table.data_ptr())
    X, Wq, Wk, Wv = (to_dev(inp[k_]) for k_ in ("X", "Wq", "Wk", "Wv"))
    gq, gk = to_dev(inp["gamma_q"]), to_dev(inp["gamma_k"])
    eps = 1e-6
    bufs = [dev_empty((N * D,)) for _ in range(3)]
    hss = [dev_empty((H, N, d)) for _ in range(3)]
    for t in bufs + hss:
        t.fill_(-1)
    cd.qkv_proj_fused(sh, X, Wq, Wk, Wv, gq, gk, eps, rope, bufs[0], bufs[1], bufs[2], cd.RECV_MAJOR, hss[0], hss[1], hss[2])
    # the stand-alone chain on the same rank range
    q, k, v = (dev_empty((N, D)) for _ in range(3))
    for t in (q, k, v):
        t.fill_(-1)
    cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v)
    _sync()
    v_plain = to_host_bits(v).copy()
    have_chain = True
    try:
        cd.qk_norm_rope(sh, q, k, gq, gk, eps, rope)
    except cd.CocodiffError:          # the stand-alone kernel takes fewer shapes (D/8 must divide or be a multiple of 64)
        have_chain = False
    _sync()
    rows = slice(0, N) if rank is None else slice(rank * (N // P), (rank + 1) * (N // P))
    for name, buf, hs, seq in (("Q", bufs[0], hss[0], q), ("K", bufs[1], hss[1], k), ("V", bufs[2], hss[2], v)):
        got_hs = to_host_bits(hs)                                     # [H][N][d]
        # destination 2 == unpack(destination 1), and nothing outside the rank range was written
        un = dev_empty((H, N, d))
        un.fill_(-1)
        cd.a2a_unpack(full, buf, un, cd.RECV_MAJOR)
        _sync()
        un_h = to_host_bits(un)
        assert np.array_equal(un_h[:, rows], got_hs[:, rows]), f"{what} {name}: the two destinations differ"
        if rank is not None:
            outside = np.ones(N, dtype=bool)
            outside[rows] = False
            assert np.all(got_hs[:, outside] == 0xFFFF), f"{what} {name}: rows outside the rank range were written"
        got_seq = got_hs.transpose(1, 0, 2).reshape(N, D)
        chain = to_host_bits(seq)
        if name == "V":
            assert np.array_equal(got_seq[rows], v_plain[rows]), f"{what}: V differs from the plain projection"
            continue
        # against the oracle chain (fp64, nothing rounded)
        wname, gname = ("Wq", "gamma_q") if name == "Q" else ("Wk", "gamma_k")
        o = oracle.rope_rotate(oracle.rms_norm(oracle.qkv_proj(inp["X"][ids], inp[wname]).reshape(len(ids), H, d),
                                               oracle.widen(inp[gname]), eps), ids, grid, pairs, 10000.0).reshape(len(ids), D)
        e = assert_float_parity(got_seq[ids], o, f"{what} fused {name} against the oracle chain")
        print(f"  {what} fused {name}: {len(ids)} tokens, abs {e[0]:.3g} rel {e[1]:.3g}", flush=True)
        # against the twice-rounded stand-alone chain: apart by what that chain's extra rounding of the projection can
        # move a normalised, rotated element (2^-8 sqrt(2) of its rotary pair's norm) plus the two final roundings
        if not have_chain:
            continue
        a_, b_ = widen_bits(got_seq[rows]), widen_bits(chain[rows])
        pair = np.repeat(np.sqrt(b_[:, 0::2] ** 2 + b_[:, 1::2] ** 2), 2, axis=1)
        bound = 2.0 ** -8 * np.sqrt(2.0) * pair + 2.0 ** -8 * np.abs(b_) + 1e-3
        assert np.all(np.abs(a_ - b_) <= bound), f"{what} {name}: too far from the stand-alone chain"


@gpu
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_proj_fused_matches_the_chain_oracle(oracle, name):
    from synth import make_layer_inputs, sample_token_ids
    cfg = CONFIGS[name]
    print(f"proj_fused {name}: plan {cd.qkv_proj_plan(cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P), 3, True)}", flush=True)
    inp = make_layer_inputs(cfg)
    ids = np.arange(cfg.N) if name in ("C1", "C2", "C3") else sample_token_ids(cfg, random_tiles_per_rank=(4 if name == "C4" else 1))
    _fused_case(oracle, cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.grid, cfg.pairs, inp, ids, what=name)


@gpu
@pytest.mark.parametrize("N,H,d,P,grid,pairs,rank", [
    (272, 4, 64, 1, (17, 16), (16, 16), None),          # a head per wavefront; ragged token tile
    (528, 3, 256, 1, (22, 24), (64, 64), None),         # a head across four wavefronts; D = 768: three tiles of 256
    (96, 5, 64, 1, (2, 4, 12), (10, 11, 11), None),     # three axes, pair split off the 2-pair grid; D = 320: ragged feature tile
    (512, 4, 128, 4, (16, 32), (40, 24), 2),            # one rank of four
    (384, 4, 64, 1, (2, 4, 48), (1, 15, 16), None),     # an axis of one pair: the rotation table is read from global memory
    (12288, 4, 64, 1, (12288,), (32,), None),           # a table (3 MB) that does not fit LDS: global memory again
    (608, 4, 128, 1, (19, 32), (63, 1), None),          # the fastest axis one pair wide
    (416, 8, 64, 1, (13, 32), (12, 20), None),          # two feature tiles, ragged third token tile
])
def test_proj_fused_other_shapes(oracle, N, H, d, P, grid, pairs, rank):
    from synth import f32_to_bf16_bits
    D = H * d
    rng = np.random.default_rng(N + d)
    inp = {"X": f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))}
    for w in ("Wq", "Wk", "Wv"):
        inp[w] = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    for g_ in ("gamma_q", "gamma_k"):
        inp[g_] = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    ids = np.arange(N) if rank is None else np.arange(rank * (N // P), (rank + 1) * (N // P))
    _fused_case(oracle, N, D, H, d, P, grid, pairs, inp, ids, rank=rank, what=f"{N}x{D}")


def _random_fused_shapes(count, seed):
    """Seeded small shapes for the fused call: 1 to 3 grid axes of odd sizes (the last a multiple of 16 so that the token
    count is), rotary pairs split unevenly over the axes (now and then an axis of one pair), heads of 64, 128 or 256."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        n_axes = int(rng.integers(1, 4))
        d = int(rng.choice([64, 128, 256]))
        H = int(rng.integers(3, 9)) if d < 256 else int(rng.integers(1, 4))
        grid = tuple(int(rng.integers(1, 8)) for _ in range(n_axes - 1)) + (16 * int(rng.integers(1, 5)),)
        N = int(np.prod(grid))
        if N > 1536 or H * d < 192:
            continue
        cuts = np.sort(rng.choice(np.arange(1, d // 2), size=n_axes - 1, replace=False)) if n_axes > 1 else np.array([], dtype=int)
        pairs = tuple(int(x) for x in np.diff(np.concatenate([[0], cuts, [d // 2]])))
        if rng.random() < 0.25 and n_axes > 1:          # an axis of a single pair
            pairs = (1,) + pairs[1:-1] + (pairs[-1] + pairs[0] - 1,) if n_axes > 2 else (1, d // 2 - 1)
        P = int(rng.choice([p_ for p_ in (1, 2, 3, 4) if H % p_ == 0 and N % (16 * p_) == 0]))
        out.append((N, H, d, P, grid, pairs))
    return out


@gpu
@pytest.mark.parametrize("N,H,d,P,grid,pairs", _random_fused_shapes(10, 20260414))
def test_proj_fused_random_small_shapes(oracle, N, H, d, P, grid, pairs):
    from synth import f32_to_bf16_bits
    assert sum(pairs) == d // 2 and int(np.prod(grid)) == N
    D = H * d
    rng = np.random.default_rng(N * 7 + d)
    inp = {"X": f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))}
    for w in ("Wq", "Wk", "Wv"):
        inp[w] = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    for g_ in ("gamma_q", "gamma_k"):
        inp[g_] = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    _fused_case(oracle, N, D, H, d, P, grid, pairs, inp, np.arange(N), what=f"{N}x{D} grid {grid} pairs {pairs} P {P}")


@gpu
@pytest.mark.parametrize("N,H,d,grid,pairs,tile_tokens", [
    (9120, 24, 128, (48, 190), (32, 32), 224),          # 41 x 12 x 3 tiles of 224 tokens, the last row 160 tokens; table 63 KB in LDS
    (20720, 47, 64, (37, 16, 35), (10, 11, 11), 256),   # 81 x 12 x 3 tiles of 256 tokens, ragged in tokens (240) and features (192)
])
def test_proj_fused_ragged_tiles_of_224_and_256_tokens(oracle, N, H, d, grid, pairs, tile_tokens):
    """The two larger tile shapes of the fused call with a ragged last tile row (C3, C4 and C5 are whole multiples)."""
    from synth import f32_to_bf16_bits
    D = H * d
    assert cd.qkv_proj_plan(cd.Shape.make(N, D, H, d, 1), 3, whole_heads=True)["tile_tokens"] == tile_tokens
    rng = np.random.default_rng(N)
    inp = {"X": f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))}
    for w in ("Wq", "Wk", "Wv"):
        inp[w] = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    for g_ in ("gamma_q", "gamma_k"):
        inp[g_] = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    last = N // tile_tokens * tile_tokens
    ids = np.unique(np.concatenate([np.arange(0, 40), np.arange(last - 24, N), rng.integers(0, N, 200)]))
    _fused_case(oracle, N, D, H, d, 1, grid, pairs, inp, ids, what=f"{N}x{D}")


@gpu
def test_proj_fused_single_destinations_and_subsets(oracle):
    """Either destination alone, and Q alone: the same bits as the call with everything."""
    import torch
    from synth import make_layer_inputs
    cfg = CONFIGS["C2"]
    N, D, H, d, P = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P
    inp = make_layer_inputs(cfg)
    sh = cd.Shape.make(N, D, H, d, P)
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    X, Wq, Wk, Wv = (to_dev(inp[k_]) for k_ in ("X", "Wq", "Wk", "Wv"))
    gq, gk = to_dev(inp["gamma_q"]), to_dev(inp["gamma_k"])
    ref_b = [dev_empty((N * D,)) for _ in range(3)]
    ref_h = [dev_empty((H, N, d)) for _ in range(3)]
    cd.qkv_proj_fused(sh, X, Wq, Wk, Wv, gq, gk, cfg.eps, rope, ref_b[0], ref_b[1], ref_b[2], cd.SEND_MAJOR, ref_h[0], ref_h[1], ref_h[2])
    b_only = [dev_empty((N * D,)) for _ in range(3)]
    h_only = [dev_empty((H, N, d)) for _ in range(3)]
    cd.qkv_proj_fused(sh, X, Wq, Wk, Wv, gq, gk, cfg.eps, rope, b_only[0], b_only[1], b_only[2], cd.SEND_MAJOR, None, None, None)
    cd.qkv_proj_fused(sh, X, None, None, Wv, None, None, cfg.eps, None, None, None, None, cd.SEND_MAJOR, None, None, h_only[2])   # V needs no rope
    cd.qkv_proj_fused(sh, X, Wq, None, None, gq, None, cfg.eps, rope, None, None, None, cd.SEND_MAJOR, h_only[0], None, None)
    cd.qkv_proj_fused(sh, X, None, Wk, None, None, gk, cfg.eps, rope, None, None, None, cd.SEND_MAJOR, None, h_only[1], None)
    _sync()
    for i in range(3):
        assert torch.equal(b_only[i], ref_b[i]) and torch.equal(h_only[i], ref_h[i]), i
    with pytest.raises(cd.CocodiffError):          # a weight without any destination
        cd.qkv_proj_fused(sh, X, Wq, None, None, gq, None, cfg.eps, rope, None, None, None, cd.SEND_MAJOR, None, None, None)
    with pytest.raises(cd.CocodiffError):          # Q without its gamma
        cd.qkv_proj_fused(sh, X, Wq, None, None, None, None, cfg.eps, rope, ref_b[0], None, None, cd.SEND_MAJOR, None, None, None)


@gpu
@pytest.mark.parametrize("name,order", [("C1", 0), ("C2", 1), ("C3", 1), ("C4", 0), ("C5", 1)])
def test_norm_rope_pack_equals_norm_rope_then_pack(oracle, name, order):
    import torch
    cfg = CONFIGS[name]
    print(f"norm_rope_pack {name} order {order}", flush=True)
    rng = np.random.default_rng(cfg.index + 70)
    from synth import f32_to_bf16_bits
    q0 = f32_to_bf16_bits(rng.standard_normal((cfg.N, cfg.D), dtype=np.float32))
    k0 = f32_to_bf16_bits(rng.standard_normal((cfg.N, cfg.D), dtype=np.float32) * np.float32(3.0))
    gq = f32_to_bf16_bits((1 + 0.1 * rng.standard_normal(cfg.d)).astype(np.float32))
    gk = f32_to_bf16_bits((1 + 0.1 * rng.standard_normal(cfg.d)).astype(np.float32))
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    sh = cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P)
    qd, kd, gqd, gkd = to_dev(q0), to_dev(k0), to_dev(gq), to_dev(gk)
    fq, fk, bq, bk = (dev_empty((cfg.N * cfg.D,)) for _ in range(4))
    for t in (fq, fk):
        t.fill_(-1)
    cd.qk_norm_rope_pack(sh, qd, kd, gqd, gkd, cfg.eps, rope, fq, fk, order)
    _sync()
    assert np.array_equal(to_host_bits(qd), q0) and np.array_equal(to_host_bits(kd), k0)     # inputs untouched
    cd.qk_norm_rope(sh, qd, kd, gqd, gkd, cfg.eps, rope)
    cd.a2a_pack(sh, qd, bq, order)
    cd.a2a_pack(sh, kd, bk, order)
    _sync()
    assert np.array_equal(to_host_bits(fq), to_host_bits(bq)) and np.array_equal(to_host_bits(fk), to_host_bits(bk))
    # one tensor alone, one rank alone
    fq.fill_(-1)
    cd.qk_norm_rope_pack(cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, 0, 1), to_dev(q0), None, gqd, None, cfg.eps, rope, fq, None, order)
    _sync()
    part, full = to_host_bits(fq).reshape(cfg.P, cfg.P, -1), to_host_bits(bq).reshape(cfg.P, cfg.P, -1)
    mine = np.zeros((cfg.P, cfg.P), dtype=bool)
    if order == cd.SEND_MAJOR:
        mine[0, :] = True
    else:
        mine[:, 0] = True
    assert np.array_equal(part[mine], full[mine]) and np.all(part[~mine] == 0xFFFF)
    # the oracle: pack(norm_rope) on the first rank's tokens
    ids = np.arange(cfg.Ns)
    want = oracle.qk_norm_rope(q0[ids].reshape(-1, cfg.H, cfg.d), ids, gq, cfg.eps, cfg.grid, cfg.pairs, cfg.theta)
    hs = dev_empty((cfg.H, cfg.N, cfg.d))
    cd.a2a_unpack(sh, bq, hs, order)
    _sync()
    got = to_host_bits(hs).transpose(1, 0, 2)[ids]
    assert_float_parity(got, want, f"norm_rope_pack {name}")


@gpu
@pytest.mark.parametrize("name,order", [("C1", 0), ("C1", 1), ("C2", 1), ("C3", 1), ("C4", 1), ("C5", 0)])
def test_unpack_norm_rope_equals_norm_rope_pack_unpack(oracle, name, order):
    """Normalising on the receiver: raw rows in the exchange buffer, norm + RoPE inside the unpack pass."""
    import torch
    cfg = CONFIGS[name]
    print(f"unpack_norm_rope {name} order {order}", flush=True)
    from synth import f32_to_bf16_bits
    rng = np.random.default_rng(cfg.index + 90)
    N, D, H, d, P = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P
    q0 = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))
    k0 = f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32) * np.float32(0.25))
    gq = f32_to_bf16_bits((1 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    gk = f32_to_bf16_bits((1 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    sh = cd.Shape.make(N, D, H, d, P)
    gqd, gkd = to_dev(gq), to_dev(gk)
    # reference: the stand-alone calls
    qd, kd = to_dev(q0), to_dev(k0)
    bq, bk, hq, hk = dev_empty((N * D,)), dev_empty((N * D,)), dev_empty((H, N, d)), dev_empty((H, N, d))
    cd.qk_norm_rope(sh, qd, kd, gqd, gkd, cfg.eps, rope)
    for src, buf, dst in ((qd, bq, hq), (kd, bk, hk)):
        cd.a2a_pack(sh, src, buf, order)
        cd.a2a_unpack(sh, buf, dst, order)
    # receiver side: raw rows packed, normalised while unpacking
    rq, rk, fq, fk = dev_empty((N * D,)), dev_empty((N * D,)), dev_empty((H, N, d)), dev_empty((H, N, d))
    cd.a2a_pack(sh, to_dev(q0), rq, order)
    cd.a2a_pack(sh, to_dev(k0), rk, order)
    for t in (fq, fk):
        t.fill_(-1)
    cd.a2a_unpack_norm_rope(sh, rq, rk, fq, fk, gqd, gkd, cfg.eps, rope, order)
    _sync()
    assert np.array_equal(to_host_bits(fq), to_host_bits(hq)) and np.array_equal(to_host_bits(fk), to_host_bits(hk))
    # one tensor, one receiving rank: only that rank's heads are written
    fk.fill_(-1)
    p0 = P - 1
    cd.a2a_unpack_norm_rope(cd.Shape.make(N, D, H, d, P, p0, 1), None, rk, None, fk, None, gkd, cfg.eps, rope, order)
    _sync()
    got = to_host_bits(fk)
    assert np.array_equal(got[p0 * cfg.Hp:], to_host_bits(hk)[p0 * cfg.Hp:]) and np.all(got[:p0 * cfg.Hp] == 0xFFFF)
    # the oracle on the first rank's tokens
    ids = np.arange(cfg.Ns)
    want = oracle.qk_norm_rope(q0[ids].reshape(-1, H, d), ids, gq, cfg.eps, cfg.grid, cfg.pairs, cfg.theta)
    assert_float_parity(to_host_bits(fq).transpose(1, 0, 2)[ids], want, f"unpack_norm_rope {name}")


@gpu
@pytest.mark.parametrize("name,order", [("C1", 0), ("C2", 1), ("C3", 1), ("C4", 0), ("C5", 0)])
def test_unpack_select_equals_unpack_then_select(oracle, name, order):
    import torch
    cfg = CONFIGS[name]
    print(f"unpack_select {name} order {order}", flush=True)
    cur, prev, changed = make_v_pair(cfg, layout="hs")            # [H][N][d]
    H, N, d, T, NT = cfg.H, cfg.N, cfg.d, cfg.tile_tokens, cfg.NT
    sh = cd.Shape.make(N, cfg.D, H, d, cfg.P)
    seq = np.ascontiguousarray(cur.transpose(1, 0, 2))             # [N][H][d]: what the senders hold
    buf = dev_empty((N * cfg.D,))
    cd.a2a_pack(sh, to_dev(seq), buf, order)
    prev_d = to_dev(prev)
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")
    outs = []
    for fused in (False, True):
        hs = dev_empty((H, N, d))
        hs.fill_(-1)
        flags, idx, n_act = dev_empty((NT,), "i32"), dev_empty((NT,), "i32"), dev_empty((1,), "i32")
        idx.fill_(-1)
        compact = dev_empty((H, NT * T, d))
        compact.fill_(-1)
        if fused:
            cd.a2a_unpack_select(sh, buf, order, hs, prev_d, T, cfg.tau, flags, idx, n_act, compact, NT, ws)
        else:
            cd.a2a_unpack(sh, buf, hs, order)
            cd.vmajor_select(H, N, d, T, hs, prev_d, cfg.tau, flags, idx, n_act, compact, NT, ws)
        _sync()
        n = int(n_act.cpu()[0])
        outs.append((to_host_bits(hs), flags.cpu().numpy(), idx.cpu().numpy()[:n], n, to_host_bits(compact)[:, :n * T]))
    a, b = outs
    assert np.array_equal(a[0], b[0]) and np.array_equal(b[0], cur)
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2]) and a[3] == b[3]
    assert np.array_equal(a[4], b[4])
    # and against the oracle / the generator's own list
    o_flags, o_idx, o_n, o_comp = oracle.vmajor_select(cur, prev, cfg.tau, T)
    assert b[3] == o_n == len(changed) and np.array_equal(b[2], o_idx[:o_n]) and np.array_equal(b[2], np.sort(changed))
    assert np.array_equal(b[1], o_flags) and np.array_equal(b[4], o_comp[:, :o_n * T])
    # a partial rank range is refused: a tile's flag needs every head
    with pytest.raises(cd.CocodiffError):
        cd.a2a_unpack_select(cd.Shape.make(N, cfg.D, H, d, cfg.P, 0, 1), buf, order, hs, prev_d, T, cfg.tau, None, idx, n_act,
                             None, NT, ws)


def _fused_select_case(oracle, N, D, H, d, P, grid, pairs, inp, T, tau, n_changed, order, cap=None, sparse=False, what=""):
    """cocodiff_qkv_proj_fused_select against cocodiff_qkv_proj_fused followed by cocodiff_vmajor_select: every output
    bit for bit; the selection also against the oracle on the GPU's V."""
    import torch
    from synth import perturb_tiles
    sh = cd.Shape.make(N, D, H, d, P)
    NT = N // T
    cap = NT if cap is None else cap
    table = torch.from_numpy(cd.rope_table(grid, pairs, 10000.0)).to("cuda:0")
    rope = cd.Rope.make(grid, pairs, 10000.0, table.data_ptr())
    X, Wq, Wk, Wv = (to_dev(inp[k_]) for k_ in ("X", "Wq", "Wk", "Wv"))
    gq, gk = to_dev(inp["gamma_q"]), to_dev(inp["gamma_k"])
    eps = 1e-6
    # previous-step V: this step's V with some tiles perturbed
    v0 = dev_empty((H, N, d))
    cd.qkv_proj_hs(sh, X, None, None, Wv, None, None, v0)
    _sync()
    cur = to_host_bits(v0)
    rng = np.random.default_rng(N + 3 * T)
    if sparse:      # one element of one head differs per changed tile: the flag must come from a single lane
        prev = cur.copy()
        changed = np.sort(rng.permutation(NT)[:n_changed]).astype(np.int32)
        for t_ in changed:
            h_, n_, i_ = int(rng.integers(H)), int(t_) * T + int(rng.integers(T)), int(rng.integers(d))
            prev[h_, n_, i_] ^= 0x4000        # flips the exponent's second bit: far apart
    else:
        prev, changed = perturb_tiles(cur, 1, T, n_changed, rng, 0.05)
    prev_d = to_dev(prev)
    outs = []
    for one_call in (False, True):
        bufs = [dev_empty((N * D,)) for _ in range(3)]
        hss = [dev_empty((H, N, d)) for _ in range(3)]
        flags, idx, n_act = dev_empty((NT,), "i32"), dev_empty((NT,), "i32"), dev_empty((1,), "i32")
        compact = dev_empty((H, cap * T, d))
        for t_ in bufs + hss + [flags, idx, compact]:
            t_.fill_(-1)
        if one_call:
            ws = torch.empty(max(cd.qkv_proj_fused_select_workspace_bytes(sh, T), 16), dtype=torch.uint8, device="cuda:0")
            ws.fill_(0xA5)                       # nothing in it needs clearing
            cd.qkv_proj_fused_select(sh, X, Wq, Wk, Wv, gq, gk, eps, rope, bufs[0], bufs[1], bufs[2], order, hss[0], hss[1], hss[2],
                                     prev_d, T, tau, flags, idx, n_act, compact, cap, ws)
        else:
            ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")
            cd.qkv_proj_fused(sh, X, Wq, Wk, Wv, gq, gk, eps, rope, bufs[0], bufs[1], bufs[2], order, hss[0], hss[1], hss[2])
            cd.vmajor_select(H, N, d, T, hss[2], prev_d, tau, flags, idx, n_act, compact, cap, ws)
        _sync()
        n = int(n_act.cpu()[0])
        outs.append(([to_host_bits(t_) for t_ in bufs + hss], flags.cpu().numpy(), idx.cpu().numpy()[:min(n, NT)], n,
                     to_host_bits(compact)[:, :min(n, cap) * T]))
    a, b = outs
    for k_ in range(6):
        assert np.array_equal(a[0][k_], b[0][k_]), f"{what}: tensor {k_} differs between the two forms"
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2]) and a[3] == b[3], f"{what}: flags / list / count differ"
    assert np.array_equal(a[4], b[4]), f"{what}: compact differs"
    assert np.array_equal(b[0][5], cur)
    o_flags, o_idx, o_n, o_comp = oracle.vmajor_select(cur, prev, tau, T)
    assert b[3] == o_n and np.array_equal(b[2], o_idx[:o_n]) and np.array_equal(b[1], o_flags), f"{what}: selection differs from the oracle"
    assert np.array_equal(b[4], o_comp[:, :min(o_n, cap) * T])
    if tau > 0 and tau < 0.01:
        assert o_n == len(changed) and np.array_equal(o_idx[:o_n], np.sort(changed))
    return o_n


@gpu
@pytest.mark.parametrize("name,order", [("C1", 0), ("C2", 1), ("C3", 1), ("C4", 0), ("C5", 1)])
def test_proj_fused_select_equals_the_two_calls(oracle, name, order):
    from synth import make_layer_inputs
    cfg = CONFIGS[name]
    print(f"fused_select {name}", flush=True)
    inp = make_layer_inputs(cfg)
    n = _fused_select_case(oracle, cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.grid, cfg.pairs, inp, cfg.tile_tokens, cfg.tau, cfg.n_changed,
                           order, what=name)
    assert n == cfg.n_changed


@gpu
@pytest.mark.parametrize("N,H,d,P,grid,pairs,T,tau,n_changed,cap,sparse", [
    (272, 4, 64, 1, (17, 16), (16, 16), 16, 1e-3, 5, None, False),       # ragged token tile (272 = 192 + 80)
    (528, 3, 256, 1, (22, 24), (64, 64), 16, 1e-3, 33, 7, False),        # list longer than the compact buffer
    (96, 5, 64, 1, (2, 4, 12), (10, 11, 11), 16, 1e-3, 6, None, False),  # D = 320: ragged feature tile, two flag bytes per tile
    (512, 4, 128, 4, (16, 32), (40, 24), 16, 1e-3, 32, None, True),      # every tile changed, each in one element only
    (512, 4, 128, 4, (16, 32), (40, 24), 16, 1e-3, 0, None, False),      # nothing changed
    (512, 4, 128, 2, (16, 32), (40, 24), 16, 0.0, 9, None, True),        # threshold 0
    (512, 4, 128, 2, (16, 32), (40, 24), 16, float("inf"), 9, None, False),   # nothing exceeds an infinite threshold
    (512, 4, 128, 2, (16, 32), (40, 24), 16, float("nan"), 9, None, False),   # NaN: every tile is active
    (512, 4, 128, 2, (16, 32), (40, 24), 32, 1e-3, 5, None, False),      # another tile height: runs as the two calls
    (256, 72, 64, 1, (16, 16), (16, 16), 16, 1e-3, 4, None, True),       # D = 4608: more than 16 feature tiles, the two calls again
])
def test_proj_fused_select_other_shapes(oracle, N, H, d, P, grid, pairs, T, tau, n_changed, cap, sparse):
    from synth import f32_to_bf16_bits
    D = H * d
    rng = np.random.default_rng(N + d + T)
    inp = {"X": f32_to_bf16_bits(rng.standard_normal((N, D), dtype=np.float32))}
    for w in ("Wq", "Wk", "Wv"):
        inp[w] = f32_to_bf16_bits(rng.standard_normal((D, D), dtype=np.float32) * np.float32(D ** -0.5))
    for g_ in ("gamma_q", "gamma_k"):
        inp[g_] = f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32))
    _fused_select_case(oracle, N, D, H, d, P, grid, pairs, inp, T, tau, n_changed, cd.RECV_MAJOR, cap=cap, sparse=sparse,
                       what=f"{N}x{D} T={T} tau={tau}")


@gpu
def test_proj_fused_select_argument_errors():
    import torch
    cfg = CONFIGS["C1"]
    sh = cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P)
    t = lambda *shape: dev_empty(shape)
    X, W, g = t(cfg.N, cfg.D), t(cfg.D, cfg.D), t(cfg.d)
    buf, hs = t(cfg.N * cfg.D), t(cfg.H, cfg.N, cfg.d)
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    idx, n_act = dev_empty((cfg.NT,), "i32"), dev_empty((1,), "i32")
    ws = torch.empty(cd.qkv_proj_fused_select_workspace_bytes(sh, 16), dtype=torch.uint8, device="cuda:0")
    assert ws.numel() == cfg.NT * 16
    ok = dict(shape=sh, x=X, wq=None, wk=None, wv=W, gamma_q=None, gamma_k=None, eps=1e-6, rope=None, qbuf=None, kbuf=None, vbuf=buf,
              slot_order=cd.SEND_MAJOR, q_hs=None, k_hs=None, v_hs=hs, v_prev=hs, tile_tokens=16, tau=0.1, flags=None, active_idx=idx,
              n_active=n_act, compact=None, cap_tiles=0, workspace=ws)
    cd.qkv_proj_fused_select(**ok)                                   # V alone, index-only: fine
    for bad in (dict(wv=None), dict(v_hs=None), dict(vbuf=None), dict(v_prev=None), dict(active_idx=None), dict(tile_tokens=24),
                dict(shape=cd.Shape.make(cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, 0, 1)), dict(workspace=ws[:16]), dict(compact=hs, cap_tiles=0)):
        with pytest.raises(cd.CocodiffError):
            cd.qkv_proj_fused_select(**{**ok, **bad})
    _sync()


def test_cache_schedule_host_arithmetic(oracle):
    for n_tokens in (9216, 900, 99840, 7):
        for step in range(1, 51):
            assert cd.cache_active_count(step, 50, 5, 10, n_tokens) == oracle.active_count(step, 50, 5, 10, n_tokens)
    assert cd.cache_active_count(0, 50, 5, 10, 100) == -1 and cd.cache_active_count(3, 50, 5, 10, 0) == -1
    assert cd.cache_active_count(30, 50, 5, 0, 90) == 90 - (90 * 25) // 45     # no periodic update


def test_next_rows_argument_errors():
    import ctypes
    from paper_2604_14561_amd import binding as B
    L = B.lib()
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    g = L.cocodiff_vmajor_gather
    assert g(4, 256, 60, 16, fake, fake, fake, fake, 4, None) == B.ERR_SHAPE
    assert g(4, 256, 64, 16, None, fake, fake, fake, 4, None) == B.ERR_NULL
    assert g(4, 256, 64, 16, fake, fake, None, fake, 4, None) == B.ERR_NULL
    assert g(4, 256, 64, 16, odd, fake, fake, fake, 4, None) == B.ERR_ALIGN
    assert g(4, 256, 64, 16, fake, fake, fake, fake, 0, None) == B.ERR_CAPACITY
    assert L.cocodiff_vmajor_scatter(4, 250, 64, 16, fake, fake, fake, fake, 4, None) == B.ERR_SHAPE
    s = cd.Shape.make(256, 256, 4, 64, 3)
    assert L.cocodiff_a2a_pack_hs(ctypes.byref(s), fake, fake, 0, None) == B.ERR_SHAPE
    s = cd.Shape.make(256, 256, 4, 64, 2)
    assert L.cocodiff_a2a_unpack_seq(ctypes.byref(s), fake, None, 0, None) == B.ERR_NULL
    assert L.cocodiff_a2a_pack_hs(ctypes.byref(s), fake, fake, 5, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_token_metric(4, 256, 60, fake, fake, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_token_metric(4, 256, 64, fake, None, fake, None) == B.ERR_NULL
    assert L.cocodiff_vmajor_token_metric(4, 256, 64, odd, fake, fake, None) == B.ERR_ALIGN
    assert L.cocodiff_vmajor_topk(1, 256, fake, 257, 0, fake, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_topk(1, 256, fake, -1, 0, fake, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_topk(0, 256, fake, 5, 0, fake, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_topk(1 << 16, 1 << 16, fake, 5, 1, fake, fake, None) == B.ERR_SHAPE
    assert L.cocodiff_vmajor_topk(1, 256, None, 5, 0, fake, fake, None) == B.ERR_NULL


# ---------------------------------------------------------------------------
# the benchmark's schedules: fused entry points on three and on two streams
# ---------------------------------------------------------------------------

@gpu
@pytest.mark.parametrize("name", ["C2", "C3"])
def test_fused_steps_equal_standalone_calls_and_oracle(oracle, name):
    """The fused V-First steps (three streams; then the two-stream form bench.py times by default) against the same step
    through the five stand-alone calls on one stream (bit-identical: every buffer and the selection), and
    sampled rows of its head-parallel Q against the oracle chain."""
    import torch
    from synth import make_layer_inputs, perturb_tiles, sample_token_ids
    cfg = CONFIGS[name]
    print(f"fused three-stream step {name}", flush=True)
    N, D, H, d, P, T, NT = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.tile_tokens, cfg.NT
    inp = make_layer_inputs(cfg)
    X, Wq, Wk, Wv = (to_dev(inp[k_]) for k_ in ("X", "Wq", "Wk", "Wv"))
    gq, gk = to_dev(inp["gamma_q"]), to_dev(inp["gamma_k"])
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    sh = cd.Shape.make(N, D, H, d, P)
    ORDER = cd.RECV_MAJOR
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")

    def fresh():
        o = {k_: dev_empty((N, D)) for k_ in ("q", "k", "v", "bq", "bk", "bv")}
        o.update({k_: dev_empty((H, N, d)) for k_ in ("hq", "hk", "hv")})
        o.update(flags=dev_empty((NT,), "i32"), idx=dev_empty((NT,), "i32"), n=dev_empty((1,), "i32"), compact=dev_empty((H, NT * T, d)))
        for t in o.values():
            t.fill_(-1)
        return o

    # previous-step V: the stand-alone path's own head-parallel V with a seeded set of tiles perturbed
    a = fresh()
    cd.qkv_proj(sh, X, None, None, Wv, None, None, a["v"])
    cd.a2a_pack(sh, a["v"], a["bv"], ORDER)
    cd.a2a_unpack(sh, a["bv"], a["hv"], ORDER)
    _sync()
    prev_host, changed = perturb_tiles(to_host_bits(a["hv"]), 1, T, cfg.n_changed, np.random.default_rng(cfg.index), cfg.noise_sigma)
    prev = to_dev(prev_host)

    # stand-alone calls, one stream
    cd.qkv_proj(sh, X, Wq, Wk, None, a["q"], a["k"], None)
    cd.qk_norm_rope(sh, a["q"], a["k"], gq, gk, cfg.eps, rope)
    for src, buf, dst in (("q", "bq", "hq"), ("k", "bk", "hk")):
        cd.a2a_pack(sh, a[src], a[buf], ORDER)
        cd.a2a_unpack(sh, a[buf], a[dst], ORDER)
    cd.vmajor_select(H, N, d, T, a["hv"], prev, cfg.tau, a["flags"], a["idx"], a["n"], a["compact"], NT, ws)
    _sync()

    # fused entry points, three streams, V first
    b = fresh()
    s_v, s_qk, s_q = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ws2 = torch.empty_like(ws)
    torch.cuda.synchronize()
    cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, b["bv"], ORDER, stream=s_v)
    v_ready = torch.cuda.Event()
    v_ready.record(s_v)
    cd.a2a_unpack_select(sh, b["bv"], ORDER, b["hv"], prev, T, cfg.tau, b["flags"], b["idx"], b["n"], b["compact"], NT, ws2, stream=s_v)
    s_qk.wait_event(v_ready)
    cd.qkv_proj(sh, X, Wq, None, None, b["q"], None, None, stream=s_qk)
    q_ready = torch.cuda.Event()
    q_ready.record(s_qk)
    cd.qkv_proj(sh, X, None, Wk, None, None, b["k"], None, stream=s_qk)
    s_q.wait_event(q_ready)
    cd.qk_norm_rope_pack(sh, b["q"], None, gq, None, cfg.eps, rope, b["bq"], None, ORDER, stream=s_q)
    cd.a2a_unpack(sh, b["bq"], b["hq"], ORDER, stream=s_q)
    cd.qk_norm_rope_pack(sh, None, b["k"], None, gk, cfg.eps, rope, None, b["bk"], ORDER, stream=s_qk)
    cd.a2a_unpack(sh, b["bk"], b["hk"], ORDER, stream=s_qk)
    torch.cuda.synchronize()

    for key in ("bq", "bk", "bv", "hq", "hk", "hv", "flags"):
        assert np.array_equal(a[key].cpu().numpy(), b[key].cpu().numpy()), key
    n = int(a["n"].cpu()[0])
    assert n == int(b["n"].cpu()[0]) == cfg.n_changed
    assert np.array_equal(a["idx"].cpu().numpy()[:n], b["idx"].cpu().numpy()[:n])
    assert np.array_equal(a["idx"].cpu().numpy()[:n], np.sort(changed))
    assert np.array_equal(to_host_bits(a["compact"])[:, :n * T], to_host_bits(b["compact"])[:, :n * T])

    # the benchmark's default: every projection straight into its exchange buffer, norm + RoPE on the receiving side
    c = fresh()
    ws3 = torch.empty_like(ws)
    torch.cuda.synchronize()
    cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, c["bv"], ORDER, stream=s_v)
    v_ready = torch.cuda.Event()
    v_ready.record(s_v)
    cd.a2a_unpack_select(sh, c["bv"], ORDER, c["hv"], prev, T, cfg.tau, c["flags"], c["idx"], c["n"], c["compact"], NT, ws3, stream=s_v)
    s_qk.wait_event(v_ready)
    cd.qkv_proj_pack(sh, X, Wq, None, None, c["bq"], None, None, ORDER, stream=s_qk)
    q_ready = torch.cuda.Event()
    q_ready.record(s_qk)
    cd.qkv_proj_pack(sh, X, None, Wk, None, None, c["bk"], None, ORDER, stream=s_qk)
    s_q.wait_event(q_ready)
    cd.a2a_unpack_norm_rope(sh, c["bq"], None, c["hq"], None, gq, None, cfg.eps, rope, ORDER, stream=s_q)
    cd.a2a_unpack_norm_rope(sh, None, c["bk"], None, c["hk"], None, gk, cfg.eps, rope, ORDER, stream=s_qk)
    torch.cuda.synchronize()
    for key in ("bv", "hq", "hk", "hv", "flags"):
        assert np.array_equal(a[key].cpu().numpy(), c[key].cpu().numpy()), key
    assert int(c["n"].cpu()[0]) == n and np.array_equal(a["idx"].cpu().numpy()[:n], c["idx"].cpu().numpy()[:n])
    assert np.array_equal(to_host_bits(a["compact"])[:, :n * T], to_host_bits(c["compact"])[:, :n * T])
    # the benchmark's default launch configuration: two streams, Q and K projected and unpacked by one launch each
    e = fresh()
    ws4 = torch.empty_like(ws)
    torch.cuda.synchronize()
    cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, e["bv"], ORDER, stream=s_v)
    v_ready = torch.cuda.Event()
    v_ready.record(s_v)
    cd.a2a_unpack_select(sh, e["bv"], ORDER, e["hv"], prev, T, cfg.tau, e["flags"], e["idx"], e["n"], e["compact"], NT, ws4, stream=s_v)
    s_qk.wait_event(v_ready)
    cd.qkv_proj_pack(sh, X, Wq, Wk, None, e["bq"], e["bk"], None, ORDER, stream=s_qk)
    cd.a2a_unpack_norm_rope(sh, e["bq"], e["bk"], e["hq"], e["hk"], gq, gk, cfg.eps, rope, ORDER, stream=s_qk)
    torch.cuda.synchronize()
    for key in ("bq", "bk", "bv", "hq", "hk", "hv", "flags"):
        assert np.array_equal(c[key].cpu().numpy(), e[key].cpu().numpy()), key
    assert int(e["n"].cpu()[0]) == n and np.array_equal(a["idx"].cpu().numpy()[:n], e["idx"].cpu().numpy()[:n])
    assert np.array_equal(to_host_bits(a["compact"])[:, :n * T], to_host_bits(e["compact"])[:, :n * T])
    # here the exchange buffers of Q and K carry the projection itself: pack(q) of the stand-alone projection
    raw = dev_empty((N, D))
    cd.a2a_pack(sh, b["q"], raw, ORDER)
    _sync()
    assert np.array_equal(to_host_bits(raw), to_host_bits(c["bq"]))

    # sampled rows of the fused path's head-parallel Q against the oracle: norm + RoPE of the GPU's own bf16 projection
    ids = np.arange(N) if name == "C2" else sample_token_ids(cfg, random_tiles_per_rank=2)
    q_proj = to_host_bits(b["q"])[ids].reshape(-1, H, d)           # the fused path leaves the projection itself in q
    assert_float_parity(q_proj.reshape(len(ids), D), oracle.qkv_proj(inp["X"][ids], inp["Wq"]), f"fused step {name}: Q projection")
    want = oracle.qk_norm_rope(q_proj, ids, inp["gamma_q"], cfg.eps, cfg.grid, cfg.pairs, cfg.theta)
    got = to_host_bits(b["hq"]).transpose(1, 0, 2)[ids]
    assert_float_parity(got, want, f"fused step {name}: head-parallel Q")


@gpu
def test_unpack_select_degenerate_cases(oracle):
    """Nothing changed, everything changed, and a compact buffer smaller than the list: same answers as the oracle."""
    import torch
    cfg = CONFIGS["C1"]
    H, N, d, T, NT = cfg.H, cfg.N, cfg.d, cfg.tile_tokens, cfg.NT
    sh = cd.Shape.make(N, cfg.D, H, d, cfg.P)
    cur, prev, changed = make_v_pair(cfg, layout="hs")
    from synth import bf16_bits_to_f32, f32_to_bf16_bits
    everything = f32_to_bf16_bits(bf16_bits_to_f32(cur) + np.float32(1.0))
    buf = dev_empty((N * cfg.D,))
    cd.a2a_pack(sh, to_dev(np.ascontiguousarray(cur.transpose(1, 0, 2))), buf, cd.SEND_MAJOR)
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")
    for prev_bits, cap in ((cur, NT), (everything, NT), (prev, 2), (prev, 1)):
        hs = dev_empty((H, N, d))
        flags, idx, n_act = dev_empty((NT,), "i32"), dev_empty((NT,), "i32"), dev_empty((1,), "i32")
        compact = dev_empty((H, cap * T, d))
        compact.fill_(-1)
        cd.a2a_unpack_select(sh, buf, cd.SEND_MAJOR, hs, to_dev(prev_bits), T, cfg.tau, flags, idx, n_act, compact, cap, ws)
        _sync()
        o_flags, o_idx, o_n, o_comp = oracle.vmajor_select(cur, prev_bits, cfg.tau, T, cap_tiles=cap)
        n = int(n_act.cpu()[0])
        assert n == o_n and np.array_equal(flags.cpu().numpy(), o_flags) and np.array_equal(idx.cpu().numpy()[:n], o_idx[:n])
        kept = min(n, cap)
        assert np.array_equal(to_host_bits(compact)[:, :kept * T], o_comp[:, :kept * T])
        assert np.all(to_host_bits(compact)[:, kept * T:] == 0xFFFF)          # nothing written beyond the capacity
        assert np.array_equal(to_host_bits(hs), cur)


@gpu
def test_fused_step_replays_from_a_hip_graph(oracle):
    """Every call only enqueues on the caller's stream (no allocation, no synchronisation, no memset), so the whole
    step can be captured into a HIP graph.  Replays, with eager work and synchronisations between them, must give
    the eager result every time."""
    import torch
    from synth import make_layer_inputs, perturb_tiles
    cfg = CONFIGS["C2"]
    N, D, H, d, P, T, NT = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.tile_tokens, cfg.NT
    inp = make_layer_inputs(cfg)
    X, Wq, Wk, Wv = (to_dev(inp[k_]) for k_ in ("X", "Wq", "Wk", "Wv"))
    gq, gk = to_dev(inp["gamma_q"]), to_dev(inp["gamma_k"])
    table = torch.from_numpy(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta)).to("cuda:0")
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    sh = cd.Shape.make(N, D, H, d, P)
    ORDER = cd.RECV_MAJOR
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device="cuda:0")
    bq, bk, bv = (dev_empty((N * D,)) for _ in range(3))
    hq, hk, hv = (dev_empty((H, N, d)) for _ in range(3))
    flags, idx, n_act = dev_empty((NT,), "i32"), dev_empty((NT,), "i32"), dev_empty((1,), "i32")
    compact = dev_empty((H, NT * T, d))

    def step(stream):
        cd.qkv_proj_pack(sh, X, Wq, Wk, Wv, bq, bk, bv, ORDER, stream=stream)
        cd.a2a_unpack_select(sh, bv, ORDER, hv, prev, T, cfg.tau, flags, idx, n_act, compact, NT, ws, stream=stream)
        cd.a2a_unpack_norm_rope(sh, bq, bk, hq, hk, gq, gk, cfg.eps, rope, ORDER, stream=stream)

    def snapshot():
        _sync()
        n = int(n_act.cpu()[0])
        return [to_host_bits(t).copy() for t in (bq, bk, bv, hq, hk, hv)] + [flags.cpu().numpy().copy(), idx.cpu().numpy()[:n].copy(),
                                                                              n, to_host_bits(compact)[:, :n * T].copy()]

    def clear():
        for t in (bq, bk, bv, hq, hk, hv, flags, idx, n_act, compact):
            t.fill_(-1)

    # previous-step V from an eager run of the projection
    prev = dev_empty((H, N, d))
    prev.fill_(0)
    clear()
    step(None)                                 # eager, current stream: also sets the kernels' LDS attributes before any capture
    _sync()
    prev_host, changed = perturb_tiles(to_host_bits(hv), 1, T, cfg.n_changed, np.random.default_rng(5), cfg.noise_sigma)
    prev.copy_(to_dev(prev_host))
    clear()
    step(None)
    want = snapshot()
    assert want[8] == cfg.n_changed and np.array_equal(want[7], np.sort(changed))

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        step(None)                             # the binding passes torch's current stream, which is the capturing one
    for rep in range(3):
        clear()
        _sync()
        graph.replay()
        got = snapshot()
        for g_, w_ in zip(got, want):
            assert np.array_equal(g_, w_) if isinstance(w_, np.ndarray) else g_ == w_, rep
        # eager work of the same kind between the replays
        cd.qkv_proj_pack(sh, X, Wv, None, None, bq, None, None, ORDER)
        _sync()


@gpu
def test_vmajor_token_loop_over_denoising_steps(oracle):
    """The V-Major loop as the paper runs it, token-granular, over a 50-step schedule (5 warm-up steps, full update
    every 10th): per step the L1 metric of every token against the receiver's cache, the top (1 - r) fraction per
    rank, gather of the active tokens' values, scatter into the cache.  The cache and the active lists are compared
    with the oracle's loop step by step (the integer decision on the GPU's own fp32 metric)."""
    import torch
    from synth import f32_to_bf16_bits, bf16_bits_to_f32
    cfg = CONFIGS["C1"]
    H, N, d, P = cfg.H, cfg.N, cfg.d, cfg.P
    Ns = N // P
    rng = np.random.default_rng(77)
    v = rng.standard_normal((H, N, d), dtype=np.float32)
    cache_host = np.zeros((H, N, d), dtype=np.uint16)               # the receiver's cached V (oracle's copy)
    cache_dev = to_dev(cache_host.copy())
    metric = torch.empty(N, dtype=torch.float32, device="cuda:0")
    idx = dev_empty((N,), "i32")
    n_act = dev_empty((P,), "i32")
    n_steps, warmup, sync = 50, 5, 10
    for step in list(range(1, 14)) + [20, 29, 30, 49, 50]:
        # this step's V: the previous one plus a drift that is large on a random quarter of the tokens
        drift = 0.02 * rng.standard_normal((H, N, d), dtype=np.float32)
        hot = rng.random(N) < 0.25
        drift[:, hot, :] *= 20.0
        v = v + drift
        cur = f32_to_bf16_bits(v)
        cur_dev = to_dev(cur)
        k = cd.cache_active_count(step, n_steps, warmup, sync, Ns)
        assert k == oracle.active_count(step, n_steps, warmup, sync, Ns)
        cd.vmajor_token_metric(H, N, d, cur_dev, cache_dev, metric)
        idx.fill_(-1)
        # device-only chain: global token ids, every rank's list and count handed on by pointer
        cd.vmajor_topk(P, Ns, metric, k, idx, n_act, global_ids=True)
        for r in range(P):
            comp = dev_empty((H, max(k, 1), d))
            cd.vmajor_gather(H, N, d, 1, cur_dev, idx[r * Ns:], n_act[r:], comp, max(k, 1))
            cd.vmajor_scatter(H, N, d, 1, comp, idx[r * Ns:], n_act[r:], cache_dev, max(k, 1))
        _sync()
        got_metric = metric.cpu().numpy()
        want_metric = oracle.token_l1_metric(cur, cache_host)
        assert np.all(np.abs(got_metric - want_metric) <= 1e-4 * np.maximum(want_metric, 1e-3))
        lists = idx.cpu().numpy().reshape(P, Ns)
        assert np.all(n_act.cpu().numpy() == k)
        for r in range(P):
            want_list = oracle.topk_active(got_metric[r * Ns:(r + 1) * Ns], k)
            tok = (want_list + r * Ns).astype(np.int32)               # global token ids of this rank's list
            assert np.array_equal(lists[r, :k], tok), (step, r)
            cache_host = oracle.vmajor_scatter(oracle.vmajor_gather(cur, tok, 1, max(k, 1)), tok, cache_host, 1)
        assert np.array_equal(to_host_bits(cache_dev), cache_host), step
        if k == Ns:                                                     # warm-up and every 10th step: full update
            assert np.array_equal(cache_host, cur)
