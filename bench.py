#!/usr/bin/env python3
"""Benchmark of the Ulysses attention-input path on one MI355X.

A step is one pass of the whole hot path over one synthetic layer input, all P logical ranks, in the V-First
order of the paper's Section III-C (V is projected first and its layout change and selection run under the
Q and K work).  Default schedule "fused2", two HIP streams, every result of the path produced (exchange buffers,
head-parallel Q, K, V, the selection's list and compact V):
  main stream: qkv_proj_pack(V -> exchange buffer) -> qkv_proj_pack(Q, K) -> a2a_unpack_norm_rope(Q, K)
  side stream: [after V's projection] a2a_unpack_select(V, V_prev); joined at the end of the step
(norm + RoPE on the receiving side of the exchange).  "fused3" projects Q and K by two launches and uses a third
stream; "fused2x" swaps the roles of the two streams; "fused3s" keeps norm + RoPE on the sending side: qkv_proj -> qk_norm_rope_pack -> a2a_unpack.
"vfirst" / "vfirst3" are the same orders through the stand-alone calls only (projection, norm+RoPE in place, pack,
unpack, select as separate launches); the default run times "vfirst" too and reports it as `standalone_calls_path`.
"serial" runs the stand-alone calls on one stream.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "tokens/s per layer (QKV+norm+RoPE+pack); pack/select GB/s vs HBM peak"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "qkv_gemm_hbm_traffic.txt")


def measured_traffic(workload: str, schedule: str):
    """Bytes per launch that crossed the L2 <-> memory-fabric boundary for the projection kernel, from the
    committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE runs of this script); None if not recorded."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and parts[0] == "traffic_bytes_per_launch" and parts[1] == workload and parts[2] == schedule:
                    return int(parts[3])
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--schedule", default="fused2", choices=["vfirst", "vfirst3", "serial", "fused2", "fused2x", "fused3", "fused3s"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs all P logical ranks of the path on ONE GPU; "
            "there is no multi-GPU path to time (--gpus must be 1).")
        return 2

    import numpy as np
    import torch

    import paper_2604_14561_amd as cd
    from synth import CONFIGS, make_layer_inputs, perturb_tiles

    if not os.path.exists(cd.binding.LIB_PATH):
        from paper_2604_14561_amd import build as _build
        _build.build()

    cfg = CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    N, D, H, d, P, T = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.tile_tokens
    log(f"bench: {cfg.name} N={N} D={D} H={H}x{d} P={P}; generating inputs")

    def up(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

    def bits(t):
        return t.cpu().numpy().view(np.uint16)

    inp = make_layer_inputs(cfg)
    X, Wq, Wk, Wv = up(inp["X"]), up(inp["Wq"]), up(inp["Wk"]), up(inp["Wv"])
    gq, gk = up(inp["gamma_q"]), up(inp["gamma_k"])
    table = up(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta))
    rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, table.data_ptr())
    sh = cd.Shape.make(N, D, H, d, P)

    def bf(shape):
        return torch.empty(shape, dtype=torch.int16, device=dev)

    q, k, v = bf((N, D)), bf((N, D)), bf((N, D))
    bq, bk, bv = bf((N * D,)), bf((N * D,)), bf((N * D,))
    hq, hk, hv = bf((H, N, d)), bf((H, N, d)), bf((H, N, d))
    NT = cfg.NT
    cap = NT
    ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), 16), dtype=torch.uint8, device=dev)
    flags = torch.empty(NT, dtype=torch.int32, device=dev)
    idx = torch.empty(NT, dtype=torch.int32, device=dev)
    n_act = torch.zeros(1, dtype=torch.int32, device=dev)
    compact = bf((H, cap * T, d))

    s_v, s_qk = torch.cuda.Stream(), torch.cuda.Stream()
    ORDER = cd.RECV_MAJOR

    # previous-step V: this layer's own head-parallel V with a seeded fraction of 16-token tiles perturbed
    cd.qkv_proj(sh, X, None, None, Wv, None, None, v)
    cd.a2a_pack(sh, v, bv, ORDER)
    cd.a2a_unpack(sh, bv, hv, ORDER)
    torch.cuda.synchronize()
    v_prev_host, changed = perturb_tiles(bits(hv), 1, T, cfg.n_changed, np.random.default_rng(cfg.index), cfg.noise_sigma)
    hv_prev = up(v_prev_host)
    del v_prev_host

    def step_vfirst(ev=None):
        """The stand-alone calls in the default schedule's shape: both projections on the main stream, V's pack,
        unpack and selection on the side stream under the Q and K work.
        ev: optional (v0, v1, qk0, qk1) timing events bracketing the two projection launches."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj(sh, X, None, None, Wv, None, None, v, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        if ev:
            ev[2].record(s_v)
        cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None, stream=s_v)
        if ev:
            ev[3].record(s_v)
        s_qk.wait_event(v_ready)            # V's layout change and selection overlap what follows its projection
        cd.a2a_pack(sh, v, bv, ORDER, stream=s_qk)
        cd.a2a_unpack(sh, bv, hv, ORDER, stream=s_qk)
        cd.vmajor_select(H, N, d, T, hv, hv_prev, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_qk)
        cd.qk_norm_rope(sh, q, k, gq, gk, cfg.eps, rope, stream=s_v)
        cd.a2a_pack(sh, q, bq, ORDER, stream=s_v)
        cd.a2a_pack(sh, k, bk, ORDER, stream=s_v)
        cd.a2a_unpack(sh, bq, hq, ORDER, stream=s_v)
        cd.a2a_unpack(sh, bk, hk, ORDER, stream=s_v)
        done = torch.cuda.Event()
        done.record(s_qk)
        s_v.wait_event(done)                # join: the next layer cannot start before everything is laid out

    s_q = torch.cuda.Stream()

    def step_vfirst3(ev=None):
        """V, then Q, then K projected one after the other (the order of the paper's Section III-C); each tensor's
        norm/RoPE and layout change run on a side stream under the next tensor's projection."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj(sh, X, None, None, Wv, None, None, v, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        cd.a2a_pack(sh, v, bv, ORDER, stream=s_v)
        cd.a2a_unpack(sh, bv, hv, ORDER, stream=s_v)
        cd.vmajor_select(H, N, d, T, hv, hv_prev, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_v)
        s_qk.wait_event(v_ready)
        if ev:
            ev[2].record(s_qk)
        cd.qkv_proj(sh, X, Wq, None, None, q, None, None, stream=s_qk)
        q_ready = torch.cuda.Event()
        q_ready.record(s_qk)
        cd.qkv_proj(sh, X, None, Wk, None, None, k, None, stream=s_qk)
        if ev:
            ev[3].record(s_qk)
        s_q.wait_event(q_ready)
        cd.qk_norm_rope(sh, q, None, gq, None, cfg.eps, rope, stream=s_q)
        cd.a2a_pack(sh, q, bq, ORDER, stream=s_q)
        cd.a2a_unpack(sh, bq, hq, ORDER, stream=s_q)
        cd.qk_norm_rope(sh, None, k, None, gk, cfg.eps, rope, stream=s_qk)
        cd.a2a_pack(sh, k, bk, ORDER, stream=s_qk)
        cd.a2a_unpack(sh, bk, hk, ORDER, stream=s_qk)
        done_q, done_k = torch.cuda.Event(), torch.cuda.Event()
        done_q.record(s_q)
        done_k.record(s_qk)
        s_v.wait_event(done_q)
        s_v.wait_event(done_k)

    def step_serial(ev=None):
        st = s_v
        if ev:
            ev[0].record(st)
        cd.qkv_proj(sh, X, None, None, Wv, None, None, v, stream=st)
        if ev:
            ev[1].record(st)
            ev[2].record(st)
        cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None, stream=st)
        if ev:
            ev[3].record(st)
        cd.qk_norm_rope(sh, q, k, gq, gk, cfg.eps, rope, stream=st)
        for src, buf, dst in ((v, bv, hv), (q, bq, hq), (k, bk, hk)):
            cd.a2a_pack(sh, src, buf, ORDER, stream=st)
            cd.a2a_unpack(sh, buf, dst, ORDER, stream=st)
        cd.vmajor_select(H, N, d, T, hv, hv_prev, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=st)

    def step_fused2x(ev=None):
        """fused2 with the streams the other way round (V's projection and its unpack + selection on one stream, the Q
        and K projection and their unpack on the other, behind an event): the Q and K projection then starts a
        cross-stream wait later, 2 % more step time at C3."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        cd.a2a_unpack_select(sh, bv, ORDER, hv, hv_prev, T, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_v)
        s_qk.wait_event(v_ready)            # V's projection goes first; its layout change overlaps what follows
        if ev:
            ev[2].record(s_qk)
        cd.qkv_proj_pack(sh, X, Wq, Wk, None, bq, bk, None, ORDER, stream=s_qk)
        if ev:
            ev[3].record(s_qk)
        cd.a2a_unpack_norm_rope(sh, bq, bk, hq, hk, gq, gk, cfg.eps, rope, ORDER, stream=s_qk)
        done = torch.cuda.Event()
        done.record(s_qk)
        s_v.wait_event(done)                # join: the next layer cannot start before Q and K are laid out

    def step_fused2(ev=None):
        """V-First with the fused calls on two streams: V's projection writes its exchange buffer; the projection of Q
        and K (one launch, straight into their exchange buffers) follows it on the same stream, so no cross-stream wait
        sits between the two projections; V's unpack, which carries the selection's flag pass, waits for V's projection
        on the side stream and runs under the Q and K projection; Q and K are normalised and rotated inside one unpack
        pass (receiving side).  4 launches and 7.2 tensor passes over HBM beside the projections, against 13 and 14.2
        with the stand-alone calls."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        if ev:
            ev[2].record(s_v)
        cd.qkv_proj_pack(sh, X, Wq, Wk, None, bq, bk, None, ORDER, stream=s_v)
        if ev:
            ev[3].record(s_v)
        s_qk.wait_event(v_ready)
        cd.a2a_unpack_select(sh, bv, ORDER, hv, hv_prev, T, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_qk)
        cd.a2a_unpack_norm_rope(sh, bq, bk, hq, hk, gq, gk, cfg.eps, rope, ORDER, stream=s_v)
        done = torch.cuda.Event()
        done.record(s_qk)
        s_v.wait_event(done)                # join

    def step_fused3(ev=None):
        """V-First order with the fused calls: every projection writes its exchange buffer itself (no [N][D] tensor
        exists), V's unpack carries the selection's flag pass, Q's and K's unpack carries norm + RoPE (done on the
        receiving side).  6 launches and 7.2 tensor passes over HBM beside the projections, against 13 and 14.2."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        cd.a2a_unpack_select(sh, bv, ORDER, hv, hv_prev, T, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_v)
        s_qk.wait_event(v_ready)
        if ev:
            ev[2].record(s_qk)
        cd.qkv_proj_pack(sh, X, Wq, None, None, bq, None, None, ORDER, stream=s_qk)
        q_ready = torch.cuda.Event()
        q_ready.record(s_qk)
        cd.qkv_proj_pack(sh, X, None, Wk, None, None, bk, None, ORDER, stream=s_qk)
        if ev:
            ev[3].record(s_qk)
        s_q.wait_event(q_ready)
        cd.a2a_unpack_norm_rope(sh, bq, None, hq, None, gq, None, cfg.eps, rope, ORDER, stream=s_q)
        cd.a2a_unpack_norm_rope(sh, None, bk, None, hk, None, gk, cfg.eps, rope, ORDER, stream=s_qk)
        done_q, done_k = torch.cuda.Event(), torch.cuda.Event()
        done_q.record(s_q)
        done_k.record(s_qk)
        s_v.wait_event(done_q)
        s_v.wait_event(done_k)

    def step_fused3s(ev=None):
        """Sender-side variant of fused3: V's projection writes the exchange buffer itself, Q and K are
        normalised and rotated on their way into theirs, V's unpack computes the selection's flags (5 fewer launches
        and 4 fewer passes over HBM per step)."""
        if ev:
            ev[0].record(s_v)
        cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER, stream=s_v)
        if ev:
            ev[1].record(s_v)
        v_ready = torch.cuda.Event()
        v_ready.record(s_v)
        cd.a2a_unpack_select(sh, bv, ORDER, hv, hv_prev, T, cfg.tau, flags, idx, n_act, compact, cap, ws, stream=s_v)
        s_qk.wait_event(v_ready)
        if ev:
            ev[2].record(s_qk)
        cd.qkv_proj(sh, X, Wq, None, None, q, None, None, stream=s_qk)
        q_ready = torch.cuda.Event()
        q_ready.record(s_qk)
        cd.qkv_proj(sh, X, None, Wk, None, None, k, None, stream=s_qk)
        if ev:
            ev[3].record(s_qk)
        s_q.wait_event(q_ready)
        cd.qk_norm_rope_pack(sh, q, None, gq, None, cfg.eps, rope, bq, None, ORDER, stream=s_q)
        cd.a2a_unpack(sh, bq, hq, ORDER, stream=s_q)
        cd.qk_norm_rope_pack(sh, None, k, None, gk, cfg.eps, rope, None, bk, ORDER, stream=s_qk)
        cd.a2a_unpack(sh, bk, hk, ORDER, stream=s_qk)
        done_q, done_k = torch.cuda.Event(), torch.cuda.Event()
        done_q.record(s_q)
        done_k.record(s_qk)
        s_v.wait_event(done_q)
        s_v.wait_event(done_k)

    schedules = {"vfirst": step_vfirst, "vfirst3": step_vfirst3, "serial": step_serial, "fused2": step_fused2, "fused2x": step_fused2x, "fused3": step_fused3,
                 "fused3s": step_fused3s}
    step = schedules[args.schedule]

    def time_schedule(step_fn):
        for _ in range(args.warmup):
            step_fn()
        torch.cuda.synchronize()
        assert int(n_act.cpu()[0]) == cfg.n_changed, "selection did not find the perturbed tiles"
        # HIP events around the projection launches, in every fourth step of the timed region: with events in every
        # step the step itself is 2 % slower (six extra marker packets between its five kernels)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] if i % 4 == 0 else None for i in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_fn(evs[i])
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        log(f"  host enqueue time per step {(t_enq - t0) * 1e3 / args.steps:.3f} ms of {(t1 - t0) * 1e3 / args.steps:.3f} ms")
        return (t1 - t0) * 1e3 / args.steps, [e for e in evs if e is not None]

    ms_per_step, events = time_schedule(step)
    tokens_per_s = N / (ms_per_step * 1e-3)
    # the same step replayed from a HIP graph (capture of the three streams): what is left when the host's launch
    # work is taken out -- a check that the step is GPU-bound, and what a launch-bound small workload gains
    graph_replay = None
    if args.schedule in ("fused2", "fused3") and not args.no_breakdown:
        try:
            graph = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=s_v):
                step()
            for _ in range(args.warmup):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            ms_g = (time.perf_counter() - t0) * 1e3 / args.steps
            assert int(n_act.cpu()[0]) == cfg.n_changed
            graph_replay = {"schedule": args.schedule, "ms_per_step": round(ms_g, 4), "value": round(N / (ms_g * 1e-3), 1), "unit": "tokens/s"}
            log(f"  HIP graph replay of the step: {graph_replay}")
            del graph
        except Exception as e:      # reported, never fatal: the headline is the eager step
            log(f"  HIP graph replay not measured: {e}")
    # the same step through the stand-alone calls only (no fused entry point), reported beside the headline
    standalone = None
    if args.schedule in ("fused2", "fused3") and not args.no_breakdown:
        sa_name = "vfirst" if args.schedule == "fused2" else "vfirst3"
        ms_sa, _ = time_schedule(schedules[sa_name])
        standalone = {"schedule": sa_name, "ms_per_step": round(ms_sa, 4), "value": round(N / (ms_sa * 1e-3), 1), "unit": "tokens/s"}
        log(f"  stand-alone calls ({sa_name} schedule): {standalone}")

    # The sender's share alone -- projection of Q, K, V + norm and RoPE of Q and K + the three packs, up to the
    # filled exchange buffers (the layer's work before the all-to-all) -- in three forms; `value` above is the longer
    # path that also holds the receiver's unpack and the selection.
    layer_only = None
    if not args.no_breakdown:
        def sender_serial():
            cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v, stream=s_v)
            cd.qk_norm_rope(sh, q, k, gq, gk, cfg.eps, rope, stream=s_v)
            for src, buf in ((v, bv), (q, bq), (k, bk)):
                cd.a2a_pack(sh, src, buf, ORDER, stream=s_v)

        def sender_vfirst():
            cd.qkv_proj(sh, X, None, None, Wv, None, None, v, stream=s_v)
            v_ready = torch.cuda.Event()
            v_ready.record(s_v)
            cd.a2a_pack(sh, v, bv, ORDER, stream=s_v)
            s_qk.wait_event(v_ready)
            cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None, stream=s_qk)
            cd.qk_norm_rope(sh, q, k, gq, gk, cfg.eps, rope, stream=s_qk)
            cd.a2a_pack(sh, q, bq, ORDER, stream=s_qk)
            cd.a2a_pack(sh, k, bk, ORDER, stream=s_qk)
            done = torch.cuda.Event()
            done.record(s_qk)
            s_v.wait_event(done)

        def sender_fused():
            cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER, stream=s_v)
            v_ready = torch.cuda.Event()
            v_ready.record(s_v)
            s_qk.wait_event(v_ready)
            cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None, stream=s_qk)
            cd.qk_norm_rope_pack(sh, q, k, gq, gk, cfg.eps, rope, bq, bk, ORDER, stream=s_qk)
            done = torch.cuda.Event()
            done.record(s_qk)
            s_v.wait_event(done)

        layer_only = {}
        for label, fn in (("serial_one_stream", sender_serial), ("vfirst_two_streams", sender_vfirst),
                          ("vfirst_fused_calls", sender_fused)):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            ms_l = (time.perf_counter() - t0) * 1e3 / args.steps
            layer_only[label] = {"ms": round(ms_l, 4), "tokens/s": round(N / (ms_l * 1e-3), 1)}
        log(f"  sender's share alone (projection + norm + RoPE + pack): {layer_only}")

    # dominant kernel: the projection GEMM (launched per step as V, then Q+K -- or V, Q, K in the vfirst3 order)
    n_launch = 3 if args.schedule in ("vfirst3", "fused3", "fused3s") else 2
    gemm_ms = [(e[0].elapsed_time(e[1]), e[2].elapsed_time(e[3])) for e in events]
    gemm_ms_per_launch = float(np.mean([a + b for a, b in gemm_ms])) / n_launch
    flops_per_launch = 2.0 * N * (3 * D) * D / n_launch
    achieved_tflops = flops_per_launch / (gemm_ms_per_launch * 1e-3) / 1e12
    roofline = {"kernel": "qkv_gemm_direct_kernel", "bound": "mfma", "achieved": round(achieved_tflops, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                "traffic": measured_traffic(cfg.name, args.schedule), "avg_launch_us": round(gemm_ms_per_launch * 1e3, 2), "launches_per_step": n_launch}

    # ---- per-kernel times, each launched alone on one stream (not part of `value`) ----
    # HBM-bound kernels are timed "cold": successive launches rotate over buffer sets whose footprint is more than
    # twice the 256 MB last-level cache, so no launch finds its input there; "warm" repeats one set.  A block is one
    # pass over the rotation (at least 8 launches) between two HIP events; median and minimum over 7 blocks.
    kernels = {}
    attainable = None
    if not args.no_breakdown:
        st = torch.cuda.current_stream()
        tensor_bytes = N * D * 2

        def timed(fns, blocks=7):
            per_block = len(fns) * max(1, -(-8 // len(fns)))
            for i in range(min(per_block, 2 * len(fns))):
                fns[i % len(fns)]()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(blocks + 1)]
            torch.cuda.synchronize()
            evs[0].record(st)
            for blk in range(blocks):
                for i in range(per_block):
                    fns[i % len(fns)]()
                evs[blk + 1].record(st)
            torch.cuda.synchronize()
            t = sorted(evs[i].elapsed_time(evs[i + 1]) / per_block * 1e3 for i in range(blocks))
            return t[len(t) // 2], t[0]                       # us per launch: median, min

        def add(name, fns, flops=None, nbytes=None):
            med, mn = timed(fns)
            ent = {"us": round(med, 2), "us_min": round(mn, 2)}
            if len(fns) > 1:
                ent["us_warm"] = round(timed(fns[:1])[0], 2)
            if flops:
                ent["TFLOP/s"] = round(flops / med / 1e6, 1)
                ent["frac_mfma_peak"] = round(flops / med / 1e6 / PEAK_BF16_TFLOPS, 4)
                if attainable:
                    ent["frac_mfma_loop"] = round(flops / med / 1e6 / attainable["mfma_loop_TFLOP/s"], 4)
            if nbytes:
                ent["GB/s"] = round(nbytes / med / 1e3, 1)
                ent["frac_hbm_peak"] = round(nbytes / med / 1e3 / PEAK_HBM_GBS, 4)
                if attainable:
                    ent["frac_copy_rate"] = round(nbytes / med / 1e3 / attainable["hbm_copy_GB/s"], 4)
            kernels[name] = ent

        def chip_state_during(fn, secs=1.2):
            """Median shader clock (MHz, rocm-smi) and socket power (W, hwmon) while `fn` keeps the GPU busy; a value
            that cannot be read is None."""
            import glob
            import re
            import subprocess
            import threading
            clocks, watts, stop = [], [], threading.Event()
            hw = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")

            def sample():
                while not stop.is_set():
                    try:
                        if hw:
                            with open(hw[0]) as f_:
                                watts.append((time.time(), int(f_.read()) / 1e6))
                        out = subprocess.run(["rocm-smi", "--showclocks", "--csv"], capture_output=True, text=True, timeout=10).stdout
                        row = [l for l in out.strip().splitlines() if l.startswith("card0")]
                        m = re.findall(r"\((\d+)Mhz\)", row[0]) if row else []
                        if len(m) >= 2:
                            clocks.append((time.time(), int(m[1])))     # columns: mclk, sclk
                    except Exception:
                        return
            th = threading.Thread(target=sample, daemon=True)
            t_begin = time.time()
            th.start()
            while time.time() < t_begin + secs:
                for _ in range(20):
                    fn()
                torch.cuda.synchronize()
            stop.set()
            th.join(timeout=15)
            late = lambda xs: [v for (ts, v) in xs if ts > t_begin + 0.3]    # the first samples still see the ramp
            return {"sclk_MHz": int(np.median(late(clocks))) if late(clocks) else None,
                    "power_W": int(np.median(late(watts))) if late(watts) else None}

        # what the chip attains on the two calibration kernels: a 1000 MiB copy and a register-only MFMA loop
        big = 1000 << 20   # not a power of two: source and destination must not alias onto the same HBM banks
        src_big = torch.empty(big + (3 << 20), dtype=torch.uint8, device=dev)
        dst_big = torch.empty(big, dtype=torch.uint8, device=dev)
        copy_us = timed([lambda: cd.util_copy(src_big, dst_big, big)])[0]
        memcpy_us = timed([lambda: dst_big.copy_(src_big[:big])])[0]      # the runtime's own device-to-device copy
        del src_big, dst_big
        src_big2 = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst_big2 = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        mfma_flops = cd.util_mfma_rate(1024, 2048, sink)
        mfma_us = timed([lambda: cd.util_mfma_rate(1024, 2048, sink)])[0]
        attainable = {"hbm_copy_GB/s": round(2 * big / copy_us / 1e3, 1), "runtime_memcpy_GB/s": round(2 * big / memcpy_us / 1e3, 1),
                      "mfma_loop_TFLOP/s": round(mfma_flops / mfma_us / 1e6, 1)}
        log(f"  attainable on this GPU: {attainable}")

        g1 = 2.0 * N * D * D
        add("qkv_proj_v", [lambda: cd.qkv_proj(sh, X, None, None, Wv, None, None, v)], flops=g1)
        add("qkv_proj_qk", [lambda: cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None)], flops=2 * g1)
        add("qkv_proj_qkv", [lambda: cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v)], flops=3 * g1)
        add("qkv_proj_pack_v", [lambda: cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, ORDER)], flops=g1)

        # rotation sets: a (token-major), b (exchange buffer), h and p (head-parallel current / previous V; never written)
        R = int(min(64, max(1, -(-(640 << 20) // (2 * tensor_bytes)))))
        sets = []
        for i in range(R):
            sets.append({"a": v.clone(), "b": bv.clone(), "h": hv if i == 0 else hv.clone(),
                         "p": hv_prev if i == 0 else hv_prev.clone()})
        log(f"  cold timings rotate over {R} buffer sets of 4 x {tensor_bytes / 1e6:.1f} MB")
        f_act = cfg.n_changed / NT
        act = bf((H, cap * T, d))
        metric = torch.empty(N, dtype=torch.float32, device=dev)
        tok_idx = torch.empty(N, dtype=torch.int32, device=dev)
        tok_n = torch.zeros(P, dtype=torch.int32, device=dev)
        k_act = cd.cache_active_count(27, 50, 5, 10, N // P)  # mid-schedule step of the paper's 50-step setup

        def each(fn):
            return [(lambda s_=s_: fn(s_)) for s_ in sets]

        add("vmajor_select", each(lambda s_: cd.vmajor_select(H, N, d, T, s_["h"], s_["p"], cfg.tau, flags, idx, n_act, compact, cap, ws)),
            nbytes=(2 + f_act) * tensor_bytes)
        add("a2a_unpack_select", each(lambda s_: cd.a2a_unpack_select(sh, s_["b"], ORDER, s_["a"], s_["p"], T, cfg.tau, flags, idx, n_act, compact, cap, ws)),
            nbytes=(3 + f_act) * tensor_bytes)
        assert int(n_act.cpu()[0]) == cfg.n_changed, "the breakdown's selection inputs were disturbed"
        add("vmajor_token_metric", each(lambda s_: cd.vmajor_token_metric(H, N, d, s_["h"], s_["p"], metric)), nbytes=2 * tensor_bytes)
        add("vmajor_topk", [lambda: cd.vmajor_topk(P, N // P, metric, k_act, tok_idx, tok_n)])   # every rank ranks its own tokens
        # rows after the hot path: sender-side gather / receiver-side scatter of the active tiles, second all-to-all
        add("vmajor_gather", each(lambda s_: cd.vmajor_gather(H, N, d, T, s_["h"], idx, n_act, act, cap)), nbytes=2 * f_act * tensor_bytes)
        add("vmajor_scatter", each(lambda s_: cd.vmajor_scatter(H, N, d, T, act, idx, n_act, s_["a"], cap)), nbytes=2 * f_act * tensor_bytes)
        add("a2a_pack_hs", each(lambda s_: cd.a2a_pack_hs(sh, s_["h"], s_["b"], ORDER)), nbytes=2 * tensor_bytes)
        add("a2a_unpack_seq", each(lambda s_: cd.a2a_unpack_seq(sh, s_["b"], s_["a"], ORDER)), nbytes=2 * tensor_bytes)
        add("a2a_pack", each(lambda s_: cd.a2a_pack(sh, s_["a"], s_["b"], ORDER)), nbytes=2 * tensor_bytes)
        add("a2a_unpack", each(lambda s_: cd.a2a_unpack(sh, s_["b"], s_["a"], ORDER)), nbytes=2 * tensor_bytes)
        add("qk_norm_rope", each(lambda s_: cd.qk_norm_rope(sh, s_["a"], s_["b"], gq, gk, cfg.eps, rope)), nbytes=4 * tensor_bytes)
        add("a2a_unpack_norm_rope", each(lambda s_: cd.a2a_unpack_norm_rope(sh, s_["h"], s_["p"], s_["a"], s_["b"], gq, gk, cfg.eps, rope, ORDER)),
            nbytes=4 * tensor_bytes)
        add("qk_norm_rope_pack", each(lambda s_: cd.qk_norm_rope_pack(sh, s_["h"], s_["p"], gq, gk, cfg.eps, rope, s_["a"], s_["b"], ORDER)),
            nbytes=4 * tensor_bytes)
        add("copy_same_bytes", each(lambda s_: cd.util_copy(s_["a"], s_["b"], tensor_bytes)), nbytes=2 * tensor_bytes)
        kernels["copy_1000MiB"] = {"us": round(copy_us, 2), "GB/s": attainable["hbm_copy_GB/s"],
                                   "frac_hbm_peak": round(attainable["hbm_copy_GB/s"] / PEAK_HBM_GBS, 4)}
        kernels["mfma_register_loop"] = {"us": round(mfma_us, 2), "TFLOP/s": attainable["mfma_loop_TFLOP/s"],
                                         "frac_mfma_peak": round(attainable["mfma_loop_TFLOP/s"] / PEAK_BF16_TFLOPS, 4)}
        del sets, act
        # the chip does not hold its top clock under matrix-core load: record what it runs at (last: the throttled
        # state lingers and would colour the timings above)
        state = {"copy": chip_state_during(lambda: cd.util_copy(src_big2, dst_big2, 256 << 20)),
                 "mfma_loop": chip_state_during(lambda: cd.util_mfma_rate(1024, 512, sink)),
                 "projection": chip_state_during(lambda: cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v))}
        attainable["sclk_MHz"] = {k_: v_["sclk_MHz"] for k_, v_ in state.items()}
        attainable["power_W"] = {k_: v_["power_W"] for k_, v_ in state.items()}
        del src_big2, dst_big2
        log(f"  chip state under load: clocks {attainable['sclk_MHz']} MHz, socket power {attainable['power_W']} W")
        roofline["frac_of_mfma_loop"] = round(achieved_tflops / attainable["mfma_loop_TFLOP/s"], 4)
        if attainable["sclk_MHz"]["projection"]:
            # the published peak is 2.4 GHz x 256 units x 4 SIMDs x 1024 flop/clk; the same at the clock the chip holds
            roofline["sclk_MHz"] = attainable["sclk_MHz"]["projection"]
            roofline["frac_at_sclk"] = round(achieved_tflops / (PEAK_BF16_TFLOPS * attainable["sclk_MHz"]["projection"] / 2400.0), 4)
        for name, ent in kernels.items():
            log(f"  {name:20s} {ent}")

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_c()
        S_tok = min(N, 24576)                                # float stages: the first S_tok tokens per pass
        ids = np.arange(S_tok)
        host_seq = bits(v).reshape(N, H, d)
        host_prev = bits(hv_prev)
        t_float = t_perm = t_pack = t_unpack = t_sel = 0.0
        passes = 0
        while t_float + t_perm < 12.0 and passes < 200:      # about 10-30 s of CPU work in whole passes
            t_a = time.perf_counter()
            o = {}
            for name, w in (("q", "Wq"), ("k", "Wk"), ("v", "Wv")):
                o[name] = oracle.qkv_proj(inp["X"][:S_tok], inp[w])
            for name, g in (("q", "gamma_q"), ("k", "gamma_k")):
                o[name] = oracle.rope_rotate(oracle.rms_norm(o[name].reshape(S_tok, H, d), oracle.widen(inp[g]), cfg.eps),
                                             ids, cfg.grid, cfg.pairs, cfg.theta)
            t_b = time.perf_counter()
            for _ in range(3):                               # Q, K and V each go through pack + unpack
                t0_ = time.perf_counter()
                buf = oracle.a2a_pack(host_seq, P, oracle.ref.RECV_MAJOR)
                t1_ = time.perf_counter()
                hs_host = oracle.a2a_unpack(buf, N, H, d, P, oracle.ref.RECV_MAJOR)
                t2_ = time.perf_counter()
                t_pack += t1_ - t0_
                t_unpack += t2_ - t1_
            t0_ = time.perf_counter()
            o_sel = oracle.vmajor_select(hs_host, host_prev, cfg.tau, T)
            t_sel += time.perf_counter() - t0_
            t_c = time.perf_counter()
            assert o_sel[2] == cfg.n_changed
            t_float += t_b - t_a
            t_perm += t_c - t_b
            passes += 1
        per_token = t_float / (passes * S_tok) + t_perm / (passes * N)
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p_.get("num_threads", 1) for p_ in threadpool_info()] or [1])
        except Exception:
            blas_threads = os.cpu_count() or 1
        cpu = {"value": round(1.0 / per_token, 1), "unit": "tokens/s", "cores": int(blas_threads), "kind": "oracle",
               "sample": f"{passes} passes of the oracle over the workload (fp64 projection + norm + RoPE on "
                         f"{S_tok} of {N} tokens per pass; pack/unpack x3 and select on the full tensors): "
                         f"{t_float + t_perm:.1f} s of CPU work",
               "stages": {"proj_norm_rope_tokens/s": round(passes * S_tok / t_float, 1),
                          "a2a_pack_GB/s": round(3 * passes * 2 * N * D * 2 / t_pack / 1e9, 2),
                          "a2a_unpack_GB/s": round(3 * passes * 2 * N * D * 2 / t_unpack / 1e9, 2),
                          "vmajor_select_GB/s": round(passes * (2 + cfg.n_changed / NT) * N * D * 2 / t_sel / 1e9, 2)}}
        log(f"  cpu oracle: {cpu}")

    out = {
        "metric": METRIC, "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N} tokens ({'x'.join(map(str, cfg.grid))} grid), D={D}, {H} heads x {d}, "
                               f"P={P} logical ranks on one GPU, {cfg.n_changed}/{NT} 16-token V tiles changed",
                   "schedule": args.schedule, "global_batch": 1, "seq_len": N},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "standalone_calls_path": standalone,
        "hip_graph_replay": graph_replay,
        "sender_share_only": layer_only,
        "attainable": attainable,
        "kernels": kernels,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
