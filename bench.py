#!/usr/bin/env python3
"""Benchmark of the Ulysses attention-input path on one MI355X.

A step is one pass of the whole hot path over one synthetic layer input, all P logical ranks, in the V-First
order of the paper's Section III-C (V is projected first; its layout change and selection come before Q's and K's).
Every headline schedule produces every result of the path: the three exchange buffers of the first all-to-all,
head-parallel Q (normalised, rotated), K (same) and V, and the selection's flags, list, count and compact V.

  fused0     one stream:  qkv_proj_fused(V, Q, K in one launch, V's tiles first: every tensor to its exchange buffer and to its
                          head-parallel tensor, norm + RoPE of Q and K in the epilogue) -> vmajor_select(V)
  fused00    one stream:  qkv_proj_fused_select(V, Q, K in one launch: as fused0, and V compared with the previous step's V on its
                          way out, so of the selection only the second pass is launched)
  fused00v   one stream:  qkv_proj_fused_select(V) -> qkv_proj_fused(Q, K)
  fused0v    one stream:  qkv_proj_fused(V) -> qkv_proj_fused(Q, K) -> vmajor_select(V)
  fused0v2   two streams: main qkv_proj_fused(V) -> qkv_proj_fused(Q, K); side [after V's launch] vmajor_select(V); joined at the end
  fused1     one stream:  qkv_proj_pack(V) -> qkv_proj_pack(Q, K) -> a2a_unpack_select(V) -> a2a_unpack_norm_rope(Q, K)
  fused1qkv  one stream:  qkv_proj_pack(V, Q, K in one launch, V's tiles first) -> a2a_unpack_select -> a2a_unpack_norm_rope
  fused2     two streams: main qkv_proj_pack(V) -> qkv_proj_pack(Q, K) -> a2a_unpack_norm_rope(Q, K);
                          side [after V's projection] a2a_unpack_select(V); joined at the end of the step
  fused3     three streams: V, Q, K projected by three launches of qkv_proj_pack, each tensor's unpack under the next projection
(in fused00 / fused00v / fused0 / fused0v / fused0v2 the exchange buffers of Q and K carry normalised values -- norm + RoPE on the sending side, the paper's
order -- in the others the projection itself, normalised by the receiver's unpack).
The default run times all nine with the same --warmup / --steps (three times each, interleaved, after a clock
ramp: see time_headline) and reports each; `value` is the fastest one measured in this run (named in config.schedule).  Also timed and reported beside it: the same step through the five
stand-alone calls only ("vfirst", two streams; "serial", one), the single-GPU direct form that writes V straight
into the head-parallel layout ("fused1_vdirect": no exchange buffer for V), a HIP-graph replay of the headline
schedule, the sender's share alone, every kernel alone (HBM-bound ones on cold data), the per-rank back-to-back
form of the rank-range calls, and the two largest workloads (`other_workloads`).
Inputs are resident in HBM before any timed region.  Prints ONE JSON line on stdout.
"""
import argparse
import glob
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "tokens/s per layer (QKV+norm+RoPE+pack); pack/select GB/s vs HBM peak"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "qkv_gemm_hbm_traffic.txt")
HEADLINE_CANDIDATES = ("fused00", "fused00v", "fused0", "fused0v", "fused0v2", "fused1", "fused1qkv", "fused2", "fused3")


def measured_traffic(workload: str, form: str, kernel_tile: str, launches_per_step: int):
    """Bytes per launch that crossed the L2 <-> memory-fabric boundary for the projection kernel, from the
    committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE runs of this script's --profile-projection mode);
    None if the summary has no line for this workload, this kernel form ("plain" / "fused" / "fused_select"), this tile shape and
    this number of launches per step (a summary of another kernel form does not count)."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if (len(parts) >= 6 and parts[0] == "traffic_bytes_per_launch" and parts[1] == workload and parts[2] == form
                        and parts[3] == kernel_tile and parts[4] == str(launches_per_step)):
                    return int(parts[5])
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class ChipSampler:
    """Shader clock (MHz) and socket power (W) read from the amdgpu hwmon files about every 2 ms by a background
    thread, so that a timed region of a few milliseconds still gets samples; a value that cannot be read is None."""

    def __init__(self):
        hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))
        self.power_file = next((p for d in hw for p in (os.path.join(d, "power1_input"), os.path.join(d, "power1_average")) if os.path.exists(p)), None)
        self.clock_file = next((os.path.join(d, "freq1_input") for d in hw if os.path.exists(os.path.join(d, "freq1_input"))), None)
        # without a hwmon clock file: the driver's clock-level table, whose current entry carries a star ("1: 1846Mhz *")
        self.dpm_file = None if self.clock_file else next(iter(sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))), None)
        cap = next((os.path.join(d, "power1_cap") for d in hw if os.path.exists(os.path.join(d, "power1_cap"))), None)
        self.power_cap_W = self._read(cap, 1e6)
        self.samples = []      # (time, MHz or None, W or None)
        self._stop = threading.Event()
        self._thread = None

    @staticmethod
    def _read(path, scale):
        if not path:
            return None
        try:
            with open(path) as f:
                return int(f.read()) / scale
        except (OSError, ValueError):
            return None

    def _clock(self):
        if self.clock_file:
            return self._read(self.clock_file, 1e6)
        if not self.dpm_file:
            return None
        try:
            with open(self.dpm_file) as f:
                for line in f:
                    if "*" in line:
                        return float(line.split(":")[1].lower().split("mhz")[0])
        except (OSError, ValueError, IndexError):
            pass
        return None

    def _run(self):
        while not self._stop.is_set():
            self.samples.append((time.perf_counter(), self._clock(), self._read(self.power_file, 1e6)))
            time.sleep(0.002)

    def start(self):
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()

    def stop(self):
        self._stop.set()
        if self._thread:
            self._thread.join(timeout=5)

    def window(self, t0, t1):
        """Medians over the samples taken in [t0, t1] (perf_counter times), with the sample count."""
        import numpy as np
        rows = [s for s in self.samples if t0 <= s[0] <= t1]
        mhz = [s[1] for s in rows if s[1] is not None]
        w = [s[2] for s in rows if s[2] is not None]
        return {"sclk_MHz": int(np.median(mhz)) if mhz else None, "power_W": int(np.median(w)) if w else None, "samples": len(rows)}


class Workload:
    """Device buffers of one workload and the step functions over them."""

    def __init__(self, cfg, cd, torch, np, dev):
        from synth import make_layer_inputs, perturb_tiles
        self.cfg, self.cd, self.torch, self.np = cfg, cd, torch, np
        N, D, H, d, P, T = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.tile_tokens
        log(f"bench: {cfg.name} N={N} D={D} H={H}x{d} P={P}; generating inputs")

        def up(a):
            a = np.ascontiguousarray(a)
            return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

        def bf(shape):
            return torch.empty(shape, dtype=torch.int16, device=dev)

        self.up, self.bf = up, bf
        self.inp = inp = make_layer_inputs(cfg)
        self.X, self.Wq, self.Wk, self.Wv = up(inp["X"]), up(inp["Wq"]), up(inp["Wk"]), up(inp["Wv"])
        self.gq, self.gk = up(inp["gamma_q"]), up(inp["gamma_k"])
        self.table = up(cd.rope_table(cfg.grid, cfg.pairs, cfg.theta))
        self.rope = cd.Rope.make(cfg.grid, cfg.pairs, cfg.theta, self.table.data_ptr())
        self.sh = cd.Shape.make(N, D, H, d, P)
        self.q, self.k, self.v = bf((N, D)), bf((N, D)), bf((N, D))
        self.bq, self.bk, self.bv = bf((N * D,)), bf((N * D,)), bf((N * D,))
        self.hq, self.hk, self.hv = bf((H, N, d)), bf((H, N, d)), bf((H, N, d))
        self.NT = cfg.NT
        self.cap = self.NT
        self.ws = torch.empty(max(cd.vmajor_select_workspace_bytes(H, N, d, T), cd.qkv_proj_fused_select_workspace_bytes(self.sh, T), 16),
                              dtype=torch.uint8, device=dev)
        self.flags = torch.empty(self.NT, dtype=torch.int32, device=dev)
        self.idx = torch.empty(self.NT, dtype=torch.int32, device=dev)
        self.n_act = torch.zeros(1, dtype=torch.int32, device=dev)
        self.compact = bf((H, self.cap * T, d))
        self.s_main, self.s_side, self.s_third = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        self.ORDER = cd.RECV_MAJOR
        # previous-step V: this layer's own head-parallel V with a seeded fraction of 16-token tiles perturbed
        cd.qkv_proj(self.sh, self.X, None, None, self.Wv, None, None, self.v)
        cd.a2a_pack(self.sh, self.v, self.bv, self.ORDER)
        cd.a2a_unpack(self.sh, self.bv, self.hv, self.ORDER)
        torch.cuda.synchronize()
        v_prev_host, _ = perturb_tiles(self.bits(self.hv), 1, T, cfg.n_changed, np.random.default_rng(cfg.index), cfg.noise_sigma)
        self.hv_prev = up(v_prev_host)
        del v_prev_host
        self.schedules = {"fused00": self.step_fused00, "fused00v": self.step_fused00v, "fused0": self.step_fused0, "fused0v": self.step_fused0v, "fused0v2": self.step_fused0v2, "fused1": self.step_fused1, "fused1qkv": self.step_fused1qkv, "fused2": self.step_fused2,
                          "fused2x": self.step_fused2x, "fused3": self.step_fused3, "fused3s": self.step_fused3s,
                          "fused1_vdirect": self.step_fused1_vdirect,
                          "vfirst": self.step_vfirst, "vfirst3": self.step_vfirst3, "serial": self.step_serial}

    def bits(self, t):
        return t.cpu().numpy().view(self.np.uint16)

    # -- helpers ---------------------------------------------------------------------------------------------
    def proj(self, rec, stream, call):
        """One projection launch.  With a recorder: a timing event on the launch stream before the step's first
        projection launch and one after its last (none between the launches: an event between two kernels costs the
        step about a percent, and a schedule with a kernel on a second stream more)."""
        if rec is None:
            call(stream)
            return
        if rec.launches_per_step is None:          # counting pass
            rec.count += 1
            call(stream)
            return
        k = rec.count % rec.launches_per_step
        if k == 0:
            rec.begin = self.torch.cuda.Event(enable_timing=True)
            rec.begin.record(stream)
        call(stream)
        if k == rec.launches_per_step - 1:
            end = self.torch.cuda.Event(enable_timing=True)
            end.record(stream)
            rec.spans.append((rec.begin, end))
        rec.count += 1

    def fork(self, src, dst):
        ev = self.torch.cuda.Event()
        ev.record(src)
        dst.wait_event(ev)

    def unpack_select(self, stream):
        c = self.cfg
        self.cd.a2a_unpack_select(self.sh, self.bv, self.ORDER, self.hv, self.hv_prev, c.tile_tokens, c.tau, self.flags, self.idx,
                                  self.n_act, self.compact, self.cap, self.ws, stream=stream)

    def select(self, stream):
        c = self.cfg
        self.cd.vmajor_select(c.H, c.N, c.d, c.tile_tokens, self.hv, self.hv_prev, c.tau, self.flags, self.idx, self.n_act,
                              self.compact, self.cap, self.ws, stream=stream)

    def unpack_norm_rope(self, stream, which="qk"):
        bq, hq, gq = (self.bq, self.hq, self.gq) if "q" in which else (None, None, None)
        bk, hk, gk = (self.bk, self.hk, self.gk) if "k" in which else (None, None, None)
        self.cd.a2a_unpack_norm_rope(self.sh, bq, bk, hq, hk, gq, gk, self.cfg.eps, self.rope, self.ORDER, stream=stream)

    # -- headline schedules (every result of the path) -------------------------------------------------------
    def step_fused0(self, rec=None):
        cd, sh, st, c = self.cd, self.sh, self.s_main, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, self.Wq, self.Wk, self.Wv, self.gq, self.gk, c.eps, self.rope,
                                                       self.bq, self.bk, self.bv, self.ORDER, self.hq, self.hk, self.hv, stream=s))
        self.select(st)

    def step_fused00(self, rec=None):
        cd, sh, st, c = self.cd, self.sh, self.s_main, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_fused_select(sh, self.X, self.Wq, self.Wk, self.Wv, self.gq, self.gk, c.eps, self.rope,
                                                              self.bq, self.bk, self.bv, self.ORDER, self.hq, self.hk, self.hv,
                                                              self.hv_prev, c.tile_tokens, c.tau, self.flags, self.idx, self.n_act,
                                                              self.compact, self.cap, self.ws, stream=s))

    def step_fused00v(self, rec=None):
        cd, sh, st, c = self.cd, self.sh, self.s_main, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_fused_select(sh, self.X, None, None, self.Wv, None, None, c.eps, None,
                                                              None, None, self.bv, self.ORDER, None, None, self.hv,
                                                              self.hv_prev, c.tile_tokens, c.tau, self.flags, self.idx, self.n_act,
                                                              self.compact, self.cap, self.ws, stream=s))
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, self.Wq, self.Wk, None, self.gq, self.gk, c.eps, self.rope,
                                                       self.bq, self.bk, None, self.ORDER, self.hq, self.hk, None, stream=s))

    def step_fused0v(self, rec=None):
        cd, sh, st, c = self.cd, self.sh, self.s_main, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, None, None, self.Wv, None, None, c.eps, None,
                                                       None, None, self.bv, self.ORDER, None, None, self.hv, stream=s))
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, self.Wq, self.Wk, None, self.gq, self.gk, c.eps, self.rope,
                                                       self.bq, self.bk, None, self.ORDER, self.hq, self.hk, None, stream=s))
        self.select(st)

    def step_fused0v2(self, rec=None):
        """fused0v with V's selection on the side stream, under the Q and K launch."""
        cd, sh, st, side, c = self.cd, self.sh, self.s_main, self.s_side, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, None, None, self.Wv, None, None, c.eps, None,
                                                       None, None, self.bv, self.ORDER, None, None, self.hv, stream=s))
        self.fork(st, side)
        self.proj(rec, st, lambda s: cd.qkv_proj_fused(sh, self.X, self.Wq, self.Wk, None, self.gq, self.gk, c.eps, self.rope,
                                                       self.bq, self.bk, None, self.ORDER, self.hq, self.hk, None, stream=s))
        self.select(side)
        self.fork(side, st)

    def step_fused1(self, rec=None):
        cd, sh, st = self.cd, self.sh, self.s_main
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, None, None, self.Wv, None, None, self.bv, self.ORDER, stream=s))
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, self.Wk, None, self.bq, self.bk, None, self.ORDER, stream=s))
        self.unpack_select(st)
        self.unpack_norm_rope(st)

    def step_fused1qkv(self, rec=None):
        cd, sh, st = self.cd, self.sh, self.s_main
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, self.Wk, self.Wv, self.bq, self.bk, self.bv, self.ORDER, stream=s))
        self.unpack_select(st)
        self.unpack_norm_rope(st)

    def step_fused2(self, rec=None):
        """Both projections on the main stream (no cross-stream wait between them); V's unpack, which carries the
        selection's flag pass, waits for V's projection on the side stream and runs under the Q and K projection."""
        cd, sh, st, side = self.cd, self.sh, self.s_main, self.s_side
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, None, None, self.Wv, None, None, self.bv, self.ORDER, stream=s))
        self.fork(st, side)
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, self.Wk, None, self.bq, self.bk, None, self.ORDER, stream=s))
        self.unpack_select(side)
        self.unpack_norm_rope(st)
        self.fork(side, st)                 # join: the next layer cannot start before everything is laid out

    # -- other forms of the step ----------------------------------------------------------------------------
    def step_fused2x(self, rec=None):
        """fused2 with the roles of the streams swapped: the Q and K projection waits behind a cross-stream event."""
        cd, sh, st, side = self.cd, self.sh, self.s_main, self.s_side
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, None, None, self.Wv, None, None, self.bv, self.ORDER, stream=s))
        self.fork(st, side)
        self.unpack_select(st)
        self.proj(rec, side, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, self.Wk, None, self.bq, self.bk, None, self.ORDER, stream=s))
        self.unpack_norm_rope(side)
        self.fork(side, st)

    def step_fused3(self, rec=None):
        """Q and K projected by separate launches, each tensor's unpack under the next projection (three streams)."""
        cd, sh, st, side, third = self.cd, self.sh, self.s_main, self.s_side, self.s_third
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, None, None, self.Wv, None, None, self.bv, self.ORDER, stream=s))
        self.fork(st, side)
        self.unpack_select(st)
        self.proj(rec, side, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, None, None, self.bq, None, None, self.ORDER, stream=s))
        self.fork(side, third)
        self.proj(rec, side, lambda s: cd.qkv_proj_pack(sh, self.X, None, self.Wk, None, None, self.bk, None, self.ORDER, stream=s))
        self.unpack_norm_rope(third, "q")
        self.unpack_norm_rope(side, "k")
        self.fork(third, st)
        self.fork(side, st)

    def step_fused3s(self, rec=None):
        """Norm + RoPE on the sending side, the order the paper describes: qkv_proj -> qk_norm_rope_pack -> a2a_unpack."""
        cd, sh, st, side, third, c = self.cd, self.sh, self.s_main, self.s_side, self.s_third, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, None, None, self.Wv, None, None, self.bv, self.ORDER, stream=s))
        self.fork(st, side)
        self.unpack_select(st)
        self.proj(rec, side, lambda s: cd.qkv_proj(sh, self.X, self.Wq, None, None, self.q, None, None, stream=s))
        self.fork(side, third)
        self.proj(rec, side, lambda s: cd.qkv_proj(sh, self.X, None, self.Wk, None, None, self.k, None, stream=s))
        cd.qk_norm_rope_pack(sh, self.q, None, self.gq, None, c.eps, self.rope, self.bq, None, self.ORDER, stream=third)
        cd.a2a_unpack(sh, self.bq, self.hq, self.ORDER, stream=third)
        cd.qk_norm_rope_pack(sh, None, self.k, None, self.gk, c.eps, self.rope, None, self.bk, self.ORDER, stream=side)
        cd.a2a_unpack(sh, self.bk, self.hk, self.ORDER, stream=side)
        self.fork(third, st)
        self.fork(side, st)

    def step_fused1_vdirect(self, rec=None):
        """Single-GPU direct form for V: its projection writes the head-parallel tensor itself (pack, exchange and
        unpack are the store address), the selection reads it there; no exchange buffer of V exists.  Q and K as in
        fused1."""
        cd, sh, st = self.cd, self.sh, self.s_main
        self.proj(rec, st, lambda s: cd.qkv_proj_hs(sh, self.X, None, None, self.Wv, None, None, self.hv, stream=s))
        self.proj(rec, st, lambda s: cd.qkv_proj_pack(sh, self.X, self.Wq, self.Wk, None, self.bq, self.bk, None, self.ORDER, stream=s))
        self.select(st)
        self.unpack_norm_rope(st)

    def step_vfirst(self, rec=None):
        """The stand-alone calls in fused2's shape: both projections on the main stream, V's pack, unpack and selection
        on the side stream under the Q and K work."""
        cd, sh, st, side, c = self.cd, self.sh, self.s_main, self.s_side, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj(sh, self.X, None, None, self.Wv, None, None, self.v, stream=s))
        self.fork(st, side)
        self.proj(rec, st, lambda s: cd.qkv_proj(sh, self.X, self.Wq, self.Wk, None, self.q, self.k, None, stream=s))
        cd.a2a_pack(sh, self.v, self.bv, self.ORDER, stream=side)
        cd.a2a_unpack(sh, self.bv, self.hv, self.ORDER, stream=side)
        self.select(side)
        cd.qk_norm_rope(sh, self.q, self.k, self.gq, self.gk, c.eps, self.rope, stream=st)
        for src, buf, dst in ((self.q, self.bq, self.hq), (self.k, self.bk, self.hk)):
            cd.a2a_pack(sh, src, buf, self.ORDER, stream=st)
            cd.a2a_unpack(sh, buf, dst, self.ORDER, stream=st)
        self.fork(side, st)

    def step_vfirst3(self, rec=None):
        """V, then Q, then K projected one after the other (the order of the paper's Section III-C); each tensor's
        norm/RoPE and layout change on a side stream under the next tensor's projection."""
        cd, sh, st, side, third, c = self.cd, self.sh, self.s_main, self.s_side, self.s_third, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj(sh, self.X, None, None, self.Wv, None, None, self.v, stream=s))
        self.fork(st, side)
        cd.a2a_pack(sh, self.v, self.bv, self.ORDER, stream=st)
        cd.a2a_unpack(sh, self.bv, self.hv, self.ORDER, stream=st)
        self.select(st)
        self.proj(rec, side, lambda s: cd.qkv_proj(sh, self.X, self.Wq, None, None, self.q, None, None, stream=s))
        self.fork(side, third)
        self.proj(rec, side, lambda s: cd.qkv_proj(sh, self.X, None, self.Wk, None, None, self.k, None, stream=s))
        cd.qk_norm_rope(sh, self.q, None, self.gq, None, c.eps, self.rope, stream=third)
        cd.a2a_pack(sh, self.q, self.bq, self.ORDER, stream=third)
        cd.a2a_unpack(sh, self.bq, self.hq, self.ORDER, stream=third)
        cd.qk_norm_rope(sh, None, self.k, None, self.gk, c.eps, self.rope, stream=side)
        cd.a2a_pack(sh, self.k, self.bk, self.ORDER, stream=side)
        cd.a2a_unpack(sh, self.bk, self.hk, self.ORDER, stream=side)
        self.fork(third, st)
        self.fork(side, st)

    def step_serial(self, rec=None):
        cd, sh, st, c = self.cd, self.sh, self.s_main, self.cfg
        self.proj(rec, st, lambda s: cd.qkv_proj(sh, self.X, None, None, self.Wv, None, None, self.v, stream=s))
        self.proj(rec, st, lambda s: cd.qkv_proj(sh, self.X, self.Wq, self.Wk, None, self.q, self.k, None, stream=s))
        cd.qk_norm_rope(sh, self.q, self.k, self.gq, self.gk, c.eps, self.rope, stream=st)
        for src, buf, dst in ((self.v, self.bv, self.hv), (self.q, self.bq, self.hq), (self.k, self.bk, self.hk)):
            cd.a2a_pack(sh, src, buf, self.ORDER, stream=st)
            cd.a2a_unpack(sh, buf, dst, self.ORDER, stream=st)
        self.select(st)

    # -- timing ----------------------------------------------------------------------------------------------
    def check_selection(self):
        assert int(self.n_act.cpu()[0]) == self.cfg.n_changed, "selection did not find the perturbed tiles"

    def time_steps(self, step_fn, warmup, steps):
        """`warmup` untimed steps, then exactly `steps` steps between two synchronisations.  Returns
        (ms per step, (t0, t1) of the timed region on the perf_counter clock).  The selection's count is checked after
        the timed region (a device-to-host copy in front of it would leave the GPU idle just before the clock starts)."""
        torch = self.torch
        for _ in range(warmup):
            step_fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step_fn()
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        self.check_selection()
        self.enqueue_ms = (t_enq - t0) * 1e3 / steps
        return (t1 - t0) * 1e3 / steps, (t0, t1)

    def projection_in_step(self, step_fn, steps):
        """A pass of its own (outside every headline timing): `steps` steps with two HIP events each, one before the
        step's first projection launch and one after its last, each on its launch stream.  Returns (average launch
        duration in us = span / launches, launches per step, ms per step of this instrumented pass).  When a step's
        projections sit on one stream back to back (every schedule but fused3 / fused3s / vfirst3) the span holds nothing
        but them."""
        torch = self.torch

        class Rec:
            launches_per_step = None
            count = 0
            begin = None
            spans = []

        rec = Rec()
        rec.spans = []
        step_fn(rec)                               # counts the projection launches of a step
        rec.launches_per_step, rec.count = rec.count, 0
        # the same clock ramp as in front of the headline timings: after even a few milliseconds of idling (the host
        # summarising the previous measurement) the next tens of milliseconds run up to 10 % slow
        t_ramp = time.perf_counter()
        while time.perf_counter() - t_ramp < RAMP_SECONDS:
            for _ in range(8):
                step_fn()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step_fn(rec)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        total_us = sum(e0.elapsed_time(e1) for e0, e1 in rec.spans) * 1e3
        return total_us / (len(rec.spans) * rec.launches_per_step), float(rec.launches_per_step), ms

    def tile_name(self, n_tensors, whole_heads=False):
        p = self.cd.qkv_proj_plan(self.sh, n_tensors, whole_heads)
        return f"{p['tile_tokens']}x{p['tile_features']}"


def timed_blocks(torch, fns, blocks=7):
    """us per call: median and minimum over `blocks` blocks of one pass over `fns` (at least 8 calls) between two HIP
    events on torch's current stream."""
    st = torch.cuda.current_stream()
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
    return t[len(t) // 2], t[0]


RAMP_SECONDS = 0.3
REPEATS = 3


def time_headline(w, names, warmup, steps, sampler):
    """Every schedule in `names` with the same warm-up and step count; returns ({name: entry}, fastest name).

    Input generation leaves the GPU idle for seconds and its clocks low, and a few warm-up steps (some milliseconds)
    do not bring them back; after that the chip's power management overshoots and settles over tens of milliseconds,
    so a region of `steps` steps a few milliseconds long is charged for whatever state it starts in.  Therefore:
    the first schedule is timed once straight away ("after_idle": reported, not used); then the schedules run
    round-robin for RAMP_SECONDS; then every schedule is timed REPEATS times, interleaved (A B C A B C ...), each time
    with its own `warmup` steps in front and exactly `steps` steps timed.  A schedule's figure is the median of its
    REPEATS measurements; all of them are reported."""
    ms_idle, _ = w.time_steps(w.schedules[names[0]], warmup, steps)
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < RAMP_SECONDS:
        for name in names:
            w.schedules[name]()
        w.torch.cuda.synchronize()
    runs = {name: [] for name in names}
    for rep in range(REPEATS):
        for name in names:
            ms, win = w.time_steps(w.schedules[name], warmup, steps)
            runs[name].append((ms, win, w.enqueue_ms))
    out = {}
    for name in names:
        ordered = sorted(runs[name], key=lambda r: r[0])
        ms, (t0, t1), enq = ordered[len(ordered) // 2]
        out[name] = {"ms_per_step": round(ms, 4), "value": round(w.cfg.N / (ms * 1e-3), 1),
                     "all_ms_per_step": [round(r[0], 4) for r in runs[name]], "host_enqueue_ms_per_step": round(enq, 4)}
        if sampler:
            out[name]["chip"] = sampler.window(t0, t1)
        log(f"  schedule {name}: {out[name]}")
    best = min(out, key=lambda n: out[n]["ms_per_step"])
    out[names[0]]["after_idle"] = {"ms_per_step": round(ms_idle, 4), "note": f"timed first, straight after input generation, before the {RAMP_SECONDS} s ramp"}
    return out, best


def roofline_of(w, schedule, steps):
    """The projection inside the step: an instrumented pass of the schedule."""
    cfg = w.cfg
    us, per_step, ms_instr = w.projection_in_step(w.schedules[schedule], steps)
    flops_per_launch = 2.0 * cfg.N * (3 * cfg.D) * cfg.D / per_step
    achieved = flops_per_launch / us / 1e6
    fused = schedule.startswith("fused0")
    form = "fused_select" if schedule.startswith("fused00") else "fused" if fused else "plain"
    tile = w.tile_name(3 if per_step == 1 else 2, fused)
    return {"kernel": "qkv_gemm_direct_kernel" + (" (norm + RoPE epilogue, two destinations)" if fused else ""), "tile": tile, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(cfg.name, form, tile, int(round(per_step))),
            "avg_launch_us": round(us, 2), "launches_per_step": round(per_step, 2), "event_steps": steps,
            "ms_per_step_instrumented": round(ms_instr, 4)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--schedule", default="auto", help="auto = time fused1, fused1qkv and fused2, report the fastest; or one schedule's name")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true")
    ap.add_argument("--profile-projection", type=int, default=0, metavar="N",
                    help="profiling aid for rocprofv3 counter runs: N launches each of the projection with one, two and three "
                         "weights (exchange-buffer epilogue), of the fused form with three weights, of a2a_unpack_select and "
                         "vmajor_select, and of a 1000 MiB calibration copy, and nothing else")
    ap.add_argument("--profile-fused-select", action="store_true",
                    help="with --profile-projection: launch cocodiff_qkv_proj_fused_select instead (V alone, then V, Q and K), "
                         "its selection pass and the calibration copy")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs all P logical ranks of the path on ONE GPU; "
            "there is no multi-GPU path to time (--gpus must be 1).")
        return 2

    import numpy as np
    import torch

    import paper_2604_14561_amd as cd
    from synth import CONFIGS

    if not os.path.exists(cd.binding.LIB_PATH):
        from paper_2604_14561_amd import build as _build
        _build.build()

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    sampler = ChipSampler()
    sampler.start()

    cfg = CONFIGS[args.config]
    N, D, H, d, P, T = cfg.N, cfg.D, cfg.H, cfg.d, cfg.P, cfg.tile_tokens
    w = Workload(cfg, cd, torch, np, dev)
    if args.schedule != "auto" and args.schedule not in w.schedules:
        log(f"bench.py: unknown schedule {args.schedule}; one of {sorted(w.schedules)}")
        return 2
    if args.profile_projection:
        big = 1000 << 20
        src_big = torch.empty(big + (3 << 20), dtype=torch.uint8, device=dev)
        dst_big = torch.empty(big, dtype=torch.uint8, device=dev)
        c_ = cfg
        for _ in range(args.profile_projection if args.profile_fused_select else 0):
            cd.qkv_proj_fused_select(w.sh, w.X, None, None, w.Wv, None, None, c_.eps, None, None, None, w.bv, w.ORDER, None, None, w.hv,
                                     w.hv_prev, c_.tile_tokens, c_.tau, w.flags, w.idx, w.n_act, w.compact, w.cap, w.ws)
            cd.qkv_proj_fused_select(w.sh, w.X, w.Wq, w.Wk, w.Wv, w.gq, w.gk, c_.eps, w.rope, w.bq, w.bk, w.bv, w.ORDER, w.hq, w.hk, w.hv,
                                     w.hv_prev, c_.tile_tokens, c_.tau, w.flags, w.idx, w.n_act, w.compact, w.cap, w.ws)
            cd.util_copy(src_big, dst_big, big)
        for _ in range(0 if args.profile_fused_select else args.profile_projection):
            cd.qkv_proj_pack(w.sh, w.X, None, None, w.Wv, None, None, w.bv, w.ORDER)
            cd.qkv_proj_pack(w.sh, w.X, w.Wq, w.Wk, None, w.bq, w.bk, None, w.ORDER)
            cd.qkv_proj_pack(w.sh, w.X, w.Wq, w.Wk, w.Wv, w.bq, w.bk, w.bv, w.ORDER)
            cd.qkv_proj_fused(w.sh, w.X, None, None, w.Wv, None, None, cfg.eps, None, None, None, w.bv, w.ORDER, None, None, w.hv)
            cd.qkv_proj_fused(w.sh, w.X, w.Wq, w.Wk, None, w.gq, w.gk, cfg.eps, w.rope, w.bq, w.bk, None, w.ORDER, w.hq, w.hk, None)
            cd.qkv_proj_fused(w.sh, w.X, w.Wq, w.Wk, w.Wv, w.gq, w.gk, cfg.eps, w.rope, w.bq, w.bk, w.bv, w.ORDER, w.hq, w.hk, w.hv)
            w.unpack_select(None)
            w.select(None)
            cd.util_copy(src_big, dst_big, big)
        torch.cuda.synchronize()
        sampler.stop()
        print(json.dumps({"profile_projection": args.profile_projection, "workload": cfg.name,
                          "plans": {str(n_): cd.qkv_proj_plan(w.sh, n_) for n_ in (1, 2, 3)}, "copy_bytes": big}), flush=True)
        return 0
    names = HEADLINE_CANDIDATES if args.schedule == "auto" else (args.schedule,)
    per_schedule, best = time_headline(w, names, args.warmup, args.steps, sampler)
    ms_per_step = per_schedule[best]["ms_per_step"]
    tokens_per_s = per_schedule[best]["value"]
    log(f"  headline: {best} {ms_per_step} ms per step; all: { {k_: v_['ms_per_step'] for k_, v_ in per_schedule.items()} }")
    roofline = roofline_of(w, best, max(args.steps, 50))
    roofline["chip_during_headline"] = per_schedule[best].get("chip")

    # ---- the same step in other forms, reported beside the headline ----
    other_forms, graph_replay, layer_only = {}, None, None
    if not args.no_breakdown:
        for name in ("vfirst", "serial", "fused1_vdirect"):
            if name not in per_schedule:
                log(f"  schedule {name}")
                ms, _ = w.time_steps(w.schedules[name], args.warmup, args.steps)
                other_forms[name] = {"ms_per_step": round(ms, 4), "value": round(N / (ms * 1e-3), 1)}
        other_forms["vfirst"]["note"] = "the five stand-alone calls only, two streams"
        other_forms["serial"]["note"] = "the five stand-alone calls only, one stream"
        other_forms["fused1_vdirect"]["note"] = ("V's projection writes the head-parallel tensor itself (no exchange buffer for V); "
                                                 "every other result as in the headline schedules")
        # the headline step replayed from a HIP graph: what is left when the host's launch work is taken out
        try:
            graph = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=w.s_main):
                w.schedules[best]()
            for _ in range(args.warmup):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            ms_g = (time.perf_counter() - t0) * 1e3 / args.steps
            w.check_selection()
            graph_replay = {"schedule": best, "ms_per_step": round(ms_g, 4), "value": round(N / (ms_g * 1e-3), 1), "unit": "tokens/s"}
            log(f"  HIP graph replay of the step: {graph_replay}")
            del graph
        except Exception as e:      # reported, never fatal: the headline is the eager step
            log(f"  HIP graph replay not measured: {e}")

        # The sender's share alone -- projection of Q, K, V + norm and RoPE of Q and K + the three packs, up to the
        # filled exchange buffers (the layer's work before the all-to-all); `value` above is the longer path that
        # also holds the receiver's unpack and the selection.
        sh, st, side, O = w.sh, w.s_main, w.s_side, w.ORDER

        def sender_serial():
            cd.qkv_proj(sh, w.X, w.Wq, w.Wk, w.Wv, w.q, w.k, w.v, stream=st)
            cd.qk_norm_rope(sh, w.q, w.k, w.gq, w.gk, cfg.eps, w.rope, stream=st)
            for src, buf in ((w.v, w.bv), (w.q, w.bq), (w.k, w.bk)):
                cd.a2a_pack(sh, src, buf, O, stream=st)

        def sender_vfirst():
            cd.qkv_proj(sh, w.X, None, None, w.Wv, None, None, w.v, stream=st)
            w.fork(st, side)
            cd.a2a_pack(sh, w.v, w.bv, O, stream=st)
            cd.qkv_proj(sh, w.X, w.Wq, w.Wk, None, w.q, w.k, None, stream=side)
            cd.qk_norm_rope(sh, w.q, w.k, w.gq, w.gk, cfg.eps, w.rope, stream=side)
            cd.a2a_pack(sh, w.q, w.bq, O, stream=side)
            cd.a2a_pack(sh, w.k, w.bk, O, stream=side)
            w.fork(side, st)

        def sender_fused():
            cd.qkv_proj_pack(sh, w.X, None, None, w.Wv, None, None, w.bv, O, stream=st)
            cd.qkv_proj(sh, w.X, w.Wq, w.Wk, None, w.q, w.k, None, stream=st)
            cd.qk_norm_rope_pack(sh, w.q, w.k, w.gq, w.gk, cfg.eps, w.rope, w.bq, w.bk, O, stream=st)

        layer_only = {}
        for label, fn in (("serial_one_stream", sender_serial), ("vfirst_two_streams", sender_vfirst),
                          ("fused_calls_one_stream", sender_fused)):
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

    # ---- per-kernel times, each launched alone on one stream (not part of `value`) ----
    # HBM-bound kernels are timed "cold": successive launches rotate over buffer sets whose footprint is more than
    # twice the 256 MB last-level cache, so no launch finds its input there; "warm" repeats one set.
    kernels, attainable = {}, None
    if not args.no_breakdown:
        tensor_bytes = N * D * 2
        sh, O = w.sh, w.ORDER
        X, Wq, Wk, Wv, q, k, v, bv = w.X, w.Wq, w.Wk, w.Wv, w.q, w.k, w.v, w.bv
        flags, idx, n_act, compact, cap, ws = w.flags, w.idx, w.n_act, w.compact, w.cap, w.ws

        def add(name, fns, flops=None, nbytes=None, extra=None):
            med, mn = timed_blocks(torch, fns)
            ent = {"us": round(med, 2), "us_min": round(mn, 2)}
            if len(fns) > 1:
                ent["us_warm"] = round(timed_blocks(torch, fns[:1])[0], 2)
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
            if extra:
                ent.update(extra)
            kernels[name] = ent
            return med

        def chip_state_during(fn, secs=1.0):
            t_begin = time.perf_counter()
            while time.perf_counter() < t_begin + secs:
                for _ in range(20):
                    fn()
                torch.cuda.synchronize()
            return sampler.window(t_begin + 0.3, time.perf_counter())      # the first samples still see the ramp

        # what the chip attains on the two calibration kernels: a 1000 MiB copy and a register-only MFMA loop
        big = 1000 << 20   # not a power of two: source and destination must not alias onto the same HBM banks
        src_big = torch.empty(big + (3 << 20), dtype=torch.uint8, device=dev)
        dst_big = torch.empty(big, dtype=torch.uint8, device=dev)
        copy_us = timed_blocks(torch, [lambda: cd.util_copy(src_big, dst_big, big)])[0]
        memcpy_us = timed_blocks(torch, [lambda: dst_big.copy_(src_big[:big])])[0]      # the runtime's own device-to-device copy
        del src_big, dst_big
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        mfma_flops = cd.util_mfma_rate(1024, 2048, sink)
        mfma_us = timed_blocks(torch, [lambda: cd.util_mfma_rate(1024, 2048, sink)])[0]
        attainable = {"hbm_copy_GB/s": round(2 * big / copy_us / 1e3, 1), "runtime_memcpy_GB/s": round(2 * big / memcpy_us / 1e3, 1),
                      "mfma_loop_TFLOP/s": round(mfma_flops / mfma_us / 1e6, 1)}
        log(f"  attainable on this GPU: {attainable}")

        g1 = 2.0 * N * D * D
        add("qkv_proj_v", [lambda: cd.qkv_proj(sh, X, None, None, Wv, None, None, v)], flops=g1, extra={"tile": w.tile_name(1)})
        add("qkv_proj_qk", [lambda: cd.qkv_proj(sh, X, Wq, Wk, None, q, k, None)], flops=2 * g1, extra={"tile": w.tile_name(2)})
        add("qkv_proj_qkv", [lambda: cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v)], flops=3 * g1, extra={"tile": w.tile_name(3)})
        add("qkv_proj_pack_v", [lambda: cd.qkv_proj_pack(sh, X, None, None, Wv, None, None, bv, O)], flops=g1)
        add("qkv_proj_hs_v", [lambda: cd.qkv_proj_hs(sh, X, None, None, Wv, None, None, w.hv)], flops=g1)
        add("qkv_proj_pack_qkv", [lambda: cd.qkv_proj_pack(sh, X, Wq, Wk, Wv, w.bq, w.bk, bv, O)], flops=3 * g1)
        add("qkv_proj_fused_qkv", [lambda: cd.qkv_proj_fused(sh, X, Wq, Wk, Wv, w.gq, w.gk, cfg.eps, w.rope, w.bq, w.bk, bv, O, w.hq, w.hk, w.hv)],
            flops=3 * g1, extra={"tile": w.tile_name(3, True)})
        alone_key = "qkv_proj_fused_qkv" if best.startswith("fused0") else "qkv_proj_pack_qkv"
        roofline["alone"] = {"frac": kernels[alone_key]["frac_mfma_peak"], "TFLOP/s": kernels[alone_key]["TFLOP/s"],
                             "launch": alone_key.replace("_qkv", "") + ", three weights, nothing beside it"}

        # rotation sets: a (token-major), b (exchange buffer), h and p (head-parallel current / previous V; never written)
        R = int(min(64, max(1, -(-(640 << 20) // (2 * tensor_bytes)))))
        sets = []
        for i in range(R):
            sets.append({"a": v.clone(), "b": bv.clone(), "h": w.hv if i == 0 else w.hv.clone(),
                         "p": w.hv_prev if i == 0 else w.hv_prev.clone()})
        log(f"  cold timings rotate over {R} buffer sets of 4 x {tensor_bytes / 1e6:.1f} MB")
        f_act = cfg.n_changed / w.NT
        act = w.bf((H, cap * T, d))
        metric = torch.empty(N, dtype=torch.float32, device=dev)
        tok_idx = torch.empty(N, dtype=torch.int32, device=dev)
        tok_n = torch.zeros(P, dtype=torch.int32, device=dev)
        k_act = cd.cache_active_count(27, 50, 5, 10, N // P)  # mid-schedule step of the paper's 50-step setup
        gq, gk, rope = w.gq, w.gk, w.rope

        def each(fn):
            return [(lambda s_=s_: fn(s_)) for s_ in sets]

        add("vmajor_select", each(lambda s_: cd.vmajor_select(H, N, d, T, s_["h"], s_["p"], cfg.tau, flags, idx, n_act, compact, cap, ws)),
            nbytes=(2 + f_act) * tensor_bytes)
        add("a2a_unpack_select", each(lambda s_: cd.a2a_unpack_select(sh, s_["b"], O, s_["a"], s_["p"], T, cfg.tau, flags, idx, n_act, compact, cap, ws)),
            nbytes=(3 + f_act) * tensor_bytes)
        assert int(n_act.cpu()[0]) == cfg.n_changed, "the breakdown's selection inputs were disturbed"
        add("vmajor_token_metric", each(lambda s_: cd.vmajor_token_metric(H, N, d, s_["h"], s_["p"], metric)), nbytes=2 * tensor_bytes)
        add("vmajor_topk", [lambda: cd.vmajor_topk(P, N // P, metric, k_act, tok_idx, tok_n)])   # every rank ranks its own tokens
        add("vmajor_gather", each(lambda s_: cd.vmajor_gather(H, N, d, T, s_["h"], idx, n_act, act, cap)), nbytes=2 * f_act * tensor_bytes)
        add("vmajor_scatter", each(lambda s_: cd.vmajor_scatter(H, N, d, T, act, idx, n_act, s_["a"], cap)), nbytes=2 * f_act * tensor_bytes)
        add("a2a_pack_hs", each(lambda s_: cd.a2a_pack_hs(sh, s_["h"], s_["b"], O)), nbytes=2 * tensor_bytes)
        add("a2a_unpack_seq", each(lambda s_: cd.a2a_unpack_seq(sh, s_["b"], s_["a"], O)), nbytes=2 * tensor_bytes)
        us_pack = add("a2a_pack", each(lambda s_: cd.a2a_pack(sh, s_["a"], s_["b"], O)), nbytes=2 * tensor_bytes)
        us_unpack = add("a2a_unpack", each(lambda s_: cd.a2a_unpack(sh, s_["b"], s_["a"], O)), nbytes=2 * tensor_bytes)
        us_nr = add("qk_norm_rope", each(lambda s_: cd.qk_norm_rope(sh, s_["a"], s_["b"], gq, gk, cfg.eps, rope)), nbytes=4 * tensor_bytes)
        add("a2a_unpack_norm_rope", each(lambda s_: cd.a2a_unpack_norm_rope(sh, s_["h"], s_["p"], s_["a"], s_["b"], gq, gk, cfg.eps, rope, O)),
            nbytes=4 * tensor_bytes)
        add("qk_norm_rope_pack", each(lambda s_: cd.qk_norm_rope_pack(sh, s_["h"], s_["p"], gq, gk, cfg.eps, rope, s_["a"], s_["b"], O)),
            nbytes=4 * tensor_bytes)
        add("copy_same_bytes", each(lambda s_: cd.util_copy(s_["a"], s_["b"], tensor_bytes)), nbytes=2 * tensor_bytes)

        # The per-rank back-to-back form: P launches, each covering one logical rank's share (rank_count = 1), for the
        # calls that take a rank range; "us" is the whole group of P launches, to compare with the one launch above.
        ranks = [cd.Shape.make(N, D, H, d, P, r, 1) for r in range(P)]

        def group(fn):
            def run(s_):
                for shr in ranks:
                    fn(shr, s_)
            return run

        us_proj_all = kernels["qkv_proj_qkv"]["us"]
        for name, fn, batched_us, kw in (
                ("qkv_proj_qkv_per_rank", lambda shr, s_: cd.qkv_proj(shr, X, Wq, Wk, Wv, q, k, v), us_proj_all, {"flops": 3 * g1}),
                ("qk_norm_rope_per_rank", lambda shr, s_: cd.qk_norm_rope(shr, s_["a"], s_["b"], gq, gk, cfg.eps, rope), us_nr, {"nbytes": 4 * tensor_bytes}),
                ("a2a_pack_per_rank", lambda shr, s_: cd.a2a_pack(shr, s_["a"], s_["b"], O), us_pack, {"nbytes": 2 * tensor_bytes}),
                ("a2a_unpack_per_rank", lambda shr, s_: cd.a2a_unpack(shr, s_["b"], s_["a"], O), us_unpack, {"nbytes": 2 * tensor_bytes})):
            fns = [lambda: group(fn)(sets[0])] if "flops" in kw else each(group(fn))
            med = add(name, fns, extra={"launches": P}, **kw)
            kernels[name]["vs_one_launch"] = round(med / batched_us, 3)
            kernels[name].pop("us_warm", None)
        kernels["qkv_proj_qkv_per_rank"]["tile"] = "{tile_tokens}x{tile_features}".format(**cd.qkv_proj_plan(ranks[0], 3))

        kernels["copy_1000MiB"] = {"us": round(copy_us, 2), "GB/s": attainable["hbm_copy_GB/s"],
                                   "frac_hbm_peak": round(attainable["hbm_copy_GB/s"] / PEAK_HBM_GBS, 4)}
        kernels["mfma_register_loop"] = {"us": round(mfma_us, 2), "TFLOP/s": attainable["mfma_loop_TFLOP/s"],
                                         "frac_mfma_peak": round(attainable["mfma_loop_TFLOP/s"] / PEAK_BF16_TFLOPS, 4)}
        del sets, act
        # the chip does not hold its top clock under matrix-core load: record what it runs at (last: the throttled
        # state lingers and would colour the timings above)
        src2 = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst2 = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        state = {"copy": chip_state_during(lambda: cd.util_copy(src2, dst2, 256 << 20)),
                 "mfma_loop": chip_state_during(lambda: cd.util_mfma_rate(1024, 512, sink)),
                 "projection": chip_state_during(lambda: cd.qkv_proj(sh, X, Wq, Wk, Wv, q, k, v))}
        del src2, dst2
        attainable["sclk_MHz"] = {k_: v_["sclk_MHz"] for k_, v_ in state.items()}
        attainable["power_W"] = {k_: v_["power_W"] for k_, v_ in state.items()}
        attainable["power_cap_W"] = int(sampler.power_cap_W) if sampler.power_cap_W else None
        log(f"  chip state under load: clocks {attainable['sclk_MHz']} MHz, socket power {attainable['power_W']} W")
        roofline["frac_of_mfma_loop"] = round(roofline["achieved"] / attainable["mfma_loop_TFLOP/s"], 4)
        if attainable["sclk_MHz"]["projection"]:
            # the published peak is 2.4 GHz x 256 units x 4 SIMDs x 1024 flop/clk; the same at the clock the chip holds
            roofline["sclk_MHz_projection_alone"] = attainable["sclk_MHz"]["projection"]
            roofline["frac_at_sclk"] = round(roofline["achieved"] / (PEAK_BF16_TFLOPS * attainable["sclk_MHz"]["projection"] / 2400.0), 4)
        for name, ent in kernels.items():
            log(f"  {name:24s} {ent}")

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_c()
        inp = w.inp
        S_tok = min(N, 24576)                                # float stages: the first S_tok tokens per pass
        ids = np.arange(S_tok)
        host_seq = w.bits(w.v).reshape(N, H, d)
        host_prev = w.bits(w.hv_prev)
        t_float = t_perm = t_pack = t_unpack = t_sel = 0.0
        passes = 0
        while t_float + t_perm < 12.0 and passes < 200:      # about 10-30 s of CPU work in whole passes
            t_a = time.perf_counter()
            o = {}
            for name, wn in (("q", "Wq"), ("k", "Wk"), ("v", "Wv")):
                o[name] = oracle.qkv_proj(inp["X"][:S_tok], inp[wn])
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
            blas_threads = max([p_.get("num_threads", 1) for p_ in threadpool_info() if p_.get("user_api") == "blas"] or [1])
        except Exception:
            blas_threads = os.cpu_count() or 1
        omp_threads = oracle.omp_max_threads()
        nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cpu = {"value": round(1.0 / per_token, 1), "unit": "tokens/s", "cores": int(max(blas_threads, omp_threads)), "kind": "oracle",
               "threads": {"blas_fp64_matmul": int(blas_threads), "openmp_index_loops": int(omp_threads), "nproc": int(nproc),
                           "cpu_count": int(os.cpu_count() or 0)},
               "sample": f"{passes} passes of the oracle over the workload (fp64 projection + norm + RoPE on "
                         f"{S_tok} of {N} tokens per pass; pack/unpack x3 and select on the full tensors): "
                         f"{t_float + t_perm:.1f} s of CPU work",
               "stages": {"proj_norm_rope_tokens/s": round(passes * S_tok / t_float, 1),
                          "a2a_pack_GB/s": round(3 * passes * 2 * N * D * 2 / t_pack / 1e9, 2),
                          "a2a_unpack_GB/s": round(3 * passes * 2 * N * D * 2 / t_unpack / 1e9, 2),
                          "vmajor_select_GB/s": round(passes * (2 + cfg.n_changed / w.NT) * N * D * 2 / t_sel / 1e9, 2)}}
        log(f"  cpu oracle: {cpu}")

    # ---- the two largest workloads, same schedules, same warm-up and step count ----
    others = None
    if not args.no_other_workloads and args.schedule == "auto" and cfg.name == "C3":
        del w
        torch.cuda.empty_cache()
        others = {}
        for name in ("C4", "C5"):
            ow = Workload(CONFIGS[name], cd, torch, np, dev)
            oc = ow.cfg
            sched, obest = time_headline(ow, HEADLINE_CANDIDATES, args.warmup, args.steps, sampler)
            ent = {"workload": f"N={oc.N} tokens, P={oc.P}", "schedule": obest, "ms_per_step": sched[obest]["ms_per_step"],
                   "value": sched[obest]["value"], "unit": "tokens/s", "schedules": sched,
                   "roofline": roofline_of(ow, obest, max(args.steps, 50))}
            tb = oc.N * oc.D * 2
            g3 = 6.0 * oc.N * oc.D * oc.D
            if obest.startswith("fused0"):
                alone_fn = lambda: cd.qkv_proj_fused(ow.sh, ow.X, ow.Wq, ow.Wk, ow.Wv, ow.gq, ow.gk, oc.eps, ow.rope, ow.bq, ow.bk, ow.bv,
                                                     ow.ORDER, ow.hq, ow.hk, ow.hv)
            else:
                alone_fn = lambda: cd.qkv_proj_pack(ow.sh, ow.X, ow.Wq, ow.Wk, ow.Wv, ow.bq, ow.bk, ow.bv, ow.ORDER)
            us_alone = timed_blocks(torch, [alone_fn], blocks=3)[0]
            ent["roofline"]["alone"] = {"frac": round(g3 / us_alone / 1e6 / PEAK_BF16_TFLOPS, 4), "TFLOP/s": round(g3 / us_alone / 1e6, 1),
                                        "launch": ("qkv_proj_fused" if obest.startswith("fused0") else "qkv_proj_pack") + ", three weights, nothing beside it"}
            f_o = oc.n_changed / ow.NT
            hbm = {}
            for kname, fn, nb in (("a2a_unpack_select", lambda: ow.unpack_select(None), (3 + f_o) * tb),
                                  ("vmajor_select", lambda: ow.select(None), (2 + f_o) * tb),
                                  ("a2a_unpack_norm_rope", lambda: ow.unpack_norm_rope(None), 4 * tb),
                                  ("a2a_pack", lambda: cd.a2a_pack(ow.sh, ow.v, ow.bv, ow.ORDER), 2 * tb),
                                  ("a2a_unpack", lambda: cd.a2a_unpack(ow.sh, ow.bv, ow.hv, ow.ORDER), 2 * tb)):
                us = timed_blocks(torch, [fn], blocks=3)[0]     # tensors of 127 MB and 613 MB: beyond the last-level cache as they are
                hbm[kname] = {"us": round(us, 2), "GB/s": round(nb / us / 1e3, 1), "frac_hbm_peak": round(nb / us / 1e3 / PEAK_HBM_GBS, 4)}
            ent["kernels_alone"] = hbm
            others[name] = ent
            log(f"  {name}: {ent}")
            del ow
            torch.cuda.empty_cache()
    sampler.stop()

    out = {
        "metric": METRIC, "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N} tokens ({'x'.join(map(str, cfg.grid))} grid), D={D}, {H} heads x {d}, "
                               f"P={P} logical ranks on one GPU, {cfg.n_changed}/{cfg.NT} 16-token V tiles changed",
                   "schedule": best, "global_batch": 1, "seq_len": N},
        "schedules": per_schedule,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "other_forms_of_the_step": other_forms or None,
        "hip_graph_replay": graph_replay,
        "sender_share_only": layer_only,
        "other_workloads": others,
        "attainable": attainable,
        "kernels": kernels,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
