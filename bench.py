#!/usr/bin/env python3
"""Benchmark of the per-layer KV-cache selection pass on one MI355X.

A step is one whole pass (criticalkv_score -> criticalkv_select -> criticalkv_compact) over one
synthetic layer whose inputs are already resident in HBM.  Prints ONE JSON line:
metric = M KV entries scored+selected per second (one entry = one (batch item, kv head, token)),
with the roofline of the dominant kernel (the bf16 MFMA projection ||V W^O||_1), the other workload
shapes timed in the same run, and the float64 CPU oracle run on the same inputs as a baseline and as
the parity reference (score errors, swapped indices under the tie rule).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM-side bytes per launch of the projection kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (FETCH_SIZE x 2.00, WRITE_SIZE x 1.00 after calibration against a 1 GiB device copy); the runs and the
# calibration are written up in profiles/whole_pass_llama_hbm_counters.md.  None where not measured.
VPROJ_TRAFFIC_BYTES = {"llama32k": int(190.0 * 2**20), "llama128k": int(607.1 * 2**20), "qwen128k": int(1751.4 * 2**20)}
# the same for the Gram-matrix kernel of the L2 variant (95.2 + 4.0 and 383.3 + 16.0 MiB)
L2_TRAFFIC_BYTES = {"llama32k": int(77.2 * 2**20), "llama128k": int(281.8 * 2**20)}


class HipEvents:
    """hipEvent_t handles from the process's HIP runtime (recorded by the library on the launch stream)."""

    def __init__(self, hip):
        self.hip = hip
        hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def new(self):
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        assert rc == 0 and e.value, f"hipEventCreate failed ({rc})"
        self.made.append(e)
        return e

    def record(self, e, stream):
        rc = self.hip.hipEventRecord(e, stream)
        assert rc == 0, f"hipEventRecord failed ({rc})"

    def ms(self, a, b):
        out = ctypes.c_float()
        rc = self.hip.hipEventSynchronize(b)
        assert rc == 0
        rc = self.hip.hipEventElapsedTime(ctypes.byref(out), a, b)
        assert rc == 0, f"hipEventElapsedTime failed ({rc})"
        return float(out.value)

    def close(self):
        for e in self.made:
            self.hip.hipEventDestroy(e)
        self.made = []


def gpu_power_state():
    """Engine-clock level and power cap of the first GPU as sysfs shows them right after the run (None where the
    files cannot be read).  The published peaks assume 2.4 GHz; under this load the chip is power limited."""
    import glob
    out = {}
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))[:1]:
        try:
            lines = open(path).read().split("\n")
            out["sclk_levels"] = [l.strip() for l in lines if l.strip()]
        except OSError:
            pass
        for cap in glob.glob(os.path.join(os.path.dirname(path), "hwmon", "hwmon*", "power1_cap")):
            try:
                out["power_cap_w"] = int(open(cap).read()) / 1e6
            except (OSError, ValueError):
                pass
    return out or None


class PowerSampler:
    """Samples the first GPU's board power (hwmon power1_input, microwatts) from a thread while a loop of passes
    runs; the sensor is slow, so the loop has to last some tenths of a second for the reading to settle."""

    def __init__(self):
        import glob
        files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.path = files[0] if files else None
        clk = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.clk_path = clk[0] if clk else None
        self.samples = []
        self.clocks = []  # MHz of the engine-clock level marked current
        self._stop = False
        self._thread = None

    def _run(self):
        while not self._stop:
            try:
                self.samples.append(int(open(self.path).read()) / 1e6)
            except (OSError, ValueError):
                return
            try:
                for line in open(self.clk_path).read().split("\n"):
                    if line.strip().endswith("*"):
                        self.clocks.append(float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip()))
            except (OSError, ValueError, IndexError, TypeError):
                pass
            time.sleep(0.005)

    def __enter__(self):
        if self.path:
            import threading
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._thread:
            self._thread.join()

    def summary(self):
        if not self.samples:
            return None
        tail = self.samples[len(self.samples) // 2:]  # the second half: the sensor has caught up with the load
        out = {"samples": len(self.samples), "mean_w_second_half": round(sum(tail) / len(tail), 1),
               "max_w": round(max(self.samples), 1)}
        if self.clocks:
            ctail = self.clocks[len(self.clocks) // 2:]
            out["sclk_mhz_mean_second_half"] = round(sum(ctail) / len(ctail), 1)
            out["sclk_mhz_min"] = round(min(self.clocks), 1)
        return out


class Workload:
    """One workload's layers resident in HBM, the output buffers of `n_streams` lanes, and the pass itself."""

    def __init__(self, P, cfg, norm, n_streams, n_sets, gen_threads, ev, want_vnorm=False):
        import numpy as np
        import torch
        from concurrent.futures import ThreadPoolExecutor
        from paper_2502_03805_amd.marshal import cfg_desc, to_device
        from workload import make_layer
        self.P, self.cfg, self.norm, self.ev = P, cfg, norm, ev
        b, H, Hkv, n, dh = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim
        self.esize = 2 if cfg.dtype == "bf16" else 4
        self.kv_bytes = 2 * b * Hkv * n * dh * self.esize
        l2 = norm == "l2"
        flags = P.CKV_WO_IS_GRAM if l2 else (P.CKV_ATTN_ONLY if norm == "none" else P.CKV_WO_OUT_IN)
        self.desc = cfg_desc(cfg, flags=flags, norm=P.CKV_NORM_L2 if l2 else P.CKV_NORM_L1)
        self.B = B = cfg.budget
        multi = cfg.n_layers > 1 and n_sets == cfg.n_layers   # every layer of the model resident, each with its own W_O
        self.sets, self.host0 = [], None

        def gen(s):
            # multi-layer workloads take the inputs of different layers, single layers different seed offsets
            return make_layer(cfg, layer=s, seed_offset=0) if cfg.n_layers > 1 else make_layer(cfg, layer=0, seed_offset=s)

        # layers are generated on the host a few at a time (a batch-4 32K layer is 1 GiB of float32 K and V)
        with ThreadPoolExecutor(max_workers=max(1, min(gen_threads, n_sets))) as pool:
            for s0 in range(0, n_sets, max(1, gen_threads)):
                chunk = list(pool.map(gen, range(s0, min(n_sets, s0 + max(1, gen_threads)))))
                for j, t in enumerate(chunk):
                    if s0 + j == 0:
                        self.host0 = t
                    dev = to_device(cfg, t, True)
                    if self.sets and not multi:
                        dev["w_o"] = self.sets[0]["w_o"]  # one layer: the projection is that layer's weight, one copy
                    self.sets.append(dev)
                del chunk
        if l2:
            # the Gram matrices depend on the pretrained projection only: prepared once per layer, outside the timed steps
            prep = cfg_desc(cfg, flags=P.CKV_WO_OUT_IN, norm=P.CKV_NORM_L2)
            ws0 = torch.empty(P.workspace_bytes(prep, B), dtype=torch.uint8, device="cuda")
            grams = {}
            for dev in self.sets:
                key = dev["w_o"].data_ptr()
                if key not in grams:
                    grams[key] = torch.empty(P.gram_bytes(prep), dtype=torch.uint8, device="cuda")
                    P.criticalkv_prepare_gram(prep, dev["w_o"], grams[key], workspace=ws0)
                dev["w_o_proj"] = dev["w_o"]
                dev["w_o"] = grams[key]
            torch.cuda.synchronize()
        self.budget = torch.full((b, Hkv), B, dtype=torch.int32, device="cuda")
        self.lanes = []
        self.use_lanes = max(1, n_streams)   # lanes the steps rotate over (one more is kept for the two-stream extra)
        for _ in range(max(2, n_streams)):
            self.lanes.append(dict(
                stream=torch.cuda.Stream(),
                ws=torch.empty(P.workspace_bytes(self.desc, B), dtype=torch.uint8, device="cuda"),
                attn=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                crit=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                vnorm=torch.empty((b, H, n), dtype=torch.float32, device="cuda") if want_vnorm else None,
                idx=torch.empty((b, Hkv, B), dtype=torch.int32, device="cuda"),
                count=torch.empty((b, Hkv), dtype=torch.int32, device="cuda"),
                k_out=torch.empty((b, Hkv, B, dh), dtype=self.sets[0]["k"].dtype, device="cuda"),
                v_out=torch.empty((b, Hkv, B, dh), dtype=self.sets[0]["k"].dtype, device="cuda")))
        self.n_slots = 2 * len(P.STAGES)
        self.none_events = (ctypes.c_void_p * self.n_slots)()
        self.score_done = None  # event after the latest score: scores are chained, only the light tail overlaps
        self.vslot = 2 * P.STAGES.index("attn_stats" if norm == "none" else "vproj")
        self.vend = 2 * P.STAGES.index("attn_colsum" if norm == "none" else "vproj") + 1
        self.np = np

    # Steps are independent layers; they are issued round-robin on the lanes' streams (each with its own workspace
    # and outputs).  The score calls are chained with events (one projection kernel at a time), so what overlaps
    # is the light selection / gather tail of one layer with the scoring of the next.  All default-priority streams.
    def one_pass(self, s, stage_events=None, lane=None, with_vnorm=False):
        import torch
        P, cfg = self.P, self.cfg
        dev = self.sets[s % len(self.sets)]
        lane = self.lanes[s % self.use_lanes] if lane is None else lane
        st = lane["stream"]
        if self.use_lanes > 1 and self.score_done is not None:
            st.wait_event(self.score_done)
        P.criticalkv_score_profiled(self.desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], lane["attn"], lane["crit"],
                                    lane["vnorm"] if with_vnorm else None, workspace=lane["ws"],
                                    stage_events=self.none_events if stage_events is None else stage_events, stream=st)
        if self.use_lanes > 1:
            self.score_done = torch.cuda.Event()
            self.score_done.record(st)
        P.criticalkv_select(self.desc, lane["attn"], lane["crit"], self.budget, cfg.alpha, self.B, lane["idx"], lane["count"],
                            workspace=lane["ws"], stream=st)
        P.criticalkv_compact(self.desc, dev["k"], dev["v"], lane["idx"], lane["count"], self.B, lane["k_out"], lane["v_out"],
                             stream=st)

    def prewarm(self, ms):
        """A device that has been idle needs some tens of milliseconds under load before its clocks and power
        state settle: the first 20 passes after idle measure 7 % slower than the same passes later.  The device
        is kept busy with untimed passes for `ms` (warm-up like the W steps that follow)."""
        import torch
        steps = 0
        p0 = time.perf_counter()
        while (time.perf_counter() - p0) * 1e3 < ms:
            for w in range(8):
                self.one_pass(w)
            torch.cuda.synchronize()
            steps += 8
        return steps

    def timed(self, steps, warmup):
        """W untimed steps, then exactly `steps` steps between two synchronisations; only the dominant kernel
        carries event marks.  Returns (ms per step, the dominant kernel's average ms)."""
        import torch
        for w in range(warmup):
            self.one_pass(w)
        step_events = []
        for _ in range(steps):
            arr = (ctypes.c_void_p * self.n_slots)()
            arr[self.vslot], arr[self.vend] = self.ev.new(), self.ev.new()
            step_events.append(arr)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            self.one_pass(s, step_events[s])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = [self.ev.ms(ctypes.c_void_p(a[self.vslot]), ctypes.c_void_p(a[self.vend])) for a in step_events]
        for lane in self.lanes[:min(self.use_lanes, steps)]:
            assert int(lane["count"].min()) == self.B and int(lane["count"].max()) == self.B
        return (t1 - t0) * 1e3 / steps, max(float(self.np.mean(ms)), 1e-6)

    def sustained(self, min_ms, per_step_ms, sample_power=False):
        """A back-to-back loop of at least `min_ms`, issued like the timed steps: the rate a serving loop sees."""
        import torch
        import contextlib
        steps = max(8, int(min_ms / max(per_step_ms, 1e-3)) + 1)
        torch.cuda.synchronize()
        with (PowerSampler() if sample_power else contextlib.nullcontext()) as power:
            t0 = time.perf_counter()
            for s in range(steps):
                self.one_pass(s)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, steps, (power.summary() if sample_power else None)

    # ---- bounds ----------------------------------------------------------------------------------------
    def flops(self):
        c = self.cfg
        # L1: the d_h x d_model projection per query head.  L2: v G v^T with the d_h x d_h Gram matrix (the split of
        # G into two bf16 matrices doubles the MFMA work actually issued; the algorithmic count does not include it)
        inner = c.d_model if self.norm == "l1" else c.head_dim if self.norm == "l2" else 0
        return 2.0 * c.batch * c.n_q_heads * c.n_ctx * c.head_dim * inner

    def lower_bound_ms(self):
        """K and V read once, W_O once, the MFMA contraction, the score arrays, the gather traffic."""
        c = self.cfg
        hbm_bytes = (self.kv_bytes
                     + c.n_q_heads * c.head_dim * c.d_model * self.esize
                     + 2 * 4.0 * c.batch * c.n_kv_heads * c.n_ctx        # attn, crit written
                     + 2 * 4.0 * c.batch * c.n_kv_heads * c.n_ctx        # and read by the selection
                     + 2.0 * self.kv_bytes * self.B / c.n_ctx)           # kept rows read and written
        return (self.flops() / (PEAK_BF16_TFLOPS * 1e12) + hbm_bytes / (PEAK_HBM_GBS * 1e9)) * 1e3

    def describe(self):
        c = self.cfg
        return (f"{c.name}: batch {c.batch}, {c.n_q_heads} q / {c.n_kv_heads} kv heads, d_h {c.head_dim}, d_model {c.d_model}, "
                f"n {c.n_ctx}, W {c.window}, pool {c.pool_kernel}, budget {self.B}/head, alpha {c.alpha}, norm {self.norm}")

    def short_summary(self, ms_per_step, dom_ms):
        out = {"workload": self.describe(), "ms_per_step": round(ms_per_step, 4),
               "m_entries_per_s": round(self.cfg.entries / (ms_per_step * 1e-3) / 1e6, 2),
               "pass_lower_bound_ms": round(self.lower_bound_ms(), 4),
               "pass_frac_of_bound": round(self.lower_bound_ms() / ms_per_step, 4)}
        if self.flops():
            tf = self.flops() / (dom_ms * 1e-3) / 1e12
            out["dominant_kernel"] = {"avg_launch_ms": round(dom_ms, 4), "achieved_tflops": round(tf, 1),
                                      "frac_of_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
        return out


def run_probes(P, ev, stream):
    """What this device sustains for the two resources the pass is priced against (the library's measurement aids):
    a register-only bf16 MFMA loop in the projection kernel's launch geometry, and plain streaming reads."""
    import numpy as np
    import torch
    sh = stream.cuda_stream or None
    out = {}
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    with torch.cuda.stream(stream):
        rnd = torch.randn(1 << 19, dtype=torch.float32, device="cuda").to(torch.bfloat16)   # 1 MiB of bf16
        zero = torch.zeros(1 << 19, dtype=torch.bfloat16, device="cuda")
        for name, ops in (("random_operands", rnd), ("zero_operands", zero)):
            flop = P.criticalkv_probe_mfma_bf16(ops, 2000, sink, stream=stream)      # warm-up
            torch.cuda.synchronize()
            ts = []
            for _ in range(5):
                e0, e1 = ev.new(), ev.new()
                ev.record(e0, sh)
                flop = P.criticalkv_probe_mfma_bf16(ops, 20000, sink, stream=stream)
                ev.record(e1, sh)
                torch.cuda.synchronize()
                ts.append(ev.ms(e0, e1))
            tf = flop / (float(np.median(ts)) * 1e-3) / 1e12
            out["mfma_bf16_16x16x32_" + name] = {"tflops": round(tf, 1), "frac_of_2500": round(tf / PEAK_BF16_TFLOPS, 4),
                                                  "launch_ms": round(float(np.median(ts)), 3)}
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        other = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(5)
        isink = torch.zeros(16, dtype=torch.int32, device="cuda")
        for mib in (256, 1024):
            nbytes = mib << 20
            res = {}
            for mode in ("cold", "after_write_elsewhere", "second_read"):
                ts = []
                for _ in range(6):
                    P.criticalkv_probe_hbm_read(other, other.numel(), isink, stream=stream)   # pushes `big` out of the caches
                    if mode == "after_write_elsewhere":
                        other[:nbytes].fill_(7)
                    if mode == "second_read":
                        P.criticalkv_probe_hbm_read(big, nbytes, isink, stream=stream)
                    e0, e1 = ev.new(), ev.new()
                    ev.record(e0, sh)
                    P.criticalkv_probe_hbm_read(big, nbytes, isink, stream=stream)
                    ev.record(e1, sh)
                    torch.cuda.synchronize()
                    ts.append(ev.ms(e0, e1))
                ms = float(np.median(ts[1:]))
                res[mode] = {"ms": round(ms, 4), "tb_per_s": round(nbytes / (ms * 1e-3) / 1e12, 2)}
            out[f"hbm_read_{mib}MiB"] = res
        del big, other
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--prewarm-ms", type=float, default=200.0,
                    help="untimed passes run for this long before the warm-up steps, to bring an idle device to its "
                         "sustained clock and power state (0 = none)")
    ap.add_argument("--workload", default="llama128k",
                    help="llama128k (default, the target configuration) | llama32k | qwen128k | mistral_prefill | tiny")
    ap.add_argument("--sets", type=int, default=0, help="independent input sets rotated over the steps (0 = auto; "
                    "mistral_prefill: all 32 layers resident, each with its own projection)")
    ap.add_argument("--sustained-ms", type=float, default=500.0, help="length of the back-to-back loop behind sustained_ms_per_step")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the other workload shapes (other_workloads)")
    ap.add_argument("--lean", action="store_true",
                    help="for profiler runs: only the timed steps, the sustained loop and the stage breakdown (no other "
                         "workloads, no oracle, no two-stream loop, no graph replay), so that a kernel trace holds the "
                         "one-stream pass alone")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (cpu_baseline and parity)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0,
                    help="tokens per kv head the oracle runs on (0 = the whole layer, at most 131072)")
    ap.add_argument("--gen-threads", type=int, default=4, help="host threads generating layers")
    ap.add_argument("--budget-sweep", action="store_true",
                    help="also time select + compact for budgets 10/20/40 %% x alpha 0.25/0.5/0.75 on one set of scores "
                         "(the Qwen-shaped workload's protocol); reported beside the pass, not in the value")
    ap.add_argument("--chunked-prefill", type=int, default=0, metavar="CHUNKS",
                    help="also time a chunked prefill of the workload's context in CHUNKS chunks with eviction to the "
                         "budget after each (causal tail, kept window); reported beside the pass")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the steps are issued on round-robin (independent layers overlap); 1 = serial")
    ap.add_argument("--norm", choices=["l1", "l2", "none"], default="l1",
                    help="l1: the paper's default (dense d_model-wide projection); l2: the L2 variant via the Gram "
                         "matrix; none: attention-only baseline selection (no projected magnitude)")
    ap.add_argument("--probes", action="store_true",
                    help="also run the library's two measurement aids on this device and report them (probes): a "
                         "register-only bf16 MFMA loop on random and on zero operands, and streaming reads of 256 MiB "
                         "and 1 GiB (cold, right after a write of the same size elsewhere, and read a second time)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, to scale profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets ONE MI355X; the pass shards by kv head / batch item with no "
              "exchange, and no multi-GPU path is built. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import paper_2502_03805_amd as P
    from paper_2502_03805_amd.marshal import cfg_desc
    from workload import CONFIGS

    P.load()
    if args.lean:
        args.no_other_workloads = args.no_cpu_baseline = True
    cfg = CONFIGS[args.workload]
    b, H, Hkv, n, dh, dm = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim, cfg.d_model
    kv_bytes = 2 * b * Hkv * n * dh * (2 if cfg.dtype == "bf16" else 4)
    # a multi-layer workload keeps every layer resident (its own K, V, queries and projection); a single layer rotates
    # enough input sets that K and V of consecutive steps cannot sit in the 256 MB Infinity Cache
    nsets = args.sets or (cfg.n_layers if cfg.n_layers > 1 else max(2, min(4, int(np.ceil(512e6 / kv_bytes)))))
    ev = HipEvents(P.hip_runtime())
    with_oracle = not args.no_cpu_baseline
    wl = Workload(P, cfg, args.norm, args.streams, nsets, args.gen_threads, ev, want_vnorm=with_oracle and args.norm != "none")
    sets, lanes, desc, B = wl.sets, wl.lanes, wl.desc, wl.B
    n_streams = wl.use_lanes
    l2 = args.norm == "l2"

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    torch.cuda.synchronize()
    prewarm_steps = wl.prewarm(args.prewarm_ms)
    # ---- timed region: exactly K steps ---------------------------------------------------------------------
    ms_per_step, vproj_avg = wl.timed(args.steps, args.warmup)

    # ---- untimed extras ------------------------------------------------------------------------------------
    # the sustained rate: the same steps back to back for at least --sustained-ms on one stream, with the board's
    # power and clock sampled meanwhile
    sustained_ms, sustained_steps, power_under_load = wl.sustained(args.sustained_ms, ms_per_step, sample_power=True)
    # throughput mode: independent layers issued on two streams, so that one layer's selection and gather (latency
    # bound, nearly idle kernels) run under the next layer's projection
    two_stream_ms = None
    if n_streams == 1 and not args.lean:
        wl.use_lanes = 2
        wl.sustained(50.0, ms_per_step)
        two_stream_ms, _, _ = wl.sustained(args.sustained_ms / 2, ms_per_step)
        wl.use_lanes, wl.score_done = 1, None
        torch.cuda.synchronize()
    # a multi-layer workload: whole sweeps over all its layers in order, each timed on its own
    sweep_ms = None
    if cfg.n_layers > 1 and nsets == cfg.n_layers:
        sweep_ms = []
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(cfg.n_layers):
                wl.one_pass(s, lane=lanes[0])
            torch.cuda.synchronize()
            sweep_ms.append((time.perf_counter() - t0) * 1e3)
    lane0 = lanes[0]
    stage_ms = {name: [] for name in P.STAGES}
    stage_ms["select"], stage_ms["compact"] = [], []
    # rows beside the hot path, timed in the same untimed breakdown: adaptive budgets and the perturbation
    # diagnostics (the latter needs the magnitudes and the projection itself, so only with --norm l1)
    extras_ms = {"allocate": []}
    with_diag = args.norm == "l1"
    if with_diag:
        extras_ms["diagnostics"] = []
        diag_out = torch.empty((b, H, 8), dtype=torch.float32, device="cuda")
    alloc_budget = torch.empty((b, Hkv), dtype=torch.int32, device="cuda")
    budget = wl.budget
    stream = lane0["stream"]
    sh = stream.cuda_stream or None
    n_slots = wl.n_slots
    for s in range(min(5, max(2, args.steps))):
        dev = sets[s % nsets]
        arr = (ctypes.c_void_p * n_slots)()
        for j in range(n_slots):
            arr[j] = ev.new()
        e_sel0, e_sel1, e_cp1 = ev.new(), ev.new(), ev.new()
        P.criticalkv_score_profiled(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], lane0["attn"], lane0["crit"], None,
                                    workspace=lane0["ws"], stage_events=arr, stream=stream)
        e_al0 = ev.new()
        ev.record(e_al0, sh)
        P.criticalkv_allocate(desc, lane0["attn"], Hkv * B, 0.2, alloc_budget, workspace=lane0["ws"], stream=stream)
        ev.record(e_sel0, sh)
        P.criticalkv_select(desc, lane0["attn"], lane0["crit"], budget, cfg.alpha, B, lane0["idx"], lane0["count"],
                            workspace=lane0["ws"], stream=stream)
        ev.record(e_sel1, sh)
        P.criticalkv_compact(desc, dev["k"], dev["v"], lane0["idx"], lane0["count"], B, lane0["k_out"], lane0["v_out"],
                             stream=stream)
        ev.record(e_cp1, sh)
        if with_diag:
            e_dg1 = ev.new()
            P.criticalkv_diagnostics(desc, dev["v"], dev["w_o"], None, lane0["idx"], lane0["count"], B, diag_out,
                                     workspace=lane0["ws"], stream=stream)
            ev.record(e_dg1, sh)
        torch.cuda.synchronize()
        extras_ms["allocate"].append(ev.ms(e_al0, e_sel0))
        if with_diag:
            extras_ms["diagnostics"].append(ev.ms(e_cp1, e_dg1))
        for i, name in enumerate(P.STAGES):
            stage_ms[name].append(ev.ms(ctypes.c_void_p(arr[2 * i]), ctypes.c_void_p(arr[2 * i + 1])))
        stage_ms["select"].append(ev.ms(e_sel0, e_sel1))
        stage_ms["compact"].append(ev.ms(e_sel1, e_cp1))
    stage_min_ms = {k: round(float(np.min(v)), 4) for k, v in stage_ms.items()}
    stage_ms = {k: round(float(np.median(v)), 4) for k, v in stage_ms.items()}
    extras_ms = {k: round(float(np.median(v)), 4) for k, v in extras_ms.items()}
    # a canonical [H*d_h, d_model] projection is laid out output-major once per layer by criticalkv_prepare_wo (or on
    # every criticalkv_score call that is handed the canonical form): the cost of that step
    if args.norm == "l1":
        canon = cfg_desc(cfg, flags=0)
        w_src = sets[0]["w_o"].t().contiguous()      # [H*d_h, d_model]
        w_dst = torch.empty(P.prepared_wo_bytes(canon), dtype=torch.uint8, device="cuda")
        ts = []
        for _ in range(5):
            e0, e1 = ev.new(), ev.new()
            ev.record(e0, sh)
            P.criticalkv_prepare_wo(canon, w_src, w_dst, stream=stream)
            ev.record(e1, sh)
            torch.cuda.synchronize()
            ts.append(ev.ms(e0, e1))
        assert torch.equal(w_dst.view(sets[0]["w_o"].dtype).view(sets[0]["w_o"].shape), sets[0]["w_o"])
        extras_ms["prepare_wo_once_per_layer"] = round(float(np.median(ts)), 4)
        del w_src, w_dst
    # the same steps replayed from HIP graphs (one captured pass per input set): the launch-bound tail of small
    # kernels is issued without per-kernel host dispatch.  Untimed extra: events recorded inside a captured graph
    # carry no timing on replay, so the headline stays on the eager steps whose projection kernel is event-marked.
    graph_ms = None
    try:
        if args.lean:
            raise RuntimeError("skipped (--lean)")
        graphs = []
        with torch.cuda.stream(stream):
            for dev in sets[:4]:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    cur = torch.cuda.current_stream()
                    P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], lane0["attn"], lane0["crit"], None,
                                       workspace=lane0["ws"], stream=cur)
                    P.criticalkv_select(desc, lane0["attn"], lane0["crit"], budget, cfg.alpha, B, lane0["idx"], lane0["count"],
                                        workspace=lane0["ws"], stream=cur)
                    P.criticalkv_compact(desc, dev["k"], dev["v"], lane0["idx"], lane0["count"], B, lane0["k_out"],
                                         lane0["v_out"], stream=cur)
                graphs.append(g)
            for w in range(args.warmup):
                graphs[w % len(graphs)].replay()
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            for s in range(args.steps):
                graphs[s % len(graphs)].replay()
            torch.cuda.synchronize()
            graph_ms = round((time.perf_counter() - g0) * 1e3 / args.steps, 4)
        assert int(lane0["count"].min()) == B
        del graphs
    except RuntimeError as exc:  # capture not available: report it, the headline does not depend on it
        graph_ms = f"unavailable: {exc}"
    # Chunked prefill with eviction between chunks: the prompt arrives in chunks; after each one the cache kept so
    # far plus the chunk is scored with the chunk's last W queries (causal inside the window, the window's own
    # tokens kept), cut to the budget and compacted.  The host loop is paper_2502_03805_amd/chunked.py; the
    # chunks are slices of input set 0 and every chunk uses the set's window queries.  Untimed extra.
    if args.chunked_prefill and args.norm == "l1":
        from paper_2502_03805_amd.chunked import chunked_prefill_evict
        n_chunks = args.chunked_prefill
        clen = n // n_chunks
        dev = sets[0]
        k_chunks = [dev["k"][:, :, c * clen:(c + 1) * clen].contiguous() for c in range(n_chunks)]
        v_chunks = [dev["v"][:, :, c * clen:(c + 1) * clen].contiguous() for c in range(n_chunks)]
        q_wins = [dev["q_win"]] * n_chunks
        cflags = P.CKV_WO_OUT_IN | P.CKV_CAUSAL_TAIL | P.CKV_PROTECT_WINDOW
        mk = lambda nn: cfg_desc(cfg, flags=cflags, norm=P.CKV_NORM_L1, n_ctx=nn)
        ts = []
        for _ in range(3):
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            with torch.cuda.stream(stream):
                k_c, v_c, kept = chunked_prefill_evict(mk, q_wins, k_chunks, v_chunks, dev["w_o"], B, cfg.alpha, stream=stream)
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - c0) * 1e3)
        assert k_c.shape[2] == min(B, n)
        extras_ms["chunked_prefill"] = {"chunks": n_chunks, "chunk_tokens": clen, "budget": B,
                                        "entries_scored_per_pass": min(B, n) + clen,
                                        "passes": sum(1 for x in kept if x is not None),
                                        "total_ms_median_of_3": round(float(np.median(ts)), 4)}
        del k_chunks, v_chunks, k_c, v_c, kept
    # The paper sweeps budget and alpha on one set of scores: `score` once (timed above), then select + compact
    # for every (budget fraction, alpha) pair on the scores the last pass left in lane 0.  Untimed extra.
    if args.budget_sweep:
        from workload import budget_from_fraction
        sweep = {}
        bmax = budget_from_fraction(0.4, n)
        ws_sweep = torch.empty(P.workspace_bytes(desc, bmax), dtype=torch.uint8, device="cuda")
        idx_s = torch.empty((b, Hkv, bmax), dtype=torch.int32, device="cuda")
        cnt_s = torch.empty((b, Hkv), dtype=torch.int32, device="cuda")
        ko_s = torch.empty((b, Hkv, bmax, dh), dtype=sets[0]["k"].dtype, device="cuda")
        vo_s = torch.empty_like(ko_s)
        dev = sets[0]
        for frac in (0.1, 0.2, 0.4):
            Bs = budget_from_fraction(frac, n)
            bud_s = torch.full((b, Hkv), Bs, dtype=torch.int32, device="cuda")
            for alpha in (0.25, 0.5, 0.75):
                ts = []
                for _ in range(5):
                    e0, e1 = ev.new(), ev.new()
                    ev.record(e0, sh)
                    P.criticalkv_select(desc, lane0["attn"], lane0["crit"], bud_s, alpha, bmax, idx_s, cnt_s,
                                        workspace=ws_sweep, stream=stream)
                    P.criticalkv_compact(desc, dev["k"], dev["v"], idx_s, cnt_s, bmax, ko_s, vo_s, stream=stream)
                    ev.record(e1, sh)
                    torch.cuda.synchronize()
                    ts.append(ev.ms(e0, e1))
                assert int(cnt_s.min()) == Bs and int(cnt_s.max()) == Bs
                sweep[f"B={Bs},alpha={alpha}"] = round(float(np.median(ts)), 4)
        extras_ms["select_compact_sweep"] = sweep
        extras_ms["select_compact_sweep_total"] = round(sum(sweep.values()), 4)
        del ws_sweep, idx_s, cnt_s, ko_s, vo_s
    # workload statistic only (torch ops, outside every timed region): share of the pooled attention score held by
    # the top 1 % of a kv head's entries
    pooled = lane0["attn"].double()
    top = torch.topk(pooled, max(1, n // 100), dim=-1).values.sum(-1) / pooled.sum(-1)
    extras_ms["workload_top_1pct_attention_mass_mean_over_kv_heads"] = round(float(top.mean()), 4)
    del pooled, top
    if with_diag:
        dg = diag_out.double().cpu().numpy()
        f = {name: j for j, name in enumerate(P.DIAG_FIELDS)}
        extras_ms["diagnostics_mean_over_heads"] = {name: round(float(dg[..., j].mean()), 5) for name, j in f.items()}
        extras_ms["heads_with_sigma_above_half"] = round(float((dg[..., f["sigma"]] > 0.5).mean()), 4)

    probes = None
    if args.probes:
        probes = run_probes(P, ev, stream)

    # ---- the GPU side of the parity figures: one pass over input set 0 with the magnitudes kept ---------------
    gpu_out = None
    if with_oracle:
        wl.one_pass(0, lane=lane0, with_vnorm=args.norm != "none")
        torch.cuda.synchronize()
        gpu_out = {k: lane0[k].cpu().numpy() for k in ("attn", "crit", "idx", "count")}
        if args.norm != "none":
            gpu_out["vnorm"] = lane0["vnorm"].cpu().numpy()

    entries = cfg.entries
    value = entries / (ms_per_step * 1e-3) / 1e6
    flops = wl.flops()
    achieved = flops / (vproj_avg * 1e-3) / 1e12
    t_bound_ms = wl.lower_bound_ms()
    # every stage against its own bound, from the medians of the stage breakdown: the two attention sweeps and the
    # gather against HBM (algorithmic bytes at 8 TB/s), the projection against the bf16 MFMA peak
    esize = wl.esize
    k_bytes = kv_bytes / 2 + b * H * cfg.window * dh * esize
    stage_frac = {
        "attn_stats_hbm": round(k_bytes / (PEAK_HBM_GBS * 1e9) / (stage_ms["attn_stats"] * 1e-3), 4),
        "attn_colsum_hbm": round((k_bytes + 4.0 * b * H * n) / (PEAK_HBM_GBS * 1e9) / (stage_ms["attn_colsum"] * 1e-3), 4),
        "compact_hbm": round(2.0 * kv_bytes * B / n / (PEAK_HBM_GBS * 1e9) / (stage_ms["compact"] * 1e-3), 4),
    }
    if flops:
        stage_frac["vproj_mfma"] = round(flops / (PEAK_BF16_TFLOPS * 1e12) / (stage_ms["vproj"] * 1e-3), 4)
    if args.norm == "none":
        # two sweeps over K (stats, then window-reduced weights), each reading K and the window queries once
        sweep_bytes = 2.0 * (kv_bytes / 2 + b * H * cfg.window * dh * esize) + 2 * 4.0 * b * H * n
        gbs = sweep_bytes / (vproj_avg * 1e-3) / 1e9
        roofline = {"kernel": "attn_stats_mfma_kernel + attn_colsum_mfma_kernel", "bound": "hbm",
                    "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "traffic": None, "avg_launch_ms": round(vproj_avg, 4), "algorithmic_bytes_per_launch": sweep_bytes}
    else:
        roofline = {"kernel": "vproj_mfma_kernel" if args.norm == "l1" else "vproj_l2_resident_kernel", "bound": "mfma",
                    "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": (VPROJ_TRAFFIC_BYTES if args.norm == "l1" else L2_TRAFFIC_BYTES).get(cfg.name),
                    "avg_launch_ms": round(vproj_avg, 4), "algorithmic_flop_per_launch": flops}
    diff_pct = (sustained_ms / ms_per_step - 1.0) * 100.0
    config = {"workload": wl.describe(),
              "w_o_layout": "[d_model, H*d_h] (CKV_WO_OUT_IN)", "input_sets_rotated": nsets,
              "prewarm_ms": args.prewarm_ms, "prewarm_steps": prewarm_steps, "streams": n_streams,
              "sustained_ms_per_step": round(sustained_ms, 4), "sustained_steps": sustained_steps,
              "sustained_m_entries_per_s": round(entries / (sustained_ms * 1e-3) / 1e6, 2),
              "sustained_vs_timed_pct": round(diff_pct, 2),
              "two_stream_sustained_ms_per_step": None if two_stream_ms is None else round(two_stream_ms, 4),
              "graph_replay_ms_per_step": graph_ms,
              "tokens_per_s": round(b * n / (ms_per_step * 1e-3), 1),
              "gpu_power_state": gpu_power_state(), "board_power_under_load": power_under_load}
    if abs(diff_pct) > 3.0:
        config["note"] = (f"the {sustained_steps}-step back-to-back loop differs from the {args.steps} timed steps by "
                          f"{diff_pct:+.1f} %: take sustained_ms_per_step as the rate under continuous load")
    if cfg.n_layers > 1:
        config["layers"] = cfg.n_layers
        if sweep_ms is not None:
            # wall-clock of whole sweeps over the resident layers (each layer its own K, V, queries and projection)
            config["total_ms_all_layers"] = round(float(np.median(sweep_ms)), 3)
            config["total_ms_all_layers_each_sweep"] = [round(x, 3) for x in sweep_ms]
            config["per_layer_ms_from_sweep"] = round(float(np.median(sweep_ms)) / cfg.n_layers, 4)
            config["layers_resident"] = nsets
        else:
            config["layers_resident"] = nsets
            config["note_layers"] = "not every layer is resident (--sets): no whole-model sweep was timed"
    out = {
        "metric": "M KV entries scored+selected per second (whole score->select->compact pass, one layer)",
        "value": round(value, 2), "unit": "M KV entries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": config,
        "roofline": roofline,
        "stages_ms": stage_ms, "stages_min_ms": stage_min_ms, "stages_frac_of_own_bound": stage_frac,
        "beside_the_pass_ms": extras_ms,
        "pass_lower_bound_ms": round(t_bound_ms, 4), "pass_frac_of_bound": round(t_bound_ms / ms_per_step, 4),
    }
    if probes is not None:
        out["probes"] = probes
    host0 = wl.host0
    # free the main workload's device memory before the other shapes are made resident
    del wl, sets, lanes, lane0, budget, alloc_budget, dev
    if with_diag:
        del diag_out
    torch.cuda.empty_cache()

    # ---- the other workload shapes, timed for the same K steps each (one layer of the multi-layer workload) ----
    if not args.no_other_workloads:
        others = {}
        for name in ("llama32k", "llama128k", "qwen128k", "mistral_prefill"):
            if name == cfg.name:
                continue
            ocfg = CONFIGS[name]
            okv = 2 * ocfg.batch * ocfg.n_kv_heads * ocfg.n_ctx * ocfg.head_dim * 2
            o_sets = max(2, min(4, int(np.ceil(512e6 / okv))))
            owl = Workload(P, ocfg, args.norm, 1, o_sets, args.gen_threads, ev)
            owl.prewarm(args.prewarm_ms / 2)
            o_ms, o_dom = owl.timed(args.steps, args.warmup)
            o_sus, o_sus_steps, _ = owl.sustained(args.sustained_ms / 2, o_ms)
            rec = owl.short_summary(o_ms, o_dom)
            rec["sustained_ms_per_step"] = round(o_sus, 4)
            rec["input_sets_rotated"] = o_sets
            if ocfg.n_layers > 1:
                rec["note"] = f"one layer's shape ({o_sets} of the {ocfg.n_layers} layers rotated, one projection)"
            others[name] = rec
            del owl
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    ev.close()

    if with_oracle:
        from oracle import cpu_oracle as O
        from oracle.parity_rules import compare_selection, score_errors
        ns = min(n, args.cpu_sample_tokens or 131072)
        whole = ns == n
        Bs = B if whole else max(1, int(round(B * ns / n)))
        sample = {k: (v[:, :, :ns] if k in ("k", "v") else v) for k, v in host0.items()}
        O.lib()
        c0 = time.perf_counter()
        if args.norm == "none":
            a = O.maxpool1d(O.window_attention(sample["q_win"], sample["k"]), cfg.pool_kernel)
            at, _ = O.group_keys(a, np.zeros_like(a), Hkv, cfg.eps)
            ix, ct, tau = O.select(at, at, Bs, 1.0)
            O.compact(sample["k"], ix, ct)
            O.compact(sample["v"], ix, ct)
            ref = O.OracleResult(a, a, None, at, at, ix, ct, tau)
        else:
            ref = O.full_pass(sample["q_win"], sample["k"], sample["v"], sample["w_o"], Bs, cfg.alpha,
                              pool_kernel=cfg.pool_kernel, eps=cfg.eps, norm=2 if l2 else 1)
        c1 = time.perf_counter()
        what = "every token of every kv head" if whole else f"the first {ns} tokens of every kv head"
        out["cpu_baseline"] = {"value": round(b * Hkv * ns / (c1 - c0) / 1e6, 4), "unit": "M KV entries/s",
                               "cores": O.num_threads(), "kind": "oracle",
                               "sample": f"{what} of input set 0, whole pass (budget {Bs}/head), {c1 - c0:.1f} s wall"}
        # parity of the GPU pass over the same inputs, by the rules the tests assert (outside every timed region)
        if whole:
            par = {"against": "the float64 oracle's own pass over input set 0 (its scores, its selection)",
                   "tolerance": 2e-3, "heads": b * Hkv, "tokens_per_head": n, "max_rel_err": {}, "median_rel_err": {}}
            for name in ("attn", "crit", "vnorm"):
                if name in gpu_out:
                    mx, med = score_errors(gpu_out[name], getattr(ref, name))
                    par["max_rel_err"][name], par["median_rel_err"][name] = float(f"{mx:.3e}"), float(f"{med:.3e}")
            try:
                par["swapped_indices"] = compare_selection(gpu_out["idx"], gpu_out["count"], ref, Bs, cfg.alpha)
                par["selection"] = "identical up to the counted swaps inside the tolerance band of the oracle's thresholds"
            except AssertionError as exc:
                par["swapped_indices"] = None
                par["selection"] = f"MISMATCH outside the tolerance band: {exc}"
            out["parity"] = par
        else:
            out["parity"] = {"note": "the oracle ran on a prefix of the context only: no whole-pass comparison"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
