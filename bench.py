#!/usr/bin/env python3
"""Benchmark of the per-layer KV-cache selection pass on one MI355X.

A step is one whole pass (criticalkv_score -> criticalkv_select -> criticalkv_compact) over one
synthetic layer whose inputs are already resident in HBM.  Prints ONE JSON line:
metric = M KV entries scored+selected per second (one entry = one (batch item, kv head, token)),
with the roofline of the dominant kernel (the bf16 MFMA projection ||V W^O||_1) and the float64 CPU
oracle timed on a bounded sample of the same workload as a baseline.
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
VPROJ_TRAFFIC_BYTES = {"llama32k": int(190.0 * 2**20), "llama128k": int(607.3 * 2**20)}
# the same for the Gram-matrix kernel of the L2 variant (95.2 + 4.0 and 383.3 + 16.0 MiB)
L2_TRAFFIC_BYTES = {"llama32k": int(99.2 * 2**20), "llama128k": int(399.3 * 2**20)}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--prewarm-ms", type=float, default=200.0,
                    help="untimed passes run for this long before the warm-up steps, to bring an idle device to its "
                         "sustained clock and power state (0 = none)")
    ap.add_argument("--workload", default="llama32k", help="llama32k (default) | llama128k | qwen128k | mistral_prefill | tiny")
    ap.add_argument("--sets", type=int, default=0, help="independent input sets rotated over the steps (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=32768)
    ap.add_argument("--budget-sweep", action="store_true",
                    help="also time select + compact for budgets 10/20/40 %% x alpha 0.25/0.5/0.75 on one set of scores "
                         "(the Qwen-shaped workload's protocol); reported beside the pass, not in the value")
    ap.add_argument("--chunked-prefill", type=int, default=0, metavar="CHUNKS",
                    help="also time a chunked prefill of the workload's context in CHUNKS chunks with eviction to the "
                         "budget after each (causal tail, protected window); reported beside the pass")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the steps are issued on round-robin (independent layers overlap); 1 = serial")
    ap.add_argument("--norm", choices=["l1", "l2", "none"], default="l1",
                    help="l1: the paper's default (dense d_model-wide projection); l2: the L2 variant via the Gram "
                         "matrix; none: attention-only baseline selection (no projected magnitude)")
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
    from paper_2502_03805_amd.marshal import cfg_desc, to_device
    from workload import CONFIGS, make_layer

    P.load()
    cfg = CONFIGS[args.workload]
    b, H, Hkv, n, dh, dm = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim, cfg.d_model
    esize = 2 if cfg.dtype == "bf16" else 4
    kv_bytes = 2 * b * Hkv * n * dh * esize
    # rotate enough input sets that K and V of consecutive steps cannot sit in the 256 MB Infinity Cache
    nsets = args.sets or max(2, min(4, int(np.ceil(512e6 / kv_bytes))))
    l2 = args.norm == "l2"
    flags = P.CKV_WO_IS_GRAM if l2 else (P.CKV_ATTN_ONLY if args.norm == "none" else P.CKV_WO_OUT_IN)
    desc = cfg_desc(cfg, flags=flags, norm=P.CKV_NORM_L2 if l2 else P.CKV_NORM_L1)
    B = cfg.budget
    sets = []
    host0 = None
    for s in range(nsets):
        # multi-layer workloads rotate the inputs of different layers, single layers rotate seed offsets
        t = make_layer(cfg, layer=s, seed_offset=0) if cfg.n_layers > 1 else make_layer(cfg, layer=0, seed_offset=s)
        if s == 0:
            host0 = t
        dev = to_device(cfg, t, True)
        if s > 0:
            dev["w_o"] = sets[0]["w_o"]  # the projection is a weight: one copy
        sets.append(dev)
    if l2:
        # the Gram matrices depend on the pretrained projection only: prepared once, outside the timed steps
        prep = cfg_desc(cfg, flags=P.CKV_WO_OUT_IN, norm=P.CKV_NORM_L2)
        gram = torch.empty(P.gram_bytes(prep), dtype=torch.uint8, device="cuda")
        ws0 = torch.empty(P.workspace_bytes(prep, B), dtype=torch.uint8, device="cuda")
        P.criticalkv_prepare_gram(prep, sets[0]["w_o"], gram, workspace=ws0)
        torch.cuda.synchronize()
        for dev in sets:
            dev["w_o"] = gram
    budget = torch.full((b, Hkv), B, dtype=torch.int32, device="cuda")
    # Steps are independent layers; they are issued round-robin on `--streams` streams (each with its own
    # workspace and outputs).  The score calls are chained with events (one projection kernel at a time),
    # so what overlaps is the light selection / gather tail of one layer with the scoring of the next.
    # All default-priority streams.
    n_streams = max(1, args.streams)
    lanes = []
    for _ in range(n_streams):
        lanes.append(dict(
            stream=torch.cuda.Stream(),
            ws=torch.empty(P.workspace_bytes(desc, B), dtype=torch.uint8, device="cuda"),
            attn=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
            crit=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
            idx=torch.empty((b, Hkv, B), dtype=torch.int32, device="cuda"),
            count=torch.empty((b, Hkv), dtype=torch.int32, device="cuda"),
            k_out=torch.empty((b, Hkv, B, dh), dtype=sets[0]["k"].dtype, device="cuda"),
            v_out=torch.empty((b, Hkv, B, dh), dtype=sets[0]["k"].dtype, device="cuda")))
    ev = HipEvents(P.hip_runtime())
    n_slots = 2 * len(P.STAGES)

    score_done = [None]  # event after the latest score: scores are chained, only the light tail overlaps

    def one_pass(dev, lane, stage_events):
        st = lane["stream"]
        if n_streams > 1 and score_done[0] is not None:
            st.wait_event(score_done[0])
        P.criticalkv_score_profiled(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], lane["attn"], lane["crit"], None,
                                    workspace=lane["ws"], stage_events=stage_events, stream=st)
        if n_streams > 1:
            score_done[0] = torch.cuda.Event()
            score_done[0].record(st)
        P.criticalkv_select(desc, lane["attn"], lane["crit"], budget, cfg.alpha, B, lane["idx"], lane["count"],
                            workspace=lane["ws"], stream=st)
        P.criticalkv_compact(desc, dev["k"], dev["v"], lane["idx"], lane["count"], B, lane["k_out"], lane["v_out"], stream=st)

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    none_events = (ctypes.c_void_p * n_slots)()
    torch.cuda.synchronize()
    # A device that has been idle needs some tens of milliseconds under load before its clocks and power state
    # settle: the first 20 passes after idle measure 7 % slower than the same passes later.  So the device is
    # first kept busy with untimed passes for --prewarm-ms (they are warm-up like the W steps that follow); the
    # timed region is the sustained rate, which is what a serving loop sees.
    prewarm_steps = 0
    p0 = time.perf_counter()
    while (time.perf_counter() - p0) * 1e3 < args.prewarm_ms:
        for w in range(8):
            one_pass(sets[w % nsets], lanes[w % n_streams], none_events)
        torch.cuda.synchronize()
        prewarm_steps += 8
    for w in range(args.warmup):
        one_pass(sets[w % nsets], lanes[w % n_streams], none_events)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; only the dominant kernel carries event marks --------------------
    # (the attention-only pass has no projection: there the two key sweeps are the dominant kernels)
    vslot = 2 * P.STAGES.index("attn_stats" if args.norm == "none" else "vproj")
    vend = 2 * P.STAGES.index("attn_colsum" if args.norm == "none" else "vproj") + 1
    step_events = []
    for _ in range(args.steps):
        arr = (ctypes.c_void_p * n_slots)()
        arr[vslot], arr[vend] = ev.new(), ev.new()
        step_events.append(arr)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_pass(sets[s % nsets], lanes[s % n_streams], step_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    vproj_ms = [ev.ms(ctypes.c_void_p(a[vslot]), ctypes.c_void_p(a[vend])) for a in step_events]
    vproj_avg = max(float(np.mean(vproj_ms)), 1e-6)
    for lane in lanes[:min(n_streams, args.steps)]:
        assert int(lane["count"].min()) == B and int(lane["count"].max()) == B

    # ---- untimed extras: the same K steps on one stream, and a per-stage breakdown -----------------------
    lane0 = lanes[0]
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for s in range(args.steps):
        one_pass(sets[s % nsets], lane0, none_events)
    torch.cuda.synchronize()
    serial_ms_per_step = (time.perf_counter() - s0) * 1e3 / args.steps
    # board power under the same back-to-back loop, kept up for about 0.4 s (untimed extra)
    power_steps = max(args.steps, int(400.0 / max(serial_ms_per_step, 1e-3)))
    with PowerSampler() as power:
        for s in range(power_steps):
            one_pass(sets[s % nsets], lane0, none_events)
        torch.cuda.synchronize()
    power_under_load = power.summary()
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
    stream = lane0["stream"]
    sh = stream.cuda_stream or None
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
    # the same steps replayed from HIP graphs (one captured pass per input set): the launch-bound tail of small
    # kernels is issued without per-kernel host dispatch.  Untimed extra: events recorded inside a captured graph
    # carry no timing on replay, so the headline stays on the eager steps whose projection kernel is event-marked.
    graph_ms = None
    try:
        graphs = []
        with torch.cuda.stream(stream):
            for dev in sets:
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
                graphs[w % nsets].replay()
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            for s in range(args.steps):
                graphs[s % nsets].replay()
            torch.cuda.synchronize()
            graph_ms = round((time.perf_counter() - g0) * 1e3 / args.steps, 4)
        assert int(lane0["count"].min()) == B
        del graphs
    except RuntimeError as exc:  # capture not available: report it, the headline does not depend on it
        graph_ms = f"unavailable: {exc}"
    extras_ms = {k: round(float(np.median(v)), 4) for k, v in extras_ms.items()}
    # Chunked prefill with eviction between chunks: the prompt arrives in chunks; after each one the cache kept so
    # far plus the chunk is scored with the chunk's last W queries (causal inside the window, the window's own
    # tokens protected), cut to the budget and compacted.  The host loop is paper_2502_03805_amd/chunked.py; the
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
    if with_diag:
        dg = diag_out.double().cpu().numpy()
        f = {name: j for j, name in enumerate(P.DIAG_FIELDS)}
        extras_ms["diagnostics_mean_over_heads"] = {name: round(float(dg[..., j].mean()), 5) for name, j in f.items()}
        extras_ms["heads_with_sigma_above_half"] = round(float((dg[..., f["sigma"]] > 0.5).mean()), 4)
    ev.close()

    entries = cfg.entries
    value = entries / (ms_per_step * 1e-3) / 1e6
    # L1: the d_h x d_model projection per query head.  L2: v G v^T with the d_h x d_h Gram matrix (the split of
    # G into two bf16 matrices doubles the MFMA work actually issued; the algorithmic count does not include it)
    flops = 2.0 * b * H * n * dh * (dm if args.norm == "l1" else dh if l2 else 0)
    achieved = flops / (vproj_avg * 1e-3) / 1e12
    # lower bound of the whole pass: K and V read once, W_O once, the MFMA contraction, the gather traffic
    hbm_bytes = (kv_bytes                      # K and V read once
                 + H * dh * dm * esize           # W_O read once
                 + 2 * 4.0 * b * Hkv * n         # attn, crit written
                 + 2 * 4.0 * b * Hkv * n         # and read by the selection
                 + 2.0 * kv_bytes * B / n)       # kept rows read and written
    t_bound_ms = (flops / (PEAK_BF16_TFLOPS * 1e12) + hbm_bytes / (PEAK_HBM_GBS * 1e9)) * 1e3
    # every stage against its own bound, from the medians of the stage breakdown: the two attention sweeps and the
    # gather against HBM (algorithmic bytes at 8 TB/s), the projection against the bf16 MFMA peak
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
        roofline = {"kernel": "attn_stats_mfma_kernel + attn_stats_reduce_log2_kernel + attn_colsum_mfma_kernel", "bound": "hbm",
                    "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "traffic": None, "avg_launch_ms": round(vproj_avg, 4), "algorithmic_bytes_per_launch": sweep_bytes}
    else:
        roofline = {"kernel": "vproj_mfma_kernel" if args.norm == "l1" else "vproj_l2_mfma_kernel", "bound": "mfma",
                    "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": (VPROJ_TRAFFIC_BYTES if args.norm == "l1" else L2_TRAFFIC_BYTES).get(cfg.name),
                    "avg_launch_ms": round(vproj_avg, 4), "algorithmic_flop_per_launch": flops}
    out = {
        "metric": "M KV entries scored+selected per second (whole score->select->compact pass, one layer)",
        "value": round(value, 2), "unit": "M KV entries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: batch {b}, {H} q / {Hkv} kv heads, d_h {dh}, d_model {dm}, n {n}, "
                               f"W {cfg.window}, pool {cfg.pool_kernel}, budget {B}/head, alpha {cfg.alpha}, norm {args.norm}",
                   "w_o_layout": "[d_model, H*d_h] (CKV_WO_OUT_IN)", "input_sets_rotated": nsets,
                   "prewarm_ms": args.prewarm_ms, "prewarm_steps": prewarm_steps,
                   "streams": n_streams, "serial_ms_per_step": round(serial_ms_per_step, 4),
                   "graph_replay_ms_per_step": graph_ms,
                   "tokens_per_s": round(b * n / (ms_per_step * 1e-3), 1),
                   "gpu_power_state": gpu_power_state(), "board_power_under_load": power_under_load,
                   **({"layers": cfg.n_layers, "total_ms_all_layers": round(cfg.n_layers * ms_per_step, 3)}
                      if cfg.n_layers > 1 else {})},
        "roofline": roofline,
        "stages_ms": stage_ms, "stages_min_ms": stage_min_ms, "stages_frac_of_own_bound": stage_frac,
        "beside_the_pass_ms": extras_ms,
        "pass_lower_bound_ms": round(t_bound_ms, 4), "pass_frac_of_bound": round(t_bound_ms / ms_per_step, 4),
    }

    if not args.no_cpu_baseline:
        from oracle import cpu_oracle as O
        ns = min(n, args.cpu_sample_tokens)
        Bs = max(1, int(round(B * ns / n)))
        sample = {k: (v[:, :, :ns] if k in ("k", "v") else v) for k, v in host0.items()}
        O.lib()
        c0 = time.perf_counter()
        if args.norm == "none":
            a = O.maxpool1d(O.window_attention(sample["q_win"], sample["k"]), cfg.pool_kernel)
            at, _ = O.group_keys(a, np.zeros_like(a), Hkv, cfg.eps)
            ix, ct, _ = O.select(at, at, Bs, 1.0)
            O.compact(sample["k"], ix, ct)
            O.compact(sample["v"], ix, ct)
        else:
            O.full_pass(sample["q_win"], sample["k"], sample["v"], sample["w_o"], Bs, cfg.alpha,
                        pool_kernel=cfg.pool_kernel, eps=cfg.eps, norm=2 if l2 else 1)
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": round(b * Hkv * ns / (c1 - c0) / 1e6, 4), "unit": "M KV entries/s",
                               "cores": O.num_threads(), "kind": "oracle",
                               "sample": f"first {ns} tokens of every kv head of input set 0, whole pass "
                                         f"(budget {Bs}/head), {c1 - c0:.1f} s wall"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
