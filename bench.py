#!/usr/bin/env python3
"""Benchmark of the QuantSpec decode-attention hot path on one MI355X.

One "step" is one speculation cycle of Algorithm 1, every stage of the hot path included: gamma = 4
draft attention calls (1 query, upper plane + buffer), one verify call (gamma + 1 = 5 causal queries,
both planes + buffer) and one quantize-on-flush of buffered tokens (quantize, append, buffer move),
each issued once per layer (one layer, except for the 32-layer stack workload).  Inputs are resident
in HBM before the timed region.  Single-layer workloads rotate over several independent cache copies
so the 256 MB last-level cache cannot serve the planes; the stack's 32 layer caches are distinct
allocations anyway.

The headline keys of the JSON line are those of the 128k-context multi-head workload (`mha128k`); the
`workloads` object carries the same figures for every workload of the baseline description, the stack
as a whole-stack step.  Every workload is timed three ways: eager calls through the C ABI (the headline),
the same cycle captured in a HIP graph and replayed, and eager with bit-reproducible dealing
(QS_FLAG_FIXED_RANGES).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import glob
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
GAMMA = 4
SPEC_GAMMAS = (1, 2, 4, 6)      # speculation lengths of the simulated decode loop (Table 6)
ALL_WORKLOADS = ("mha128k", "tiny", "mha32k", "gqa128k_b4", "stack64k_b8")
# tokens flushed per cycle: the baseline description names 256 for the tiny and the stack workload;
# the others take the paper's cadence (G = 128 tokens once 2G are buffered, Section 4.3.2)
FLUSH_TOKENS = {"tiny": 256, "stack64k_b8": 256}
PRECONDITION_S = 1.0            # untimed run of the cycle before the warm-up steps (see precondition())

# HBM traffic per launch of the attention kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (calibrated against a plain copy kernel: FETCH_SIZE x 1.99991, WRITE_SIZE x 1.0, KiB per dispatch).
# Filled from profiles/attn_hbm_traffic.md; a workload without an entry reports null.
MEASURED_TRAFFIC_BYTES = {
    ("mha128k", "draft"): int((281027.7 * 1.99991 + 585.0) * 1024),
    ("mha128k", "verify"): int((543496.3 * 1.99991 + 2926.0) * 1024),
    ("gqa128k_b4", "draft"): int((288478.6 * 1.99991 + 4420.7) * 1024),
    ("gqa128k_b4", "verify"): int((544773.0 * 1.99991 + 11701.5) * 1024),
}


class PowerSampler:
    """Board power (hwmon, microwatts) read every 20 ms while a timed region runs: the long-context
    kernels sit at the board's power limit, which is what bounds them (see precondition())."""

    def __init__(self):
        hits = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                      glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))
        self.path = hits[0] if hits else None
        self.samples = []

    def __enter__(self):
        self.samples, self._stop = [], False
        if self.path:
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def _run(self):
        while not self._stop:
            try:
                with open(self.path) as f:
                    self.samples.append(int(f.read()) / 1e6)
            except (OSError, ValueError):
                pass
            time.sleep(0.02)

    def __exit__(self, *exc):
        self._stop = True
        if self.path:
            self._thread.join()

    def summary(self):
        if not self.samples:
            return None
        return {"mean": round(float(np.mean(self.samples)), 1), "max": round(float(np.max(self.samples)), 1),
                "samples": len(self.samples)}


def algorithmic_bytes(w, nq, verify):
    """Bytes one attention call on one layer must move (fp16 metadata): per quantized token and unit
    64 (K upper) + 64 (V upper) + 4 (K scale/zero, amortised over the group) + 4 (V scale/zero); twice
    the plane bytes for verify; plus the fp16 buffer and q / out."""
    per_tok = (128 + 128 + 8) if verify else (64 + 64 + 8)
    return w.units * (w.n_quant * per_tok + w.n_buf * 128 * 2 * 2) + w.batch * w.n_q_heads * nq * 128 * 2 * 2


def flush_bytes(w, n):
    return w.units * n * (128 * 2 * 2 + (128 + 128 + 4 + 4))


class Bench:
    """One workload resident on the GPU: `groups` is the list of cache groups a cycle may run on - one
    cache per group for a single-layer workload (the cycle rotates over the groups), all 32 layer caches
    in one group for the stack."""

    def __init__(self, torch, B, synth, w, copies, keep_fp16=False):
        self.torch, self.B, self.w = torch, B, w
        self.sm_scale = 1.0 / float(np.sqrt(w.head_dim))
        self.n_flush = FLUSH_TOKENS.get(w.name, 128)
        dev = "cuda"
        t0 = time.time()
        self.k_host, self.v_host = synth.gen_layer_kv(w, workers=min(16, os.cpu_count() or 8))
        self.q_draft = torch.from_numpy(synth.gen_layer_q(w, 1)).to(dev)
        self.q_verify = torch.from_numpy(synth.gen_layer_q(w, w.nq_verify)).to(dev)
        kd, vd = torch.from_numpy(self.k_host).to(dev), torch.from_numpy(self.v_host).to(dev)
        n_caches = w.n_layers if w.n_layers > 1 else copies
        q_cap = w.n_quant + 640            # room for the groups flushed during the run
        caches = []
        self.prefill = None
        for i in range(n_caches):
            c = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, q_cap, w.n_buf + 8)
            if i == 0:
                B.qs_quantize_prefill(c, kd, vd, w.n_quant)
                if keep_fp16:
                    self.prefill = time_prefill(torch, B, c, kd, vd, w)
            else:      # further copies / layers: the same codes in memory of their own
                for name in B.PLANES:
                    getattr(c, name).copy_(getattr(caches[0], name))
            c.k_buf[:, :, :w.n_buf] = kd[:, :, w.n_quant:]
            c.v_buf[:, :, :w.n_buf] = vd[:, :, w.n_quant:]
            c.n_quant[:] = w.n_quant
            c.n_buf[:] = w.n_buf
            caches.append(c)
        self.caches = caches
        self.groups = [caches] if w.n_layers > 1 else [[c] for c in caches]
        self.fp16 = (kd, vd) if keep_fp16 else None
        del kd, vd
        self.ws = torch.empty(max(B.qs_workspace_bytes(caches[0], n) for n in (1, w.nq_verify, max(SPEC_GAMMAS) + 1)),
                              dtype=torch.uint8, device=dev)
        self.out_d = torch.empty_like(self.q_draft)
        self.out_v = torch.empty_like(self.q_verify)
        self.set_flags(0)
        torch.cuda.synchronize()
        self.setup_s = time.time() - t0

    def set_flags(self, flags):
        for c in self.caches:
            c.flags = flags
        # descriptors are built once per setting: the host lengths do not move during the timed cycles
        self.structs = [[c.struct() for c in g] for g in self.groups]

    def cycle(self, i, events=None):
        """One speculation cycle on cache group i: per layer gamma draft calls, then per layer the verify
        call, then per layer the flush (host lengths stay put: the same group slots are rewritten each
        cycle).  events: four HIP events to record around the three phases."""
        B, s = self.B, self.structs[i % len(self.structs)]
        if events:
            events[0].record()
        for _ in range(GAMMA):
            for c in s:
                B.qs_attn_draft(c, self.q_draft, self.sm_scale, out=self.out_d, workspace=self.ws)
        if events:
            events[1].record()
        for c in s:
            B.qs_attn_verify(c, self.q_verify, self.sm_scale, out=self.out_v, workspace=self.ws)
        if events:
            events[2].record()
        for c in s:
            B.qs_quantize_flush(c, self.n_flush)
        if events:
            events[3].record()

    def precondition(self, seconds):
        """Runs the cycle untimed for `seconds`.  The chip's power management needs about half a second
        of a steady load to settle: the first ~20 ms of a 128k-context loop run at boost clocks (the
        20-row verify call: 176 us), the next few hundred ms below the steady state (up to 275 us), then
        it stays put (184 us) at the 1400 W board limit.  Figures taken inside that transient depend on
        what ran before; the steady state is what a decoder lives in."""
        torch = self.torch
        t0, i = time.perf_counter(), 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(4):
                self.cycle(i)
                i += 1
            torch.cuda.synchronize()
        return i

    def run_eager(self, steps, warmup):
        """`warmup` untimed cycles, then exactly `steps` timed ones.  Returns seconds per cycle (host clock
        around the timed cycles, synchronized on both sides) and per-call microseconds of each phase
        from HIP events on the launch stream."""
        torch = self.torch
        layers = len(self.groups[0])
        for i in range(warmup):
            self.cycle(i)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        gc.collect()
        gc.disable()                      # no collector pause inside the timed region
        t_start = time.perf_counter()
        for i in range(steps):
            self.cycle(warmup + i, ev[i])
            if i >= 2:
                # stay at most two cycles ahead of the GPU (a decoder reads each cycle's outcome anyway);
                # letting the host queue hundreds of launches ahead has stalled the runtime for tens of ms
                ev[i - 2][3].synchronize()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        gc.enable()
        calls = {"draft": GAMMA * layers, "verify": layers, "flush": layers}
        per_call = {k: np.array([1e3 * e[j].elapsed_time(e[j + 1]) / calls[k] for e in ev])
                    for j, k in enumerate(("draft", "verify", "flush"))}
        return elapsed / steps, per_call

    def run_graph(self, steps, warmup):
        """The same cycles captured once into a HIP graph (one cycle per cache group) and replayed: no
        host work between the launches.  Returns seconds per cycle."""
        torch = self.torch
        n = len(self.groups)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):     # the library's first launches on the capture stream happen before capture
            self.cycle(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(n):
                self.cycle(i)
        replays, warm = max(1, -(-steps // n)), max(1, -(-warmup // n))
        for _ in range(warm):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / (replays * n)
        del graph
        return dt

    def time_flush(self, n_tokens, reps=40):
        """A flush of n_tokens on one layer, alone: microseconds per call (HIP events around `reps` calls)."""
        torch, B = self.torch, self.B
        s = [g[0] for g in self.structs]
        for i in range(4):
            B.qs_quantize_flush(s[i % len(s)], n_tokens)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            B.qs_quantize_flush(s[i % len(s)], n_tokens)
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / reps


def pick_counts(cycle_s, timed_s=0.6, warm_s=0.2, lo=20, hi=4000):
    """Timed and warm-up cycle counts for a workload whose cycle takes cycle_s seconds."""
    steps = int(min(hi, max(lo, timed_s / cycle_s)))
    return steps, int(min(hi, max(5, warm_s / cycle_s)))


def measure(bench, steps=None, warmup=None, graph=True, fixed=True, precondition_s=PRECONDITION_S):
    """All figures of one workload.  steps / warmup: given for the headline workload, chosen from the
    cycle time otherwise."""
    w, layers = bench.w, len(bench.groups[0])
    n_pre = bench.precondition(precondition_s) if precondition_s > 0 else 0
    if steps is None:
        est, _ = bench.run_eager(8, 2)
        steps, warmup = pick_counts(est)
    with PowerSampler() as power:
        cyc_s, per_call = bench.run_eager(steps, warmup)
    avg = {k: float(v.mean()) for k, v in per_call.items()}
    bytes_d, bytes_v = algorithmic_bytes(w, 1, False), algorithmic_bytes(w, w.nq_verify, True)
    cycle_bytes = layers * (GAMMA * bytes_d + bytes_v + flush_bytes(w, bench.n_flush))
    gb = lambda nbytes, us: nbytes / (us * 1e-6) / 1e9
    res = {
        "workload": f"{w.name}: {w.n_layers} layer(s) x batch {w.batch}, {w.n_q_heads} q-heads / {w.n_kv_heads} kv-heads x 128, "
                    f"ctx {w.ctx} = {w.n_quant} quantized + {w.n_buf} fp16 buffer, G=128, gamma=4",
        "layers": layers, "steps": steps, "warmup": warmup, "precondition_cycles": n_pre,
        "flush_tokens_per_cycle": bench.n_flush,
        "us_per_decode_step": round(cyc_s * 1e6 / (GAMMA + 1), 3),
        "ms_per_cycle": round(cyc_s * 1e3, 5),
        "cycle_GBps": round(cycle_bytes / cyc_s / 1e9, 1),
        "cycle_bytes": cycle_bytes,
        "draft_us": round(avg["draft"], 2), "verify_us": round(avg["verify"], 2), "flush_us": round(avg["flush"], 2),
        "median_us": {k: round(float(np.median(v)), 2) for k, v in per_call.items()},
        "min_us": {k: round(float(v.min()), 2) for k, v in per_call.items()},
        "draft_GBps": round(gb(bytes_d, avg["draft"]), 1), "verify_GBps": round(gb(bytes_v, avg["verify"]), 1),
        "draft_frac": round(gb(bytes_d, avg["draft"]) / HBM_PEAK_GBPS, 4),
        "verify_frac": round(gb(bytes_v, avg["verify"]) / HBM_PEAK_GBPS, 4),
        "draft_bytes": bytes_d, "verify_bytes": bytes_v,
        "flush128_us": round(bench.time_flush(128), 2), "flush256_us": round(bench.time_flush(256), 2),
        "board_power_W": power.summary(),
        "traffic": {k: MEASURED_TRAFFIC_BYTES.get((w.name, k)) for k in ("draft", "verify")},
    }
    if layers > 1:
        res["whole_stack"] = {
            "draft_pass_us": round(avg["draft"] * layers, 1), "verify_pass_us": round(avg["verify"] * layers, 1),
            "flush_pass_us": round(avg["flush"] * layers, 1),
            "us_per_decode_step": res["us_per_decode_step"], "GBps": res["cycle_GBps"],
            "bytes_per_cycle": cycle_bytes, "resident_plane_bytes": sum(c.plane_bytes() for c in bench.caches)}
    if graph:
        g_s = bench.run_graph(steps, warmup)
        res["graph"] = {"us_per_decode_step": round(g_s * 1e6 / (GAMMA + 1), 3), "ms_per_cycle": round(g_s * 1e3, 5),
                        "cycle_GBps": round(cycle_bytes / g_s / 1e9, 1)}
    if fixed:
        bench.set_flags(bench.B.QS_FLAG_FIXED_RANGES)
        f_s, f_call = bench.run_eager(max(20, steps // 2), max(5, warmup // 2))
        bench.set_flags(0)
        res["fixed_ranges"] = {"us_per_decode_step": round(f_s * 1e6 / (GAMMA + 1), 3),
                               "draft_us": round(float(f_call["draft"].mean()), 2),
                               "verify_us": round(float(f_call["verify"].mean()), 2)}
    return res, avg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000, help="timed cycles of the headline workload")
    ap.add_argument("--warmup", type=int, default=200, help="untimed cycles of the headline workload before them")
    ap.add_argument("--workload", default="all",
                    help="'all' (headline mha128k, then the other baseline workloads), one workload's name, 'other_shapes' "
                         "(only the call times of the other (head_dim, group) shapes, for kernel traces) or 'w4_linear' (only the "
                         "draft model's 4-bit-weight linear layers)")
    ap.add_argument("--copies", type=int, default=4, help="independent cache copies a single-layer workload rotates over")
    ap.add_argument("--precondition", type=float, default=PRECONDITION_S,
                    help="seconds of the cycle run untimed before the warm-up steps (0 for counter collection runs)")
    ap.add_argument("--trace-transient", choices=("cycle", "draft", "verify"), default=None,
                    help="instead of the benchmark: start the chosen workload's cycle (or its draft / verify call alone, "
                         "back to back) on an idle chip and print, as one JSON line, the call times and the board power "
                         "over the first seconds")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the eager timed cycle of the chosen workload(s): no graph / fixed-range timing, prefill, "
                         "fp16 baseline or speculation loop (for kernel traces)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; every figure is the one GPU's throughput. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_10424_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()
    if args.workload == "other_shapes":
        # --steps below 100: a few launches per kernel only (counter collection)
        print(json.dumps({"other_shapes": other_shapes(torch, B, seconds=0.25 if args.steps >= 100 else 0.002)}), flush=True)
        return
    if args.workload == "w4_linear":
        print(json.dumps({"w4_linear": w4_linear(torch, B, seconds=0.25 if args.steps >= 100 else 0.002)}), flush=True)
        return
    names = ALL_WORKLOADS if args.workload == "all" else (args.workload,)
    if args.trace_transient:
        print(json.dumps(trace_transient(torch, B, synth, synth.WORKLOADS[names[0]], args.copies, args.trace_transient)), flush=True)
        return
    extras = not args.no_extras
    t_all = time.time()

    # ---- headline workload ------------------------------------------------------------------------
    w = synth.WORKLOADS[names[0]]
    bench = Bench(torch, B, synth, w, args.copies, keep_fp16=extras and w.n_layers == 1)
    head, avg = measure(bench, args.steps, args.warmup, graph=extras, fixed=extras, precondition_s=args.precondition)
    kern = {"draft": "attn_kernel<1,8,false,true>" if w.n_q_heads == w.n_kv_heads else "attn_kernel_cu",
            "verify": "attn_kernel<1,8,true>" if w.nq_verify * w.n_q_heads // w.n_kv_heads <= 8 else "attn_kernel<2,8,true>"}
    roof = lambda what, plane: {
        "bound": "hbm", "kernel": f"{what} call: {kern[what]} + merge_kernel ({plane})",
        "achieved": head[f"{what}_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": head[f"{what}_frac"],
        "algorithmic_bytes_per_launch": head[f"{what}_bytes"],
        "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, what))}
    result = {
        "metric": "draft/verify attention us per decode step + achieved HBM GB/s at 128k ctx",
        "value": head["us_per_decode_step"],
        "unit": "us/decode-step (mean over a cycle of 4 draft + 1 verify call per layer, flush included)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_cycle"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": head["workload"], "cache_copies_rotated": len(bench.groups),
                   "flush_tokens_per_cycle": bench.n_flush, "fixed_ranges": False,
                   "precondition_s": args.precondition},
        "draft_us": head["draft_us"], "verify_us": head["verify_us"], "flush_us": head["flush_us"],
        "median_us": head["median_us"], "min_us": head["min_us"],
        "draft_GBps": head["draft_GBps"], "verify_GBps": head["verify_GBps"], "cycle_GBps": head["cycle_GBps"],
        "roofline": roof("draft", "upper plane"),
        "roofline_verify": roof("verify", "both planes"),
        "setup_s": round(bench.setup_s, 1),
    }
    if "graph" in head:
        result["graph"] = head["graph"]
    if "fixed_ranges" in head:
        result["fixed_ranges"] = head["fixed_ranges"]
    if extras and bench.fp16 is not None:
        kd, vd = bench.fp16
        fp16_cache = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, 0, w.ctx)
        fp16_cache.k_buf, fp16_cache.v_buf = kd, vd
        fp16_cache.n_buf[:] = w.ctx
        result["prefill_quantize"] = bench.prefill
        result["fp16_baseline"] = fp16_baseline(torch, B, fp16_cache, w, bench.sm_scale, bench.q_draft, bench.q_verify,
                                                avg["draft"], avg["verify"])
        result["speculation"] = speculation_loop(torch, B, bench.caches[0], w, bench.sm_scale, bench.ws)
        result["paged_cache"] = paged_cache(torch, B, w, kd, vd, bench.sm_scale, bench.q_draft, bench.q_verify)
        del fp16_cache, kd, vd
    k_host, v_host, sm_scale = bench.k_host, bench.v_host, bench.sm_scale
    workloads = {w.name: head}
    del bench
    torch.cuda.empty_cache()

    # ---- the other workloads ------------------------------------------------------------------------
    for name in names[1:]:
        b = Bench(torch, B, synth, synth.WORKLOADS[name], args.copies)
        workloads[name], _ = measure(b, graph=extras, fixed=extras, precondition_s=args.precondition)
        workloads[name]["setup_s"] = round(b.setup_s, 1)
        del b
        gc.collect()
        torch.cuda.empty_cache()
    result["workloads"] = workloads
    if extras and args.workload == "all":
        result["other_shapes"] = other_shapes(torch, B)
        result["w4_linear"] = w4_linear(torch, B)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, k_host, v_host, sm_scale)
    result["wall_s"] = round(time.time() - t_all, 1)
    print(json.dumps(result), flush=True)


def trace_transient(torch, B, synth, w, copies, what, seconds=3.0, idle_s=3.0):
    """How the call times and the board power move when work starts on an idle chip.  what = "cycle":
    batches of four cycles, each batch's mean draft and verify call time (HIP events) next to the power
    read after it; "draft" / "verify": that call alone, back to back, in batches of twenty."""
    bench = Bench(torch, B, synth, w, copies)
    bench.run_eager(4, 2)                 # first launches (code objects, descriptors) are not part of the trace
    time.sleep(idle_s)
    power = PowerSampler()
    layers = len(bench.groups[0])
    rows, i, t0 = [], 0, time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        if what == "cycle":
            ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(4)]
            for e in ev:
                bench.cycle(i, e)
                i += 1
            torch.cuda.synchronize()
            times = [float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e3 / (GAMMA * layers),
                     float(np.mean([e[1].elapsed_time(e[2]) for e in ev])) * 1e3 / layers]
        else:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                for c in bench.structs[i % len(bench.structs)]:
                    if what == "draft":
                        B.qs_attn_draft(c, bench.q_draft, bench.sm_scale, out=bench.out_d, workspace=bench.ws)
                    else:
                        B.qs_attn_verify(c, bench.q_verify, bench.sm_scale, out=bench.out_v, workspace=bench.ws)
                i += 1
            e1.record()
            torch.cuda.synchronize()
            times = [e0.elapsed_time(e1) * 1e3 / (20 * layers)]
        watts = None
        if power.path:
            with open(power.path) as f:
                watts = round(int(f.read()) / 1e6)
        rows.append((round(time.perf_counter() - t0, 3), *[round(t, 1) for t in times], watts))
    pick = sorted(set(list(range(0, min(12, len(rows)))) + list(range(12, len(rows), max(1, len(rows) // 30)))))
    cols = ["draft call us", "verify call us"] if what == "cycle" else [f"{what} call us"]
    return {"workload": w.name, "traced": what, "columns": ["seconds since start", *cols, "board power W"],
            "batches": len(rows), "rows": [rows[j] for j in pick]}


def time_prefill(torch, B, cache, kd, vd, w, reps=3):
    """Bulk quantization of the whole prompt (Algorithm 1, prefill stage): fp16 K/V read once, both
    planes and the metadata written once."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for i in range(reps):
        ev[i].record()
        B.qs_quantize_prefill(cache, kd, vd, w.n_quant)
    ev[reps].record()
    torch.cuda.synchronize()
    us = min(ev[i].elapsed_time(ev[i + 1]) for i in range(reps)) * 1e3
    nbytes = w.units * w.n_quant * (128 * 2 * 2 + 264)
    # vector instructions per element from the SQ counters in profiles/quantize_mha128k_pipe_utilisation.md;
    # peak = 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
    lane_ops = 24.3 * w.units * w.n_quant * 128 * 2
    return {"us": round(us, 1), "GBps_read_plus_write": round(nbytes / us / 1e3, 1), "bytes": nbytes,
            "tokens_per_unit": w.n_quant,
            "roofline_hbm": {"bound": "hbm", "achieved": round(nbytes / us / 1e3, 1), "peak": HBM_PEAK_GBPS,
                             "unit": "GB/s", "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)},
            "roofline": {"bound": "alu", "achieved": round(lane_ops / us / 1e6, 2), "peak": 39.32,
                         "unit": "T lane-ops/s", "frac": round(lane_ops / us / 1e6 / 39.32, 4)}}


def fp16_baseline(torch, B, cache, w, sm_scale, q_draft, q_verify, draft_us, verify_us, reps=10):
    """The library's own attention over the same context held entirely in fp16 (q_cap = 0): what the
    INT4 draft and INT8 verify calls are compared with, as in Table 4."""
    ws = torch.empty(B.qs_workspace_bytes(cache, q_verify.shape[1]), dtype=torch.uint8, device=q_draft.device)
    res = {}
    nbytes = w.units * w.ctx * 128 * 2 * 2
    for tag, q in (("1_query", q_draft), (f"{q_verify.shape[1]}_queries", q_verify)):
        out = torch.empty_like(q)
        for _ in range(3):
            B.qs_attn_verify(cache, q, sm_scale, out=out, workspace=ws)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        for i in range(reps):
            ev[i].record()
            B.qs_attn_verify(cache, q, sm_scale, out=out, workspace=ws)
        ev[reps].record()
        torch.cuda.synchronize()
        us = float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)])) * 1e3
        res[tag] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1)}
    res["bytes"] = nbytes
    res["draft_speedup_vs_fp16"] = round(res["1_query"]["us"] / draft_us, 3)
    res["verify_speedup_vs_fp16"] = round(res[f"{q_verify.shape[1]}_queries"]["us"] / verify_us, 3)
    return res


def paged_cache(torch, B, w, kd, vd, sm_scale, q_draft, q_verify, reps=60):
    """The headline workload once more as a paged cache: the same codes, every 128-token group at a random
    place of shared pools, found through the group table.  Call times of draft and verify."""
    groups = w.n_quant // 128
    pool = w.units * groups
    c = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.n_quant, w.n_buf + 8, pool_groups=pool)
    perm = np.random.default_rng(11).permutation(pool).astype(np.int32)
    c.group_table.copy_(torch.from_numpy(perm).view_as(c.group_table))
    B.qs_quantize_prefill(c, kd, vd, w.n_quant)
    c.k_buf[:, :, :w.n_buf] = kd[:, :, w.n_quant:]
    c.v_buf[:, :, :w.n_buf] = vd[:, :, w.n_quant:]
    c.n_quant[:], c.n_buf[:] = w.n_quant, w.n_buf
    ws = torch.empty(B.qs_workspace_bytes(c, q_verify.shape[1]), dtype=torch.uint8, device=q_draft.device)
    st, res = c.struct(), {"pool_groups": pool}
    for tag, fn, q in (("draft_us", B.qs_attn_draft, q_draft), ("verify_us", B.qs_attn_verify, q_verify)):
        out = torch.empty_like(q)
        for _ in range(10):
            fn(st, q, sm_scale, out=out, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn(st, q, sm_scale, out=out, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        res[tag] = round(e0.elapsed_time(e1) * 1e3 / reps, 2)
    return res


def speculation_loop(torch, B, cache, w, sm_scale, ws, gammas=SPEC_GAMMAS, accept=0.9, cycles=24):
    """Algorithm 1's decode loop with the buffer policy of Section 4.3.2, acceptance simulated: per
    cycle gamma x (append one token, draft attention), rollback, append gamma + 1 target tokens,
    verify attention, drop the rejected tokens, flush G tokens once 2G verified ones are buffered.
    Reports cache-side microseconds per generated token (accepted drafts + the target's own token)."""
    rng = np.random.default_rng(2502)
    dev = cache.k_buf.device
    out = {"accept_prob": accept, "cycles": cycles, "per_gamma": {}}
    hkv, hq, G = w.n_kv_heads, w.n_q_heads, 128
    for gamma in gammas:
        nq = gamma + 1
        k_new = torch.randn((w.batch, nq, hkv, 128), device=dev, dtype=torch.float16)
        v_new = torch.randn_like(k_new)
        q1 = torch.randn((w.batch, 1, hq, 128), device=dev, dtype=torch.float16)
        qv = torch.randn((w.batch, nq, hq, 128), device=dev, dtype=torch.float16)
        o1, ov = torch.empty_like(q1), torch.empty_like(qv)
        tokens = flushes = 0
        warm = 2                                        # untimed cycles: first launches of this gamma's kernels
        for cyc in range(warm + cycles):
            if cyc == warm:
                tokens = flushes = 0
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            if cache.n_buf.max() >= 2 * G:
                B.qs_quantize_flush(cache, G)
                cache.n_quant += G
                cache.n_buf -= G
                flushes += 1
            for i in range(gamma):
                B.qs_append(cache, k_new[:, i:i + 1].contiguous(), v_new[:, i:i + 1].contiguous())
                cache.n_buf += 1
                B.qs_attn_draft(cache, q1, sm_scale, out=o1, workspace=ws)
            cache.n_buf -= gamma                        # the target pass rewrites the drafted positions
            B.qs_append(cache, k_new, v_new)
            cache.n_buf += nq
            B.qs_attn_verify(cache, qv, sm_scale, out=ov, workspace=ws)
            n_acc = 0
            while n_acc < gamma and rng.random() < accept:
                n_acc += 1
            cache.n_buf -= gamma - n_acc                # rejected tokens leave the buffer
            tokens += n_acc + 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out["per_gamma"][str(gamma)] = {"us_per_token": round(dt * 1e6 / tokens, 2),
                                        "tokens_per_cycle": round(tokens / cycles, 3), "flushes": flushes}
    return out


OTHER_SHAPES = ((64, 32), (64, 64), (128, 32), (128, 64), (256, 32), (256, 64), (256, 128))


def other_shapes(torch, B, ctx=32768, n_buf=256, heads=32, nq_verify=5, seconds=0.25):
    """The other (head_dim, group) shapes on one layer of `heads` kv-heads (no grouped queries) at a 32k
    context: call times of draft and verify with the kernels these shapes share, against the same HBM
    roofline.  Seeded normal K / V; parity of these shapes is the tests' business."""
    out = {}
    gen = torch.Generator(device="cuda").manual_seed(7)
    for d, g in OTHER_SHAPES:
        n_quant = ctx - n_buf
        cache = B.KVCache(1, heads, heads, n_quant, n_buf + 8, head_dim=d, group=g)
        k = torch.randn((1, heads, ctx, d), generator=gen, device="cuda", dtype=torch.float16)
        v = torch.randn((1, heads, ctx, d), generator=gen, device="cuda", dtype=torch.float16)
        B.qs_quantize_prefill(cache, k, v, n_quant)
        cache.k_buf[:, :, :n_buf] = k[:, :, n_quant:]
        cache.v_buf[:, :, :n_buf] = v[:, :, n_quant:]
        cache.n_quant[:], cache.n_buf[:] = n_quant, n_buf
        del k, v
        c = cache.struct()
        ws = torch.empty(B.qs_workspace_bytes(c, nq_verify), dtype=torch.uint8, device="cuda")
        sm = 1.0 / float(np.sqrt(d))
        entry = {"heads": heads, "ctx": ctx}
        for what, nq in (("draft", 1), ("verify", nq_verify)):
            q = torch.randn((1, nq, heads, d), generator=gen, device="cuda", dtype=torch.float16)
            o = torch.empty_like(q)
            call = (lambda: B.qs_attn_verify(c, q, sm, out=o, workspace=ws)) if what == "verify" else \
                   (lambda: B.qs_attn_draft(c, q, sm, out=o, workspace=ws))
            for _ in range(5):
                call()
            torch.cuda.synchronize()
            t0 = time.time()
            call()
            torch.cuda.synchronize()
            reps = int(min(2000, max(10, seconds / max(time.time() - t0, 1e-5))))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1000.0 / reps
            codes = (2 * d) if what == "verify" else d          # K and V codes of one token, bytes
            meta = 4 * (d // g) + 4.0 * d / g                    # value (S, Z) + the token's share of the key (S, Z)
            nbytes = heads * (n_quant * (codes + meta) + n_buf * d * 4) + heads * nq * d * 4
            entry[f"{what}_us"] = round(us, 2)
            entry[f"{what}_GBps"] = round(nbytes / us / 1e3, 1)
            entry[f"{what}_frac"] = round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 3)
        out[f"d{d}_g{g}"] = entry
        del cache, ws
        torch.cuda.empty_cache()
    return out


# The linear layers of one decoder layer of a 7B model (hidden 4096, MLP 11008, 32 layers) and its output
# layer, as the draft model's decode step sees them: 4-bit weights, one row of x.
W4_LAYERS = (("qkv_proj", 12288, 4096), ("o_proj", 4096, 4096), ("gate_up_proj", 22016, 4096), ("down_proj", 4096, 11008),
             ("lm_head", 32000, 4096))
# the same projections of a 70B model (hidden 8192, MLP 28672, 8 kv-heads): where a launch's fixed cost no longer dominates
W4_LAYERS_LARGE = (("qkv_proj_70b", 10240, 8192), ("o_proj_70b", 8192, 8192), ("gate_up_proj_70b", 57344, 8192),
                   ("down_proj_70b", 8192, 28672))


def w4_linear(torch, B, copies_bytes=1 << 30, seconds=0.25):
    """Call times of qs_w4_linear (one row of x) per layer shape, each timed back to back over enough
    independent copies of the weights (1 GiB of them) that the 256 MB last-level cache cannot serve them, as in a
    decode step that walks through the model once per token.  Bytes: the packed weights, x and y."""
    out = {}
    gen = torch.Generator(device="cuda").manual_seed(11)
    for name, n_out, n_in in W4_LAYERS + W4_LAYERS_LARGE:
        nbytes_w = B.qs_w4_bytes(n_out, n_in)
        copies = max(4, -(-copies_bytes // nbytes_w))
        layers = []
        w = torch.randn((n_out, n_in), generator=gen, device="cuda", dtype=torch.float16) * 0.02
        for _ in range(copies):
            layer = B.W4Linear(n_out, n_in)
            B.qs_w4_quantize(layer, w)
            layers.append(layer.struct())
            layers[-1]._keep = layer
        del w
        x = torch.randn((1, n_in), generator=gen, device="cuda", dtype=torch.float16)
        y = torch.empty((1, n_out), device="cuda", dtype=torch.float16)
        lib, stream = B.lib(), torch.cuda.current_stream().cuda_stream or None
        import ctypes

        def run(reps):
            for i in range(reps):
                rc = lib.qs_w4_linear(ctypes.byref(layers[i % copies]), x.data_ptr(), 1, y.data_ptr(), stream)
                if rc != 0:
                    raise B.QsError(rc, "qs_w4_linear")
        run(copies)
        torch.cuda.synchronize()
        t0 = time.time()
        run(copies)
        torch.cuda.synchronize()
        reps = int(min(4000, max(2 * copies, seconds / max((time.time() - t0) / copies, 1e-6))))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(reps)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1000.0 / reps
        nbytes = nbytes_w + 2 * n_in + 2 * n_out
        out[name] = {"n_out": n_out, "n_in": n_in, "copies": copies, "us": round(us, 2), "bytes": nbytes,
                     "GBps": round(nbytes / us / 1e3, 1), "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 3)}
        del layers, x, y
        torch.cuda.empty_cache()
    per_layer = sum(out[n]["us"] for n, _, _ in W4_LAYERS[:4])
    out["decoder_layer_us"] = round(per_layer, 2)
    out["model_32_layers_us"] = round(32 * per_layer + out["lm_head"]["us"], 1)
    return out


def cpu_baseline(w, k_host, v_host, sm_scale, sample_units=6):
    """The float64 oracle, as it stands, on the same cycle for `sample_units` of the workload's
    (sequence, kv-head) units, scaled to all units."""
    from oracle import quantspec_oracle as O
    from paper_2502_10424_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    rep = w.n_q_heads // w.n_kv_heads
    sample_units = min(sample_units, w.n_kv_heads)
    ks, vs = k_host[:1, :sample_units], v_host[:1, :sample_units]
    oc = O.build_cache(ks, vs, rep * sample_units, w.group, w.n_buf)      # prefill quantize: not timed
    qd = synth.gen_layer_q(w, 1)[:1, :, :rep * sample_units]
    qv = synth.gen_layer_q(w, w.nq_verify)[:1, :, :rep * sample_units]
    t0 = time.perf_counter()
    oc.attn_draft(qd, sm_scale)                                           # one of the gamma draft calls
    t_draft = time.perf_counter() - t0
    t0 = time.perf_counter()
    oc.attn_verify(qv, sm_scale)
    t_verify = time.perf_counter() - t0
    t0 = time.perf_counter()
    oc.flush(128)
    t_flush = time.perf_counter() - t0
    scale = w.units * w.n_layers / sample_units
    cyc = (GAMMA * t_draft + t_verify + t_flush) * scale
    return {"value": round(cyc * 1e6 / (GAMMA + 1), 1), "unit": "us/decode-step (same cycle, scaled to all units)",
            "cores": threads, "kind": "oracle",
            "sample": f"{sample_units} of {w.units * w.n_layers} units of {w.name}: 1 draft call (x{GAMMA}), 1 verify call, "
                      f"1 flush of 128 tokens; {t_draft:.2f}s + {t_verify:.2f}s + {t_flush:.3f}s measured, scaled x{scale:.0f}",
            "draft_us": round(t_draft * scale * 1e6, 1), "verify_us": round(t_verify * scale * 1e6, 1)}


if __name__ == "__main__":
    main()
