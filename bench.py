#!/usr/bin/env python3
"""Benchmark of the QuantSpec decode-attention hot path on one MI355X.

One "step" is one speculation cycle of Algorithm 1 over one layer's cache, every stage of the hot
path included: gamma = 4 draft attention calls (1 query, upper plane + buffer), one verify call
(gamma + 1 = 5 causal queries, both planes + buffer) and one quantize-on-flush of G = 128 buffered
tokens (quantize, append, buffer move).  Inputs are resident in HBM before the timed region.  The
cycle rotates over several independent cache copies so the 256 MB last-level cache cannot serve the
planes.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
GAMMA = 4
SPEC_GAMMAS = (1, 2, 4, 6)      # speculation lengths of the simulated decode loop (Table 6)

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (calibrated against a plain copy kernel).  Filled from the summaries under profiles/; None = not measured.
MEASURED_TRAFFIC_BYTES = {
    # profiles/attn_mha128k_hbm_traffic.md: (FETCH_SIZE x 1.99991 + WRITE_SIZE x 1.0) KiB per dispatch
    ("mha128k", "draft"): int((288598.1 * 1.99991 + 1105.1) * 1024),
    ("mha128k", "verify"): int((550709.6 * 1.99991 + 5528.3) * 1024),
}


def algorithmic_bytes(w, nq, verify):
    """Bytes one attention call must move (fp16 metadata): per quantized token and unit 64 (K upper)
    + 64 (V upper) + 4 (K scale/zero, amortised over the group) + 4 (V scale/zero); twice the plane
    bytes for verify; plus the fp16 buffer and q / out."""
    per_tok = (128 + 128 + 8) if verify else (64 + 64 + 8)
    return w.units * (w.n_quant * per_tok + w.n_buf * 128 * 2 * 2) + w.batch * w.n_q_heads * nq * 128 * 2 * 2


def flush_bytes(w, n):
    return w.units * n * (128 * 2 * 2 + (128 + 128 + 4 + 4))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="mha128k")
    ap.add_argument("--copies", type=int, default=4, help="independent cache copies to rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--deterministic", action="store_true",
                    help="time the bit-reproducible setting (QS_FLAG_FIXED_RANGES) instead of the default")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed cycle: no prefill timing, fp16 baseline or speculation loop (for kernel traces)")
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
    if args.deterministic:
        B.KVCache.default_flags = B.QS_FLAG_FIXED_RANGES
    w = synth.WORKLOADS[args.workload]
    sm_scale = 1.0 / float(np.sqrt(w.head_dim))
    nqv = w.nq_verify
    dev = "cuda"

    # ---- synthetic inputs, resident in HBM ------------------------------------------------------
    t0 = time.time()
    workers = min(16, os.cpu_count() or 8)
    k_host, v_host = synth.gen_layer_kv(w, workers=workers)
    q_draft = torch.from_numpy(synth.gen_layer_q(w, 1)).to(dev)
    q_verify = torch.from_numpy(synth.gen_layer_q(w, nqv)).to(dev)
    q_cap = w.n_quant + 640            # room for the groups flushed during the run
    caches = []
    kd, vd = torch.from_numpy(k_host).to(dev), torch.from_numpy(v_host).to(dev)
    for i in range(args.copies):
        c = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, q_cap, w.n_buf + 8)
        if i == 0:
            B.qs_quantize_prefill(c, kd, vd, w.n_quant)
            prefill = None if args.no_extras else time_prefill(torch, B, c, kd, vd, w)
        else:
            for name in B.PLANES:
                getattr(c, name).copy_(getattr(caches[0], name))
        c.k_buf[:, :, :w.n_buf] = kd[:, :, w.n_quant:]
        c.v_buf[:, :, :w.n_buf] = vd[:, :, w.n_quant:]
        c.n_quant[:] = w.n_quant
        c.n_buf[:] = w.n_buf
        caches.append(c)
    # the same tokens as a plain fp16 cache (no quantized region): the baseline of Table 4
    fp16_cache = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, 0, w.ctx)
    fp16_cache.k_buf, fp16_cache.v_buf = kd, vd
    fp16_cache.n_buf[:] = w.ctx
    del kd, vd
    ws = torch.empty(max(B.qs_workspace_bytes(caches[0], n) for n in (1, nqv, max(SPEC_GAMMAS) + 1)),
                     dtype=torch.uint8, device=dev)
    out_d = torch.empty_like(q_draft)
    out_v = torch.empty_like(q_verify)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    ev = lambda: torch.cuda.Event(enable_timing=True)
    timed = {"draft": [], "verify": [], "flush": []}

    def cycle(i, record):
        """One speculation cycle on cache copy i.  With record=True four events bracket the three
        phases (the draft figure is the mean of the gamma back-to-back calls)."""
        c = caches[i % len(caches)]
        if record:
            e = [ev() for _ in range(4)]
            e[0].record()
        for _ in range(GAMMA):
            B.qs_attn_draft(c, q_draft, sm_scale, out=out_d, workspace=ws)
        if record:
            e[1].record()
        B.qs_attn_verify(c, q_verify, sm_scale, out=out_v, workspace=ws)
        if record:
            e[2].record()
        B.qs_quantize_flush(c, 128)     # host lengths stay put: the same group slot is rewritten each cycle
        if record:
            e[3].record()
            timed["draft"].append((e[0], e[1], GAMMA))
            timed["verify"].append((e[1], e[2], 1))
            timed["flush"].append((e[2], e[3], 1))

    for i in range(args.warmup):
        cycle(i, False)
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()                      # no collector pause inside the timed region
    t_start = time.perf_counter()
    for i in range(args.steps):
        cycle(args.warmup + i, True)
        if i >= 2:
            # stay at most two cycles ahead of the GPU (a decoder reads each cycle's outcome anyway);
            # letting the host queue hundreds of launches ahead has stalled the runtime for tens of ms
            timed["flush"][i - 2][1].synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    gc.enable()

    ms_per_step = elapsed * 1e3 / args.steps
    per_call = {k: np.array([1e3 * a.elapsed_time(b) / n for a, b, n in v]) for k, v in timed.items()}
    avg_us = {k: float(v.mean()) for k, v in per_call.items()}
    bytes_d, bytes_v = algorithmic_bytes(w, 1, False), algorithmic_bytes(w, nqv, True)
    gbps_d = bytes_d / (avg_us["draft"] * 1e-6) / 1e9
    gbps_v = bytes_v / (avg_us["verify"] * 1e-6) / 1e9
    cycle_bytes = GAMMA * bytes_d + bytes_v + flush_bytes(w, 128)

    result = {
        "metric": "draft/verify attention us per decode step + achieved HBM GB/s at 128k ctx",
        "value": round(ms_per_step * 1e3 / (GAMMA + 1), 3),
        "unit": "us/decode-step (mean over a cycle of 4 draft + 1 verify call, flush included)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads} q-heads / {w.n_kv_heads} kv-heads x 128, "
                               f"ctx {w.ctx} = {w.n_quant} quantized + {w.n_buf} fp16 buffer, G=128, gamma=4",
                   "cache_copies_rotated": len(caches), "flush_tokens_per_cycle": 128,
                   "deterministic": bool(args.deterministic)},
        "draft_us": round(avg_us["draft"], 2), "verify_us": round(avg_us["verify"], 2),
        "flush_us": round(avg_us["flush"], 2),
        "median_us": {k: round(float(np.median(v)), 2) for k, v in per_call.items()},
        "min_us": {k: round(float(v.min()), 2) for k, v in per_call.items()},
        "draft_GBps": round(gbps_d, 1), "verify_GBps": round(gbps_v, 1),
        "cycle_GBps": round(cycle_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "kernel": "draft call: attn_kernel_cu<false,true> + merge_kernel (upper plane)",
                     "achieved": round(gbps_d, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps_d / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": bytes_d,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "draft"))},
        "roofline_verify": {"bound": "hbm", "kernel": "verify call: attn_kernel_cu<true,false> + merge_kernel (both planes)",
                            "achieved": round(gbps_v, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": round(gbps_v / HBM_PEAK_GBPS, 4),
                            "algorithmic_bytes_per_launch": bytes_v,
                            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "verify"))},
        "setup_s": round(setup_s, 1),
    }

    if not args.no_extras:
        result["prefill_quantize"] = prefill
        result["fp16_baseline"] = fp16_baseline(torch, B, fp16_cache, w, sm_scale, q_draft, q_verify,
                                                avg_us["draft"], avg_us["verify"])
        result["speculation"] = speculation_loop(torch, B, caches[0], w, sm_scale, ws)
    del fp16_cache
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, k_host, v_host, sm_scale)
    print(json.dumps(result), flush=True)


def time_prefill(torch, B, cache, kd, vd, w, reps=3):
    """Bulk quantization of the whole prompt (Algorithm 1, prefill stage): fp16 K/V read once, both
    planes and the metadata written once.  The kernel is bound by the quantizer's vector arithmetic."""
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
    scale = w.units / sample_units
    cyc = (GAMMA * t_draft + t_verify + t_flush) * scale
    return {"value": round(cyc * 1e6 / (GAMMA + 1), 1), "unit": "us/decode-step (same cycle, scaled to all units)",
            "cores": threads, "kind": "oracle",
            "sample": f"{sample_units} of {w.units} units: 1 draft call (x{GAMMA}), 1 verify call, 1 flush of 128 "
                      f"tokens; {t_draft:.2f}s + {t_verify:.2f}s + {t_flush:.3f}s measured, scaled x{scale:.0f}",
            "draft_us": round(t_draft * scale * 1e6, 1), "verify_us": round(t_verify * scale * 1e6, 1)}


if __name__ == "__main__":
    main()
