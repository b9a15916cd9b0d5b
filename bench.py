#!/usr/bin/env python3
"""Benchmark of the AhaKV eviction hot path on one MI355X.

One "step" is the prefill eviction of one layer of synthetic input already
resident in HBM: eviction scores -> top-k selection -> KV compaction, on the
32K-context GQA layer (batch 1, 32 query / 8 KV heads, head_dim 128, bf16,
window 64, budget 2048).  The generation step with running eviction on the fresh
cache is timed beside it (`decode_step_c3`, and `decode_c4` for the batched
configuration), as the metric quotes the two separately.

Prints ONE JSON line: the step time (mean over the timed steps; median and minimum from
per-step events) and throughput, per-kernel times from HIP events on the launch stream, the
roofline of the dominant kernel, side measurements of the other configurations and the CPU
oracle timed on the same step.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, GB/s
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


SETTLE_MS = 40.0


def settle(torch, fn, ms=SETTLE_MS):
    """Keep the GPU busy with `fn` for about `ms` of host time, then drain.  After the seconds of
    idle time in which a workload is generated the device sits in a low power state, and the
    first milliseconds of work run 5 - 7 % slower than the steady state an inference loop sees
    (measured: 20 steps of the 32K layer take 92 - 94 us each after idling and 87 us each right
    after a busy period).  Called before the warm-up steps of every timed section; the timed
    region itself is untouched."""
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        fn()
    torch.cuda.synchronize()


def avg_ms(pairs):
    return sum(a.elapsed_time(b) for a, b in pairs) / max(len(pairs), 1)


def us_stats(pairs):
    """mean / median / min in microseconds of event pairs (already synchronised)."""
    t = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
    if not t:
        return {"mean": None, "median": None, "min": None}
    mid = len(t) // 2
    med = t[mid] if len(t) % 2 else 0.5 * (t[mid - 1] + t[mid])
    return {"mean": sum(t) / len(t), "median": med, "min": t[0]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle timing (used under rocprofv3)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the C4 decode and C2 full-accumulation side measurements")
    ap.add_argument("--only", choices=["decode_c4", "full_c2", "full_c3", "c5_layer", "c2_layer", "window_attn"], default=None,
                    help="run one side measurement alone and print it (for profiling that kernel)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB elementwise kernel (calibrates the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters against a known size)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_03762_amd import binding as B, synth, workload as H

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.load()
    K_STEPS, W_STEPS = args.steps, args.warmup

    if args.copy_probe:
        # an elementwise kernel that reads 256 MiB and writes 256 MiB
        src = torch.ones(64 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if args.only:
        fn = {"decode_c4": lambda: bench_decode_c4(torch, B, synth, H, K_STEPS),
              "full_c2": lambda: bench_full_c2(torch, B, synth, H, max(5, K_STEPS // 5)),
              "full_c3": lambda: bench_full_c3_alone(torch, B, synth, H),
              "c5_layer": lambda: bench_c5_layer(torch, B, synth, H, max(5, K_STEPS // 5)),
              "c2_layer": lambda: bench_windowed_layer(torch, B, synth, H, synth.C2, K_STEPS),
              "window_attn": lambda: bench_window_attn_alone(torch, B, synth, H, K_STEPS)}[args.only]
        print(json.dumps({"only": args.only, args.only: fn()}))
        return

    # ------------------------------------------------------------ workload --
    w = synth.C3
    log("generating", w.name)
    Q, K, V = synth.make_prefill(w, threads=16)
    q, k, v = (H.to_device(a, w.dtype) for a in (Q, K, V))
    p = H.params_for(w).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    b, hq, hk, n, d, G = w.batch, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim, w.group
    scores = torch.empty((b, hk, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((b, hk, w.budget), dtype=torch.int32, device="cuda")
    cache = B.CompactCache.empty(p)
    qn, kn, vn = (H.to_device(a, w.dtype) for a in synth.make_decode_inputs(w, 0))
    out = torch.empty((b, hq, d), dtype=torch.bfloat16, device="cuda")

    def step():
        B.aha_prefill_scores(p, q, k, v, scores, ws)
        B.aha_select_topk(p, scores, idx, ws)
        B.aha_compact_kv(p, k, v, scores, idx, cache.k, cache.v, cache.scores, cache.pos,
                         cache.free_slot)

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    settle(torch, step)
    for _ in range(W_STEPS):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K_STEPS):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K_STEPS
    # the same steps once more, each between two events: median and minimum
    step_evs = []
    for _ in range(K_STEPS):
        e0 = ev(); step(); step_evs.append((e0, ev()))
    torch.cuda.synchronize()
    step_us = us_stats(step_evs)

    # the same layer with the configuration's other budget (1024): selection and compaction change
    import dataclasses
    p_small = dataclasses.replace(p, budget=w.budget // 2)
    idx_small = torch.empty((b, hk, w.budget // 2), dtype=torch.int32, device="cuda")
    cache_small = B.CompactCache.empty(p_small)

    def step_small():
        B.aha_prefill_scores(p_small, q, k, v, scores, ws)
        B.aha_select_topk(p_small, scores, idx_small, ws)
        B.aha_compact_kv(p_small, k, v, scores, idx_small, cache_small.k, cache_small.v,
                         cache_small.scores, cache_small.pos, cache_small.free_slot)

    for _ in range(W_STEPS):
        step_small()
    e0 = ev()
    for _ in range(K_STEPS):
        step_small()
    e1 = ev()
    torch.cuda.synchronize()
    step_small_us = e0.elapsed_time(e1) * 1e3 / K_STEPS

    # ------------------------------------------- per-kernel times (events) --
    # Events on the launch stream bracket every launch; between two launches that were
    # enqueued back to back they measure the kernel plus the dispatch gap before it (2-3 us
    # more than the kernel duration a profiler reports).
    stage_sets, call_sets = [], []
    for _ in range(K_STEPS):
        st = [ev() for _ in range(4)]
        B.profile_events(st)
        B.aha_prefill_scores(p, q, k, v, scores, ws)
        B.profile_events(None)
        e0 = ev(); B.aha_select_topk(p, scores, idx, ws)
        e1 = ev(); B.aha_compact_kv(p, k, v, scores, idx, cache.k, cache.v, cache.scores,
                                    cache.pos, cache.free_slot)
        e2 = ev(); B.aha_decode_step(p, qn, kn, vn, cache.k, cache.v, cache.scores, cache.pos,
                                     cache.free_slot, n + 1, out, ws)
        e3 = ev()
        stage_sets.append(st)
        call_sets.append((e0, e1, e2, e3))
    torch.cuda.synchronize()
    # generation steps on that cache launched back to back, as a generation loop issues them
    # (an event pair around a single step adds the dispatch gap of an idle stream)
    n_dec = 64
    d0 = ev()
    for t in range(n_dec):
        B.aha_decode_step(p, qn, kn, vn, cache.k, cache.v, cache.scores, cache.pos,
                          cache.free_slot, n + 2 + t, out, ws)
    d1 = ev()
    torch.cuda.synchronize()
    decode_b2b_us = d0.elapsed_time(d1) * 1e3 / n_dec
    # (bf16 windowed scores form the value prior inside the row-statistics launch: the
    # library records events[0] and [1] back to back and pass 1 is bracketed by [1] and [2])
    kstats = {
        "score_pass1": us_stats([(s[1], s[2]) for s in stage_sets]),
        "score_pass2": us_stats([(s[2], s[3]) for s in stage_sets]),
        "topk": us_stats([(c[0], c[1]) for c in call_sets]),
        "compact": us_stats([(c[1], c[2]) for c in call_sets]),
        "decode_step": us_stats([(c[2], c[3]) for c in call_sets]),
    }
    event_gap = us_stats([(s[0], s[1]) for s in stage_sets])   # two events, nothing between
    kt = {name: st["mean"] * 1e-3 for name, st in kstats.items()}   # ms
    e = 2  # bf16 bytes
    kbytes = b * hk * n * d * e
    qbytes = b * hq * w.window * d * e
    alg = {  # algorithmic HBM bytes per launch
        "score_pass1": 2 * kbytes + qbytes + b * hk * n * 4,   # K, V (value prior), Q rows; gamma out
        "score_pass2": kbytes + qbytes + b * hk * n * 4,
        "topk": b * hk * n * 4 + b * hk * w.budget * 4,
        "compact": 4 * b * hk * w.budget * d * e + b * hk * w.budget * 12,
        "decode_step": b * hk * (2 * (w.budget + 1) * d * e + 8 * (w.budget + 1) + 2 * d * e)
                       + 2 * b * hq * d * e,
    }
    kernels = {name: {"us": kt[name] * 1e3, "median_us": kstats[name]["median"],
                      "min_us": kstats[name]["min"], "alg_bytes": alg[name],
                      "GBps": alg[name] / (kt[name] * 1e-3) / 1e9 if kt[name] > 1e-6 else None}
               for name in kt}
    score_flops_pass = 2.0 * d * b * hq * (w.window * n - w.window * (w.window - 1) / 2)
    for name in ("score_pass1", "score_pass2"):
        kernels[name]["TFLOPs"] = score_flops_pass / (kt[name] * 1e-3) / 1e12
    dom = max(("score_pass1", "score_pass2", "topk", "compact"), key=lambda nm: kt[nm])
    # HBM bytes per launch from the committed rocprofv3 counter summary of this workload
    traffic = None
    try:
        tj = json.load(open(os.path.join(ROOT, "profiles", "c3_hbm_traffic.json")))
        if tj.get("workload") == w.name and dom in tj["kernels"]:
            traffic = tj["kernels"][dom]["total_bytes"]
    except (OSError, ValueError, KeyError):
        traffic = None
    roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels[dom]["GBps"] / HBM_PEAK_GBS,
                "traffic": traffic,
                "timing": "mean of HIP events around the launch on its stream (kernel + dispatch gap)",
                "kernel_us": kt[dom] * 1e3, "alg_bytes": alg[dom]}
    # the whole score stage against the bytes the method needs once (K + V + Q window)
    stage_ms = kt["score_pass1"] + kt["score_pass2"]
    stage_bytes = 2 * kbytes + qbytes + b * hk * n * 4
    roofline_stage = {"stage": "prefill_scores (all its launches)", "bound": "hbm",
                      "achieved": stage_bytes / (stage_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                      "unit": "GB/s", "frac": stage_bytes / (stage_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "mfma_TFLOPs": 2 * score_flops_pass / (stage_ms * 1e-3) / 1e12}

    result = {
        "metric": "prefill eviction us/layer @32K ctx (scores + top-k + compaction)",
        "value": ms_per_step * 1e3, "unit": "us/layer", "n_gpus": 1, "steps": K_STEPS,
        "warmup": W_STEPS, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": b, "n_q_heads": hq, "n_kv_heads": hk,
                   "head_dim": d, "seq_len": n, "window": w.window, "budget": w.budget,
                   "recent": w.recent, "scale": "adaptive", "value_prior": True},
        "tokens_per_s": b * n / (ms_per_step * 1e-3),
        "step_us": {"mean_wall_clock": ms_per_step * 1e3, "median_events": step_us["median"],
                    "min_events": step_us["min"]},
        "step_us_budget_1024": step_small_us,
        "device_settle_ms": SETTLE_MS,  # untimed busy period before the warm-up steps (see settle)
        "decode_step_c3": {"back_to_back_us": decode_b2b_us,
                           "median_us": kstats["decode_step"]["median"],
                           "min_us": kstats["decode_step"]["min"],
                           "tokens_per_s": b / (decode_b2b_us * 1e-6),
                           "note": "one generation step on the 8-head cache (two launches, "
                                   "latency-bound): 64 steps back to back, and single steps "
                                   "between two events (which adds the dispatch gap)"},
        "roofline": roofline, "roofline_stage": roofline_stage, "kernels": kernels,
        "event_gap_us": event_gap["median"],
        "note": "the 134 MB of C3 inputs are re-read every step and fit the 256 MB last-level "
                "cache: GB/s figures of this workload are fabric-side rates; prefill_c5_layer is "
                "the HBM-bound shape",
    }

    if not args.no_extras:
        result["decode_c4"] = bench_decode_c4(torch, B, synth, H, K_STEPS)
        result["decode_c4_grouped_query"] = bench_decode_gqa(torch, B)
        result["full_accumulation_c2"] = bench_full_c2(torch, B, synth, H, max(5, K_STEPS // 5))
        result["prefill_c5_layer"] = bench_c5_layer(torch, B, synth, H, max(5, K_STEPS // 5))
        result["prefill_c2_layer"] = bench_windowed_layer(torch, B, synth, H, synth.C2, K_STEPS)
        result["scores_from_lse_c3"] = bench_lse_c3(torch, B, H, w, p, q, k, v, scores, ws, K_STEPS)
        result["window_attention_c3"] = bench_window_attn_c3(torch, B, w, p, q, k, v, scores, ws, K_STEPS)
        result["full_accumulation_c3"] = bench_full_c3(torch, B, w, p, q, k, v, scores)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, (Q, K, V))
    print(json.dumps(result))


def bench_decode_c4(torch, B, synth, H, steps):
    """Decode step at batch 8 x 32 heads, budget 1024 (bound by HBM bandwidth)."""
    w = synth.C4
    log("generating", w.name)
    Q, K, V = synth.make_prefill(w, threads=16)
    q, k, v = (H.to_device(a, w.dtype) for a in (Q, K, V))
    p = H.params_for(w).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    b, hq, hk, n, d = w.batch, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    scores = torch.empty((b, hk, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((b, hk, w.budget), dtype=torch.int32, device="cuda")
    B.aha_prefill_scores(p, q, k, v, scores, ws)
    B.aha_select_topk(p, scores, idx, ws)
    ncopies = 4  # 4 x 134 MB of cache state: more than the 256 MB last-level cache
    caches = [B.CompactCache.empty(p) for _ in range(ncopies)]
    for c in caches:
        B.aha_compact_kv(p, k, v, scores, idx, c.k, c.v, c.scores, c.pos, c.free_slot)
    del q
    nsteps = w.decode_steps
    g = torch.Generator(device="cuda"); g.manual_seed(1234)
    qs = torch.randn((nsteps, b, hq, d), device="cuda", generator=g).to(torch.bfloat16)
    ks = torch.randn((nsteps, b, hk, d), device="cuda", generator=g).to(torch.bfloat16)
    vs = torch.randn((nsteps, b, hk, d), device="cuda", generator=g).to(torch.bfloat16)
    out = torch.empty((b, hq, d), dtype=torch.bfloat16, device="cuda")
    alg = b * hk * (2 * (w.budget + 1) * d * 2 + 8 * (w.budget + 1) + 2 * d * 2) + 2 * b * hq * d * 2

    def run(rotate):
        # the paper-shaped run: 256 consecutive steps, enqueued back to back as a generation
        # loop does; two events bracket steps 32..255 and the step time is their mean (an
        # event pair around every single step adds 2-3 us of dispatch gap to each)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        for t in range(nsteps):
            c = caches[t % ncopies] if rotate else caches[0]
            if t == 32:
                e0.record()
            B.aha_decode_step(p, qs[t], ks[t], vs[t], c.k, c.v, c.scores, c.pos, c.free_slot,
                              n + 1 + (t // ncopies if rotate else t), out, ws)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (nsteps - 32)

    def reset():
        for c in caches:
            B.aha_compact_kv(p, k, v, scores, idx, c.k, c.v, c.scores, c.pos, c.free_slot)

    for _ in range(4):  # warm-up passes over all 256 steps (and out of the idle power state)
        run(False)
    reset()
    us_hot = run(False)
    reset()
    us_cold = run(True)
    return {"workload": w.name, "decode_step_us": us_hot, "tokens_per_s": b / (us_hot * 1e-6),
            "alg_bytes": alg,
            "roofline": {"bound": "hbm", "achieved": alg / (us_hot * 1e-6) / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": alg / (us_hot * 1e-6) / 1e9 / HBM_PEAK_GBS,
                         "note": "134 MB of cache state fits the 256 MB last-level cache"},
            "cache_defeated": {"decode_step_us": us_cold, "copies": ncopies,
                               "achieved": alg / (us_cold * 1e-6) / 1e9,
                               "frac": alg / (us_cold * 1e-6) / 1e9 / HBM_PEAK_GBS}}


def bench_decode_gqa(torch, B):
    """The batched decode size (256 KV heads x budget 1024, bf16) with grouped-query attention:
    4 and 8 query heads per KV head.  Caches filled with random rows (timing only), four in
    rotation, steps launched back to back."""
    res = {}
    bsz, hk, d, budget = 8, 32, 128, 1024
    g = torch.Generator(device="cuda"); g.manual_seed(99)
    for G in (4, 8):
        hq = hk * G
        p = B.Params(batch=bsz, n_q_heads=hq, n_kv_heads=hk, head_dim=d, seq_len=0, window=0,
                     budget=budget, recent=64)
        caches = []
        for _ in range(4):
            c = B.CompactCache.empty(p)
            c.k.copy_(torch.randn(c.k.shape, device="cuda", generator=g)); c.v.copy_(c.k)
            c.scores.uniform_(); c.free_slot.fill_(budget)
            c.pos.copy_(torch.arange(budget + 1, dtype=torch.int32, device="cuda")
                        .expand(bsz, hk, budget + 1))
            c.pos[:, :, budget] = -1
            caches.append(c)
        q = torch.randn((bsz, hq, d), device="cuda", generator=g).to(torch.bfloat16)
        kv = torch.randn((bsz, hk, d), device="cuda", generator=g).to(torch.bfloat16)
        out = torch.empty_like(q)
        ws = torch.empty(max(256, B.workspace_bytes(p)), dtype=torch.uint8, device="cuda")
        alg = bsz * hk * (2 * (budget + 1) * d * 2 + 8 * (budget + 1) + 2 * d * 2) + 2 * bsz * hq * d * 2

        def run(steps):
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            for t in range(steps):
                c = caches[t % 4]
                if t == 16:
                    e0.record()
                B.aha_decode_step(p, q, kv, kv, c.k, c.v, c.scores, c.pos, c.free_slot,
                                  budget + 100 + t // 4, out, ws)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / (steps - 16)

        run(1024)  # (also brings the device out of its idle power state: see settle)
        us = run(144)
        res["group_%d" % G] = {"decode_step_us": us, "alg_bytes": alg,
                               "hbm_frac": alg / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    res["note"] = ("random cache contents, four caches in rotation; 8 query heads per KV head: "
                   "dots on the matrix core")
    return res


def bench_full_c2(torch, B, synth, H, steps):
    """Full accumulation (window = n, fixed 1/sqrt(d), no value prior) on the
    Llama-2-7B-shaped layer: the n x n contraction, bound by the matrix cores."""
    w = synth.C2
    log("generating", w.name)
    Q, K, V = synth.make_prefill(w, threads=16)
    q, k, v = (H.to_device(a, w.dtype) for a in (Q, K, V))
    p = H.params_for(w, window=w.seq_len, scale_mode=B.AHA_SCALE_FIXED,
                     fixed_scale=1 / math.sqrt(w.head_dim), value_prior=False).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    b, hq, hk, n, d = w.batch, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    scores = torch.empty((b, hk, n), dtype=torch.float32, device="cuda")
    settle(torch, lambda: B.aha_prefill_scores(p, q, k, v, scores, ws))
    sets = []
    for _ in range(steps):
        st = []
        for _ in range(4):
            e = torch.cuda.Event(enable_timing=True); e.record(); st.append(e)
        B.profile_events(st)
        B.aha_prefill_scores(p, q, k, v, scores, ws)
        B.profile_events(None)
        sets.append(st)
    torch.cuda.synchronize()
    p1 = avg_ms([(s[1], s[2]) for s in sets]); p2 = avg_ms([(s[2], s[3]) for s in sets])
    flops_pass = 2.0 * d * b * hq * n * (n + 1) / 2
    tf = 2 * flops_pass / ((p1 + p2) * 1e-3) / 1e12
    return {"workload": w.name + " window=n fixed-scale", "pass1_us": p1 * 1e3, "pass2_us": p2 * 1e3,
            "flops_per_pass": flops_pass,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS},
            "pass1_TFLOPs": flops_pass / (p1 * 1e-3) / 1e12,
            "pass2_TFLOPs": flops_pass / (p2 * 1e-3) / 1e12}


def bench_full_c3(torch, B, w, p, q, k, v, scores, steps=3):
    """Full accumulation (window = n, fixed 1/sqrt(d), no value prior) at the 32K-context GQA
    shape: 8.8e12 flops over the two passes, the n x n contraction at its full size."""
    import dataclasses
    n, d = w.seq_len, w.head_dim
    pf = dataclasses.replace(p, window=n, scale_mode=B.AHA_SCALE_FIXED, fixed_scale=1.0 / math.sqrt(d),
                             value_prior=0)
    ws = B.alloc_workspace(pf)
    B.aha_prefill_scores(pf, q, k, v, scores, ws)
    sets = []
    for _ in range(steps):
        st = []
        for _ in range(4):
            e = torch.cuda.Event(enable_timing=True); e.record(); st.append(e)
        B.profile_events(st)
        B.aha_prefill_scores(pf, q, k, v, scores, ws)
        B.profile_events(None)
        sets.append(st)
    torch.cuda.synchronize()
    p1 = avg_ms([(s[1], s[2]) for s in sets]); p2 = avg_ms([(s[2], s[3]) for s in sets])
    flops_pass = 2.0 * d * w.batch * w.n_q_heads * n * (n + 1) / 2
    tf = 2 * flops_pass / ((p1 + p2) * 1e-3) / 1e12
    total = float(scores.sum()) / (w.batch * w.n_q_heads * n)   # rows sum to one: must be 1
    return {"workload": w.name + " window=n fixed-scale", "pass1_us": p1 * 1e3, "pass2_us": p2 * 1e3,
            "flops_per_pass": flops_pass, "mean_row_sum": total,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS}}


def bench_full_c3_alone(torch, B, synth, H):
    """bench_full_c3 with inputs of its own (for profiling that measurement alone)."""
    w = synth.C3
    log("generating", w.name)
    q, k, v = (H.to_device(a, w.dtype) for a in synth.make_prefill(w, threads=16))
    p = H.params_for(w).with_strides(q, k, v)
    scores = torch.empty((w.batch, w.n_kv_heads, w.seq_len), dtype=torch.float32, device="cuda")
    return bench_full_c3(torch, B, w, p, q, k, v, scores)


def bench_lse_c3(torch, B, H, w, p, q, k, v, scores, ws, steps):
    """The score stage on the C3 layer with the standard scale 1/sqrt(d): two passes, against
    one pass when the caller hands over the rows' log-sum-exp (as an attention forward pass
    keeps it).  The log-sum-exp fed here is formed with torch from the same Q and K."""
    import dataclasses
    n, d, r, G = w.seq_len, w.head_dim, w.window, w.group
    scale = 1.0 / math.sqrt(d)
    pf = dataclasses.replace(p, scale_mode=B.AHA_SCALE_FIXED, fixed_scale=scale)
    qw = q[:, :, n - r:, :].float()                                    # [b, Hq, r, d]
    kf = k.float().repeat_interleave(G, dim=1)                         # [b, Hq, n, d]
    logits = torch.einsum("bhrd,bhnd->bhrn", qw, kf) * scale
    causal = torch.arange(n, device="cuda")[None, :] <= (n - r + torch.arange(r, device="cuda"))[:, None]
    lse = torch.logsumexp(logits.masked_fill(~causal, float("-inf")), dim=-1).contiguous()
    del logits, kf

    def timed(fn):
        settle(torch, fn)
        evs = []
        for _ in range(steps):
            e0 = torch.cuda.Event(enable_timing=True); e0.record()
            fn()
            e1 = torch.cuda.Event(enable_timing=True); e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return avg_ms(evs) * 1e3

    two = timed(lambda: B.aha_prefill_scores(pf, q, k, v, scores, ws))
    ref = scores.clone()
    one = timed(lambda: B.aha_prefill_scores_lse(pf, q, k, v, lse, scores, ws))
    err = float(((scores - ref).abs() / (ref.abs() + 1e-6)).max())
    return {"workload": w.name + " fixed scale 1/sqrt(d)", "two_pass_us": two, "from_lse_us": one,
            "max_rel_diff": err}


def bench_window_attn_c3(torch, B, w, p, q, k, v, scores, ws, steps):
    """Attention output of the 64 observed rows of all heads on the C3 layer (one flash-style
    pass on the matrix cores, two contractions), and output + scores through its log-sum-exp
    (that launch, then the column-sum pass alone) against the two-pass scores alone."""
    import dataclasses
    n, d, r = w.seq_len, w.head_dim, w.window
    pf = dataclasses.replace(p, scale_mode=B.AHA_SCALE_FIXED, fixed_scale=1.0 / math.sqrt(d))
    wsa = torch.empty(max(B.window_attention_workspace_bytes(pf), 256), dtype=torch.uint8, device="cuda")
    out = torch.empty((w.batch, w.n_q_heads, r, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((w.batch, w.n_q_heads, r), dtype=torch.float32, device="cuda")

    def timed(fn):
        settle(torch, fn)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps

    def both():
        B.aha_prefill_window_attention(pf, q, k, v, out, lse, wsa)
        B.aha_prefill_scores_lse(pf, q, k, v, lse, scores, ws)

    attn = timed(lambda: B.aha_prefill_window_attention(pf, q, k, v, out, lse, wsa))
    flops = 2 * 2.0 * d * w.batch * w.n_q_heads * (r * n - r * (r - 1) / 2)
    return {"workload": w.name + " window rows, standard scale", "attention_us": attn,
            "flops": flops, "TFLOPs": flops / (attn * 1e-6) / 1e12,
            "mfma_frac": flops / (attn * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "attention_plus_scores_us": timed(both),
            "two_pass_scores_alone_us": timed(lambda: B.aha_prefill_scores(pf, q, k, v, scores, ws))}


def bench_window_attn_alone(torch, B, synth, H, steps):
    """bench_window_attn_c3 with inputs of its own (for profiling that measurement alone)."""
    w = synth.C3
    log("generating", w.name)
    q, k, v = (H.to_device(a, w.dtype) for a in synth.make_prefill(w, threads=16))
    p = H.params_for(w).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    scores = torch.empty((w.batch, w.n_kv_heads, w.seq_len), dtype=torch.float32, device="cuda")
    return bench_window_attn_c3(torch, B, w, p, q, k, v, scores, ws, steps)


def bench_c5_layer(torch, B, synth, H, steps):
    """One layer of the full-depth sweep (batch 4 x 32 heads x 16384, budget 3276): the
    shape at which the windowed score, the value prior and the compaction are bound by HBM
    bandwidth."""
    return bench_windowed_layer(torch, B, synth, H, synth.C5, steps)


def bench_windowed_layer(torch, B, synth, H, w, steps):
    """The prefill step (scores, top-k, compaction) of one layer of workload `w`, per kernel
    between events and as a whole back to back.  Timing only: seeded Gaussian Q/K/V drawn on
    the device."""
    b, hq, hk, n, d = w.batch, w.n_q_heads, w.n_kv_heads, w.seq_len, w.head_dim
    g = torch.Generator(device="cuda"); g.manual_seed(synth.BASE_SEED + 1000 * w.cfg_id)
    q, k, v = (torch.randn((b, hh, n, d), device="cuda", generator=g).to(torch.bfloat16)
               for hh in (hq, hk, hk))
    p = H.params_for(w).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    scores = torch.empty((b, hk, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((b, hk, w.budget), dtype=torch.int32, device="cuda")
    cache = B.CompactCache.empty(p)

    def ev():
        e = torch.cuda.Event(enable_timing=True); e.record(); return e

    def step():
        B.aha_prefill_scores(p, q, k, v, scores, ws)
        B.aha_select_topk(p, scores, idx, ws)
        B.aha_compact_kv(p, k, v, scores, idx, cache.k, cache.v, cache.scores, cache.pos,
                         cache.free_slot)

    settle(torch, step)
    sets = []
    for it in range(steps + 2):
        st = [ev() for _ in range(4)]
        B.profile_events(st)
        B.aha_prefill_scores(p, q, k, v, scores, ws)
        B.profile_events(None)
        e0 = ev(); B.aha_select_topk(p, scores, idx, ws)
        e1 = ev(); B.aha_compact_kv(p, k, v, scores, idx, cache.k, cache.v, cache.scores,
                                    cache.pos, cache.free_slot)
        e2 = ev()
        if it >= 2:
            sets.append((st, e0, e1, e2))
    torch.cuda.synchronize()
    t = {"score_pass1": avg_ms([(s[0][1], s[0][2]) for s in sets]),
         "score_pass2": avg_ms([(s[0][2], s[0][3]) for s in sets]),
         "topk": avg_ms([(s[1], s[2]) for s in sets]),
         "compact": avg_ms([(s[2], s[3]) for s in sets])}
    kb = b * hk * n * d * 2
    # pass 1 also forms the value prior of its key range: it reads K and V once each
    alg = {"score_pass1": 2 * kb + b * hq * w.window * d * 2 + b * hk * n * 4,
           "score_pass2": kb + b * hq * w.window * d * 2 + b * hk * n * 4,
           "topk": b * hk * (n + w.budget) * 4,
           "compact": 4 * b * hk * w.budget * d * 2 + b * hk * w.budget * 12}
    e0 = ev()
    for _ in range(4 * steps):
        step()
    e1 = ev()
    torch.cuda.synchronize()
    out = {"workload": w.name + " (one layer)", "us_per_layer": sum(t.values()) * 1e3,
           "back_to_back_us": e0.elapsed_time(e1) * 1e3 / (4 * steps),
           "tokens_per_s": b * n / (sum(t.values()) * 1e-3), "kernels": {}}
    for name in t:
        gbs = alg[name] / (t[name] * 1e-3) / 1e9
        out["kernels"][name] = {"us": t[name] * 1e3, "alg_bytes": alg[name], "GBps": gbs,
                                "hbm_frac": gbs / HBM_PEAK_GBS}
    return out


def cpu_baseline(w, inputs):
    """The float64 oracle, as it stands, on the host cores: the same step (scores, selection,
    compaction of one layer), repeated for about ten seconds."""
    import numpy as np
    import oracle
    Q, K, V = inputs
    log("timing the CPU oracle on", w.name)
    cfg = oracle.Config(window=w.window, budget=w.budget, recent=w.recent)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or time.perf_counter() - t0 < 10.0:
        S = oracle.prefill_scores(Q, K, V, cfg)
        idx = oracle.select_topk(S, w.budget, w.recent)
        oracle.compact_kv(K64, V64, S, idx, slots=w.budget + 1)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    cores = min(oracle.num_threads(), w.batch * w.n_kv_heads)
    return {"value": dt * 1e6, "unit": "us/layer", "cores": cores, "kind": "oracle",
            "sample": "the whole step (1 layer, all 8 KV heads; OpenMP over (batch, KV head)), mean of %d runs" % reps,
            "tokens_per_s": w.batch * w.seq_len / dt}


if __name__ == "__main__":
    main()
