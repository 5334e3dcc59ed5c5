#!/usr/bin/env python3
"""Benchmark of the SABlock compression hot path on one MI355X.

A step is one pass of the whole path (score, refine, search_blocks + select in
their one-call form, compact: four C-ABI calls) over every layer of one synthetic workload whose
Q/K/V already sit in HBM.  Prints ONE JSON line:
  value     tokens/s per layer = n_seq * L * n_layers / step time
  roofline  the scoring step (the kernels that stream K): algorithmic bytes per
            step / their HIP-event time per step inside the timed region, against
            the 8 TB/s HBM peak
  stages_ms per-call breakdown from a second loop (events after every call)
  cpu_baseline  the fp64 oracle timed on the host on a bounded sample
"""

from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM traffic of the scoring kernels per step (bytes) from two rocprofv3 --pmc runs, FETCH_SIZE then WRITE_SIZE,
# each scaled by what the counter reads for a plain copy of known size
# (profiles/score_mfma_llama8b_128k_hbm_traffic.md); None for workloads that were not measured.
MEASURED_TRAFFIC = {"llama8b_128k": 17.60e9}


def algorithmic_bytes(w, budget, append_window=True):
    """Bytes the method must move per step (all layers), per stage."""
    elt = 4 if w.dtype == "f32" else 2
    n, nl, Hkv, Hq, L, T, W, D = w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.seq_len, w.T, w.window, w.head_dim
    P = n * nl * Hkv
    rows = budget + (W if append_window else 0)
    return {
        "score": P * L * D * elt + n * nl * Hq * W * D * elt + 2 * 4 * P * L,
        "refine": 3 * 4 * P * T,
        "search": 4 * P * T,
        "select": 4 * P * budget,
        "compact": 2 * 2 * P * rows * D * elt,
    }


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, q, k, v, off, ptr, budget, n_layers_sample, threads):
    """Time the fp64 oracle (all five steps) on `n_layers_sample` layers of sequence 0."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import gpu_helpers as H

    oracle.build()
    so = off[ptr[0]:ptr[1]]
    jobs = []
    for layer in range(n_layers_sample):
        for h in range(w.n_kv_heads):
            jobs.append((H.to_np(q[0, layer, h * w.G:(h + 1) * w.G]), H.to_np(k[0, layer, h]), H.to_np(v[0, layer, h])))

    def one(job):
        qraw, kraw, vraw = job          # raw bits as the kernels saw them; widened to fp64 inside the timed region
        return oracle.pipeline_head(H.widen(qraw), H.widen(kraw), None, so, w.cand, budget, w.eps, w.alpha, w.eta,
                                    w.tau, k_raw=kraw, v_raw=vraw)["n_sel"]

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, jobs))
    dt = time.perf_counter() - t0
    return {
        "value": w.seq_len * n_layers_sample / dt,
        "unit": "tokens/s per layer",
        "cores": min(threads, len(jobs)),
        "host_cpus": os.cpu_count(),
        "cpu_model": _cpu_model(),
        "kind": "oracle",
        "sample": f"{n_layers_sample} of {w.n_layers} layers of sequence 0 ({len(jobs)} KV-head problems, "
                  f"full L={w.seq_len}), all five steps, {dt:.2f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--budget-index", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count (profiling runs only)")
    ap.add_argument("--cpu-layers", type=int, default=4, help="layers of the oracle sample (0: skip)")
    ap.add_argument("--cpu-threads", type=int, default=8)
    ap.add_argument("--no-row-lse", action="store_true",
                    help="skip the extra timing of scoring when it is handed the rows' log-sum-exp")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the timed steps and the stage breakdown (profiling runs: keeps the other entries' "
                         "launches of the same kernels out of the per-kernel averages)")
    ap.add_argument("--layer-by-layer-only", action="store_true",
                    help="only the per-layer calls on one stream (profiling runs: the kernels of that mode alone)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="first run a plain device copy of this many MiB (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_22556_amd import binding as B
    from paper_2510_22556_amd import synth

    B.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    if args.layers > 0:
        import dataclasses
        w = dataclasses.replace(w, n_layers=args.layers, name=f"{w.name}[{args.layers} layers]")
    budget = w.budget(args.budget_index)
    q, k, v = synth.device_tensors(w, dev)
    off, ptr = synth.workload_segments(w)
    shape = B.make_shape(q, k, v)
    seg = B.make_segments(off, ptr, dev)
    buf = B.Buffers(shape, seg, budget, dev, append_window=True)
    torch.cuda.synchronize()

    if args.calibrate_copy > 0:
        src = torch.empty((args.calibrate_copy << 20,), dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # elementwise copy kernel: reads and writes calibrate_copy MiB each
        torch.cuda.synchronize()
        del src, dst
    names = ["score", "refine", "search_select", "compact"]

    if args.layer_by_layer_only:
        shape_l = B.make_shape(q[:, :1], k[:, :1], v[:, :1])
        buf_l = B.Buffers(shape_l, seg, budget, dev, append_window=True)

        def layer_calls_only():
            for l in range(w.n_layers):
                ql, kl, vl = q[:, l:l + 1], k[:, l:l + 1], v[:, l:l + 1]
                B.sablock_score(shape_l, ql, kl, buf_l.s, buf_l.ent, buf_l.ws, w.eps)
                B.sablock_refine(shape_l, buf_l.s, buf_l.ent, seg, buf_l.s_tilde, buf_l.ws, w.alpha, w.eta, buf_l.omega)
                B.sablock_search_select(shape_l, buf_l.s_tilde, seg, w.cand, budget, w.tau, buf_l.seg_budget,
                                        buf_l.block_size, buf_l.idx, buf_l.n_sel, buf_l.ws, topb_out=buf_l.topb)
                B.sablock_compact(shape_l, kl, vl, buf_l.idx, buf_l.n_sel, budget, True, buf_l.k_out, buf_l.v_out)

        for _ in range(args.warmup):
            layer_calls_only()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            layer_calls_only()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"workload": w.name, "layer_by_layer": {"ms_per_step": dt * 1e3, "ms_per_layer": dt * 1e3 / w.n_layers,
                                                                 "value": w.n_seq * w.seq_len * w.n_layers / dt}}))
        return

    def step(events=None, score_only_events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        if score_only_events is not None:
            score_only_events[0].record()
        B.sablock_score(shape, q, k, buf.s, buf.ent, buf.ws, w.eps)
        if score_only_events is not None:
            score_only_events[1].record()
        mark(1)
        B.sablock_refine(shape, buf.s, buf.ent, seg, buf.s_tilde, buf.ws, w.alpha, w.eta, buf.omega)
        mark(2)
        B.sablock_search_select(shape, buf.s_tilde, seg, w.cand, budget, w.tau, buf.seg_budget, buf.block_size,
                                buf.idx, buf.n_sel, buf.ws, topb_out=buf.topb)
        mark(3)
        B.sablock_compact(shape, k, v, buf.idx, buf.n_sel, budget, True, buf.k_out, buf.v_out)
        mark(4)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly `steps` steps; the only events inside it bracket the scoring step (the kernels
    # that the roofline entry is about), on the stream the kernels are launched on
    sev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(score_only_events=sev[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    score_ms = sum(e[0].elapsed_time(e[1]) for e in sev) / args.steps
    # per-stage breakdown from a second, untimed loop with an event after every call (the extra events cost a
    # few per cent, so they stay out of the timed region)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    stage_ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(names)}
    per_step = sorted(e[0].elapsed_time(e[4]) for e in evs)      # whole steps of that second loop, by their events
    score_per_step = sorted(e[0].elapsed_time(e[1]) for e in sev)

    alg = algorithmic_bytes(w, budget)
    score_gbs = alg["score"] / (score_ms * 1e-3) / 1e9
    result = {
        "metric": "compressed context tokens/sec per layer (score+select+compact); % HBM roofline",
        "value": w.n_seq * w.seq_len * w.n_layers / (dt / args.steps),
        "unit": "tokens/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n_seq": w.n_seq, "n_layers": w.n_layers, "seq_len": w.seq_len,
                   "window": w.window, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "cand": list(w.cand), "cache_budget": w.cache_budgets[args.budget_index],
                   "budget_B": budget, "segments": int(seg.max_segments)},
        "end_to_end": {"algorithmic_GB": sum(alg.values()) / 1e9,
                       "GBps": sum(alg.values()) / (dt / args.steps) / 1e9,
                       "frac_hbm_peak": sum(alg.values()) / (dt / args.steps) / 1e9 / HBM_PEAK_GBS},
        "stages_ms": stage_ms,
        "step_events_ms": {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]},
        "score_events_ms": {"median": score_per_step[len(score_per_step) // 2], "min": score_per_step[0],
                            "max": score_per_step[-1]},
        "roofline": {"kernel": "sablock_score (all kernels of the scoring step: row statistics + column pass)",
                     "bound": "hbm", "achieved": score_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": score_gbs / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get(w.name),
                     "algorithmic_bytes": alg["score"], "ms": score_ms},
    }
    if args.headline_only:
        print(json.dumps(result))
        return
    # the same work issued layer by layer, the way a prefill loop would call it: n_layers x 4 calls on per-layer
    # views (outputs of all layers land in one per-layer set of buffers, which is enough for timing)
    if w.n_layers > 1:
        shape_l = B.make_shape(q[:, :1], k[:, :1], v[:, :1])
        buf_l = B.Buffers(shape_l, seg, budget, dev, append_window=True)

        def layer_calls():
            for l in range(w.n_layers):
                ql, kl, vl = q[:, l:l + 1], k[:, l:l + 1], v[:, l:l + 1]
                B.sablock_score(shape_l, ql, kl, buf_l.s, buf_l.ent, buf_l.ws, w.eps)
                B.sablock_refine(shape_l, buf_l.s, buf_l.ent, seg, buf_l.s_tilde, buf_l.ws, w.alpha, w.eta, buf_l.omega)
                B.sablock_search_select(shape_l, buf_l.s_tilde, seg, w.cand, budget, w.tau, buf_l.seg_budget,
                                        buf_l.block_size, buf_l.idx, buf_l.n_sel, buf_l.ws, topb_out=buf_l.topb)
                B.sablock_compact(shape_l, kl, vl, buf_l.idx, buf_l.n_sel, budget, True, buf_l.k_out, buf_l.v_out)

        layer_calls()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(5):
            layer_calls()
        torch.cuda.synchronize()
        dt3 = (time.perf_counter() - t3) / 5
        result["layer_by_layer"] = {"ms_per_step": dt3 * 1e3, "ms_per_layer": dt3 * 1e3 / w.n_layers,
                                    "value": w.n_seq * w.seq_len * w.n_layers / dt3}
        del buf_l
        # the same calls with the layers dealt out to three streams, each with its own buffers: a layer's small
        # selection kernels (latency bound, few workgroups) then run beside the next layers' scoring, the way a
        # prefill loop can overlap a layer's compression with the next layer's forward pass
        n_str = 3
        streams = [torch.cuda.Stream() for _ in range(n_str)]
        bufs = [B.Buffers(shape_l, seg, budget, dev, append_window=True) for _ in range(n_str)]

        def layer_calls_streams():
            for l in range(w.n_layers):
                st, bl = streams[l % n_str], bufs[l % n_str]
                ql, kl, vl = q[:, l:l + 1], k[:, l:l + 1], v[:, l:l + 1]
                B.sablock_score(shape_l, ql, kl, bl.s, bl.ent, bl.ws, w.eps, stream=st)
                B.sablock_refine(shape_l, bl.s, bl.ent, seg, bl.s_tilde, bl.ws, w.alpha, w.eta, bl.omega, stream=st)
                B.sablock_search_select(shape_l, bl.s_tilde, seg, w.cand, budget, w.tau, bl.seg_budget,
                                        bl.block_size, bl.idx, bl.n_sel, bl.ws, stream=st, topb_out=bl.topb)
                B.sablock_compact(shape_l, kl, vl, bl.idx, bl.n_sel, budget, True, bl.k_out, bl.v_out, stream=st)

        torch.cuda.synchronize()
        layer_calls_streams()
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        for _ in range(5):
            layer_calls_streams()
        torch.cuda.synchronize()
        dt4 = (time.perf_counter() - t4) / 5
        result["layer_by_layer"]["three_streams"] = {"ms_per_step": dt4 * 1e3, "ms_per_layer": dt4 * 1e3 / w.n_layers,
                                                    "value": w.n_seq * w.seq_len * w.n_layers / dt4}
        del bufs, streams
    # a plain device copy on the same box as a second yardstick (reads and writes 1 GiB each)
    src = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    result["device_copy_GBps"] = copy_gbs
    result["roofline"]["frac_of_device_copy"] = score_gbs / copy_gbs
    # the step in front of the path: punctuation-based segmentation of the prompt on the device (once per
    # prompt, shared by all layers; both calls plus the read-back of the counts between them)
    tok = torch.as_tensor(synth.token_ids(w.seed(0, 0), w.n_seq, w.T, w.seg_means[0])).to(dev)
    B.segment(tok, synth.DELIMS)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        sg = B.segment(tok, synth.DELIMS)
    torch.cuda.synchronize()
    seg_ms = (time.perf_counter() - t1) / 5 * 1e3
    result["segmentation"] = {"ms_per_prompt": seg_ms, "tokens": w.n_seq * w.T, "segments": int(sg.max_segments),
                              "tokens_per_s": w.n_seq * w.T / (seg_ms * 1e-3)}
    # the step behind the path: one decode step (one new token per layer) over the full cache and over the cache
    # the path just wrote (the comparison behind the paper's decoding-latency figures, attention only)
    qn = synth.normal_torch(w.seed(0, 0), synth.STREAM_Q, (w.n_seq, w.n_layers, w.n_q_heads, w.head_dim), dev,
                            q.dtype, start=1 << 40)
    rows = budget + w.window
    kc = buf.k_out.view(w.n_seq, w.n_layers, w.n_kv_heads, rows, w.head_dim)
    vc = buf.v_out.view(w.n_seq, w.n_layers, w.n_kv_heads, rows, w.head_dim)
    dec = {}
    elt = 4 if w.dtype == "f32" else 2
    for name, (kk, vv, ns_, bb) in {"full_cache": (k, v, None, 0), "compacted_cache": (kc, vc, buf.n_sel, budget)}.items():
        cs = B.make_cache_shape(qn, kk, vv)
        dws = torch.empty((B.sablock_decode_workspace_bytes(cs),), dtype=torch.uint8, device=dev)
        dout = torch.empty(qn.shape, dtype=torch.float32, device=dev)
        B.sablock_decode_attention(cs, qn, kk, vv, dout, dws, n_sel=ns_, budget=bb)
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(5):
            B.sablock_decode_attention(cs, qn, kk, vv, dout, dws, n_sel=ns_, budget=bb)
        d1.record()
        torch.cuda.synchronize()
        ms = d0.elapsed_time(d1) / 5
        nbytes = 2 * w.n_seq * w.n_layers * w.n_kv_heads * kk.shape[3] * w.head_dim * elt
        dec[name] = {"rows": int(kk.shape[3]), "ms_per_token": ms, "GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    dec["speedup"] = dec["full_cache"]["ms_per_token"] / dec["compacted_cache"]["ms_per_token"]
    dec["cache_bytes_ratio"] = rows / w.seq_len
    result["decode_attention"] = dec
    # the head mean taken literally (one score row per layer): scoring alone, for comparison with the per-KV-head step
    try:
        aws = torch.empty((B.sablock_score_all_heads_workspace_bytes(shape),), dtype=torch.uint8, device=dev)
        s_l = torch.empty((w.n_seq * w.n_layers, w.seq_len), dtype=torch.float32, device=dev)
        e_l = torch.empty_like(s_l)
        B.sablock_score_all_heads(shape, q, k, s_l, e_l, aws, w.eps)
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        for _ in range(5):
            B.sablock_score_all_heads(shape, q, k, s_l, e_l, aws, w.eps)
        a1.record()
        torch.cuda.synchronize()
        result["score_all_heads"] = {"ms": a0.elapsed_time(a1) / 5, "workspace_GB": aws.numel() / 1e9}
        del aws, s_l, e_l
    except B.SablockError as ex:
        result["score_all_heads"] = {"unsupported": str(ex)}
    if not args.no_row_lse:
        # The path handed the rows' log-sum-exp, which a prefill attention kernel has anyway (single pass over K).
        # Where the shape allows it the values come from this library's own attention of the window queries
        # (sablock_window_attention, timed below as an entry of its own), else from library calls; in both cases
        # outside the timed region of the step: they are an INPUT of the path.
        lse = torch.empty((w.n_seq, w.n_layers, w.n_q_heads, w.window), dtype=torch.float32, device=dev)
        G = w.n_q_heads // w.n_kv_heads
        try:
            wws = torch.empty((B.sablock_window_attention_workspace_bytes(shape),), dtype=torch.uint8, device=dev)
            wout = torch.empty((w.n_seq, w.n_layers, w.n_q_heads, w.window, w.head_dim), dtype=torch.float32, device=dev)
            B.sablock_window_attention(shape, q, k, v, wout, lse, wws)
            w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            w0.record()
            for _ in range(5):
                B.sablock_window_attention(shape, q, k, v, wout, lse, wws)
            w1.record()
            torch.cuda.synchronize()
            wms = w0.elapsed_time(w1) / 5
            kv_bytes = 2 * w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len * w.head_dim * elt
            result["window_attention"] = {"ms": wms, "GBps": kv_bytes / (wms * 1e-3) / 1e9,
                                          "frac_hbm_peak": kv_bytes / (wms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                          "TFLOPs": 4.0 * w.n_seq * w.n_layers * w.n_q_heads * w.window * w.seq_len
                                                    * w.head_dim / (wms * 1e-3) / 1e12}
            lse_from = "sablock_window_attention"
            del wws, wout
        except B.SablockError:
            qi = torch.arange(w.window, device=dev)[:, None]
            for b in range(w.n_seq):
                for l in range(w.n_layers):
                    for h in range(w.n_kv_heads):
                        qq = q[b, l, h * G:(h + 1) * G].reshape(G * w.window, w.head_dim).float()
                        sc = (qq @ k[b, l, h].float().T) / math.sqrt(w.head_dim)          # [G * W, seq_len]
                        tail = sc[:, w.T:].view(G, w.window, w.window)                     # causal inside the window
                        tail.masked_fill_(torch.arange(w.window, device=dev)[None, :] > qi, float("-inf"))
                        lse[b, l, h * G:(h + 1) * G] = torch.logsumexp(sc, dim=1).view(G, w.window)
            del sc, qq, tail
            lse_from = "torch.logsumexp"

        def step_lse(score_events=None):
            if score_events is not None:
                score_events[0].record()
            B.sablock_score(shape, q, k, buf.s, buf.ent, buf.ws, w.eps, row_lse=lse)
            if score_events is not None:
                score_events[1].record()
            B.sablock_refine(shape, buf.s, buf.ent, seg, buf.s_tilde, buf.ws, w.alpha, w.eta, buf.omega)
            B.sablock_search_select(shape, buf.s_tilde, seg, w.cand, budget, w.tau, buf.seg_budget, buf.block_size,
                                    buf.idx, buf.n_sel, buf.ws, topb_out=buf.topb)
            B.sablock_compact(shape, k, v, buf.idx, buf.n_sel, budget, True, buf.k_out, buf.v_out)

        for _ in range(args.warmup):
            step_lse()
        torch.cuda.synchronize()
        lev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        t2 = time.perf_counter()
        for i in range(args.steps):
            step_lse(lev[i])
        torch.cuda.synchronize()
        dt2 = (time.perf_counter() - t2) / args.steps
        ms = sum(e[0].elapsed_time(e[1]) for e in lev) / args.steps
        result["score_with_row_lse"] = {"ms": ms, "GBps": alg["score"] / (ms * 1e-3) / 1e9,
                                        "frac": alg["score"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        result["step_with_row_lse"] = {"row_lse_from": lse_from, "ms_per_step": dt2 * 1e3, "value": w.n_seq * w.seq_len * w.n_layers / dt2,
                                       "GBps": sum(alg.values()) / dt2 / 1e9,
                                       "frac_hbm_peak": sum(alg.values()) / dt2 / 1e9 / HBM_PEAK_GBS}
    if args.cpu_layers > 0:
        result["cpu_baseline"] = cpu_baseline(w, q, k, v, off, ptr, budget, min(args.cpu_layers, w.n_layers),
                                              args.cpu_threads)
        # the oracle on ONE thread on the two small configurations (whole workload each), for scale
        single = {}
        for name in ("tiny", "llama8b_8k"):
            ws_ = synth.WORKLOADS[name]
            qs, ks_, vs = synth.device_tensors(ws_, dev)
            offs, ptrs = synth.workload_segments(ws_)
            r = cpu_baseline(ws_, qs, ks_, vs, offs, ptrs, ws_.budget(), ws_.n_layers, 1)
            single[name] = {"value": r["value"], "unit": r["unit"], "sample": r["sample"]}
        result["cpu_baseline"]["single_thread"] = single
    print(json.dumps(result))


if __name__ == "__main__":
    main()
