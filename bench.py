#!/usr/bin/env python3
"""Benchmark of the SABlock compression hot path on one MI355X.

A step is one pass of the whole path (score, refine, search_blocks + select in
their one-call form, compact: four C-ABI calls) over every layer of one synthetic workload whose
Q/K/V already sit in HBM.  Prints ONE JSON line:
  value     tokens/s per layer = n_seq * L * n_layers / step time, headline workload llama8b_128k
            (the configuration the target is quoted on), the path standing alone (it computes the
            rows' softmax denominators itself: two passes over K)
  roofline  the scoring step (the kernels that stream K): algorithmic bytes per
            step / their HIP-event time per step inside the timed region, against
            the 8 TB/s HBM peak; `traffic` from rocprofv3 counters where a committed
            summary under profiles/ holds them (named in `traffic_source`), else null
  stages_ms per-call breakdown from a second loop (events after every call)
  configs   every other configuration (and the paper's own settings) in both modes:
            standalone, and with the rows' log-sum-exp handed over as an input
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
FP32_VALU_PEAK_TFLOPS = 157.3   # MI355X fp32 vector peak, published (the generic kernels' arithmetic)

# HBM traffic of the scoring kernels per step (bytes) from two rocprofv3 --pmc runs, FETCH_SIZE then WRITE_SIZE,
# each scaled by what the counter reads for a plain copy of known size; the summary that holds the counter rows
# is named next to the figure.  Workloads without an entry report null.
MEASURED_TRAFFIC = {
    "llama8b_128k": (17.60e9, "profiles/score_mfma_llama8b_128k_hbm_traffic.md"),
    "llama8b_4x64k": (35.33e9, "profiles/score_mfma_llama8b_4x64k_hbm_traffic.md"),
    "llama8b_32k_heavy": (4.506e9, "profiles/score_mfma_llama8b_32k_heavy_hbm_traffic.md"),
}


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


def score_flops(w, passes):
    """Multiply-adds of the window-query x key contraction, as flops, per step."""
    return passes * 2.0 * w.n_seq * w.n_layers * w.n_q_heads * w.window * w.seq_len * w.head_dim


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


class Path:
    """One workload resident in HBM with the buffers of its step; `step()` enqueues the four calls."""

    def __init__(self, torch, B, synth, w, budget_index, dev):
        self.torch, self.B, self.w = torch, B, w
        self.budget = w.budget(budget_index)
        self.cache_budget = w.cache_budgets[budget_index]
        self.q, self.k, self.v = synth.device_tensors(w, dev)
        self.off, self.ptr = synth.workload_segments(w)
        self.shape = B.make_shape(self.q, self.k, self.v)
        self.seg = B.make_segments(self.off, self.ptr, dev)
        self.buf = B.Buffers(self.shape, self.seg, self.budget, dev, append_window=True)
        self.dev = dev
        self.lse = None
        self.lse_from = None

    def set_budget(self, budget_index):
        self.budget = self.w.budget(budget_index)
        self.cache_budget = self.w.cache_budgets[budget_index]
        self.buf = None
        self.buf = self.B.Buffers(self.shape, self.seg, self.budget, self.dev, append_window=True)

    def step(self, events=None, score_events=None, row_lse=None):
        B, w, buf, shape = self.B, self.w, self.buf, self.shape

        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        if score_events is not None:
            score_events[0].record()
        B.sablock_score(shape, self.q, self.k, buf.s, buf.ent, buf.ws, w.eps, row_lse=row_lse)
        if score_events is not None:
            score_events[1].record()
        mark(1)
        B.sablock_refine(shape, buf.s, buf.ent, self.seg, buf.s_tilde, buf.ws, w.alpha, w.eta, buf.omega)
        mark(2)
        B.sablock_search_select(shape, buf.s_tilde, self.seg, w.cand, self.budget, w.tau, buf.seg_budget,
                                buf.block_size, buf.idx, buf.n_sel, buf.ws, topb_out=buf.topb)
        mark(3)
        B.sablock_compact(shape, self.k, self.v, buf.idx, buf.n_sel, self.budget, True, buf.k_out, buf.v_out)
        mark(4)

    def timed(self, steps, warmup, row_lse=None):
        """`warmup` untimed steps, then exactly `steps` steps between two synchronisations; the only events inside
        the timed region bracket the scoring call, on the stream the kernels are launched on.
        Returns (seconds per step, scoring ms per step, sorted scoring ms of the steps)."""
        torch = self.torch
        for _ in range(warmup):
            self.step(row_lse=row_lse)
        torch.cuda.synchronize()
        sev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(score_events=sev[i], row_lse=row_lse)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        per = sorted(e[0].elapsed_time(e[1]) for e in sev)
        return dt, sum(per) / steps, per

    def row_lse(self):
        """The rows' log-sum-exp, an INPUT of the path in its second mode: from this library's own attention of the
        window queries where the shape allows it (also timed, as an entry of its own), else from library calls."""
        torch, B, w = self.torch, self.B, self.w
        if self.lse is not None:
            return self.lse, self.lse_from, None
        dev = self.dev
        lse = torch.empty((w.n_seq, w.n_layers, w.n_q_heads, w.window), dtype=torch.float32, device=dev)
        G = w.n_q_heads // w.n_kv_heads
        info = None
        try:
            wws = torch.empty((B.sablock_window_attention_workspace_bytes(self.shape),), dtype=torch.uint8, device=dev)
            wout = torch.empty((w.n_seq, w.n_layers, w.n_q_heads, w.window, w.head_dim), dtype=torch.float32, device=dev)
            B.sablock_window_attention(self.shape, self.q, self.k, self.v, wout, lse, wws)
            w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            w0.record()
            for _ in range(5):
                B.sablock_window_attention(self.shape, self.q, self.k, self.v, wout, lse, wws)
            w1.record()
            torch.cuda.synchronize()
            wms = w0.elapsed_time(w1) / 5
            elt = 4 if w.dtype == "f32" else 2
            kv_bytes = 2 * w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len * w.head_dim * elt
            info = {"ms": wms, "GBps": kv_bytes / (wms * 1e-3) / 1e9,
                    "frac_hbm_peak": kv_bytes / (wms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "TFLOPs": 2 * score_flops(w, 1) / (wms * 1e-3) / 1e12,
                    "frac_mfma_peak": 2 * score_flops(w, 1) / (wms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
            self.lse_from = "sablock_window_attention"
            del wws, wout
        except B.SablockError:
            qi = torch.arange(w.window, device=dev)[:, None]
            for b in range(w.n_seq):
                for l in range(w.n_layers):
                    for h in range(w.n_kv_heads):
                        qq = self.q[b, l, h * G:(h + 1) * G].reshape(G * w.window, w.head_dim).float()
                        sc = (qq @ self.k[b, l, h].float().T) / math.sqrt(w.head_dim)          # [G * W, seq_len]
                        tail = sc[:, w.T:].view(G, w.window, w.window)                          # causal inside the window
                        tail.masked_fill_(torch.arange(w.window, device=dev)[None, :] > qi, float("-inf"))
                        lse[b, l, h * G:(h + 1) * G] = torch.logsumexp(sc, dim=1).view(G, w.window)
            self.lse_from = "torch.logsumexp"
        self.lse = lse
        return lse, self.lse_from, info


def mode_entry(w, alg, dt, score_ms, passes):
    """Figures of one mode of one configuration: the step, the scoring call, both rooflines."""
    total = sum(alg.values())
    mfma_path = w.dtype == "bf16" and w.head_dim == 128
    peak = MFMA_BF16_PEAK_TFLOPS if mfma_path else FP32_VALU_PEAK_TFLOPS
    tflops = score_flops(w, passes) / (score_ms * 1e-3) / 1e12
    hbm_frac = alg["score"] / (score_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    # which roof is nearer: flops per algorithmic byte of the scoring step against the ridge of the two peaks
    intensity = score_flops(w, passes) / alg["score"]
    ridge = peak * 1e12 / (HBM_PEAK_GBS * 1e9)
    return {
        "ms_per_step": dt * 1e3,
        "value": w.n_seq * w.seq_len * w.n_layers / dt,
        "frac_hbm_peak": total / dt / 1e9 / HBM_PEAK_GBS,
        "score_ms": score_ms,
        "score_frac_hbm_peak": hbm_frac,
        "score_TFLOPs": tflops,
        "score_frac_compute_peak": tflops / peak,
        "compute_peak": "bf16 MFMA 2500 TFLOP/s" if mfma_path else "fp32 vector 157.3 TFLOP/s",
        "bound": ("mfma" if mfma_path else "alu") if intensity > ridge else "hbm",
        "flop_per_algorithmic_byte": intensity,
    }


def config_entries(torch, B, synth, dev, name, steps, warmup):
    """One configuration in both modes, for each of its cache budgets."""
    w = synth.WORKLOADS[name]
    path = Path(torch, B, synth, w, 0, dev)
    torch.cuda.synchronize()
    traffic, traffic_source = MEASURED_TRAFFIC.get(name, (None, None))
    out = {"score_traffic_standalone": traffic, "traffic_source": traffic_source,
           "n_seq": w.n_seq, "n_layers": w.n_layers, "seq_len": w.seq_len, "window": w.window,
           "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "dtype": w.dtype,
           "cand": list(w.cand), "K_bytes": w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len * w.head_dim
           * (4 if w.dtype == "f32" else 2),
           "cache_resident": w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len * w.head_dim * (4 if w.dtype == "f32" else 2)
           <= (256 << 20), "budgets": {}}
    lse, lse_from, wa = path.row_lse()
    out["row_lse_from"] = lse_from
    if wa is not None:
        out["window_attention"] = wa
    # small configurations finish a step in microseconds: more steps for a stable figure
    n = steps if w.n_layers * w.n_seq > 1 else max(steps, 50)
    for bi in range(len(w.cache_budgets)):
        if bi:
            path.set_budget(bi)
        alg = algorithmic_bytes(w, path.budget)
        dt, sms, _ = path.timed(n, warmup)
        dt2, sms2, _ = path.timed(n, warmup, row_lse=lse)
        out["budgets"][str(w.cache_budgets[bi])] = {
            "budget_B": path.budget, "algorithmic_GB": sum(alg.values()) / 1e9,
            "standalone": mode_entry(w, alg, dt, sms, 2),
            "with_row_lse": mode_entry(w, alg, dt2, sms2, 1),
        }
    del path
    torch.cuda.empty_cache()
    return out


def yardstick(torch, B, path, reps=10):
    """What the memory system delivers to the scoring kernels' access pattern, and whether a second read served by
    the caches is any faster: (1) the key stream alone (sablock_stream_probe) over all of K from HBM; (2) the same
    over a few problems read again and again, which stay in the memory-side cache (<= 128 MiB) or in the L2s
    (32 MiB over 8 XCDs); (3) the two scoring passes issued on groups of problems small enough for the second
    pass to find its keys in that cache, against the one call over all problems."""
    w, q, k, buf, shape = path.w, path.q, path.k, path.buf, path.shape
    sink = torch.zeros((1,), dtype=torch.int32, device=path.dev)
    elt = 2
    out = {"workload": w.name}

    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    k_bytes = w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len * w.head_dim * elt
    for read_lds, stores in ((False, False), (True, False), (True, True)):
        so, eo = (buf.s, buf.ent) if stores else (None, None)
        ms = timed(lambda: B.sablock_stream_probe(shape, k, sink, read_lds, so, eo), reps)
        out["stream_all_K" + ("_with_lds_reads" if read_lds else "") + ("_and_score_stores" if stores else "")] = {
            "bytes": k_bytes + (2 * 4 * w.n_seq * w.n_layers * w.n_kv_heads * w.seq_len if stores else 0),
            "ms": ms, "TBps_of_K": k_bytes / (ms * 1e-3) / 1e12}
    G = w.n_q_heads // w.n_kv_heads
    # launches of n problems each: the same n problems again and again (their keys stay in the memory-side cache
    # when n * 32 MiB fits it, in the L2s at 32 MiB) against launches that walk through all of K (every launch
    # reads keys that were last touched 8 GiB ago, i.e. from HBM); same launch size, so the launch overhead cancels
    out["stream_groups"] = {}
    for n in (1, 2, 4, 8):
        if n > w.n_kv_heads or w.n_kv_heads % n:
            continue
        nbytes = n * w.seq_len * w.head_dim * elt
        views = [(B.make_shape(q[b:b + 1, l:l + 1, h0 * G:(h0 + n) * G], k[b:b + 1, l:l + 1, h0:h0 + n]),
                  k[b:b + 1, l:l + 1, h0:h0 + n])
                 for b in range(w.n_seq) for l in range(w.n_layers) for h0 in range(0, w.n_kv_heads, n)]
        sg, kg = views[0]
        ms_same = timed(lambda: B.sablock_stream_probe(sg, kg, sink, False), 64)

        def walk():
            for sh_, k_ in views:
                B.sablock_stream_probe(sh_, k_, sink, False)
        ms_walk = timed(walk, 2) / len(views)
        out["stream_groups"][f"{n}_problems_{nbytes >> 20}_MiB"] = {
            "bytes": nbytes, "same_keys_ms": ms_same, "same_keys_TBps": nbytes / (ms_same * 1e-3) / 1e12,
            "walking_all_K_ms": ms_walk, "walking_all_K_TBps": nbytes / (ms_walk * 1e-3) / 1e12}
    # the two scoring passes, whole call against groups of n problems (a group's second pass starts right after its
    # first, so its keys are the most recently used bytes of the memory-side cache)
    ms_all = timed(lambda: B.sablock_score(shape, q, k, buf.s, buf.ent, buf.ws, w.eps), reps)
    out["score_two_passes"] = {"one_call_all_problems_ms": ms_all, "groups": {}}
    if G == 4 and w.window == 32:
        # the statistics pass by the other kernel design (a lane per window query, four wavefronts per SIMD sharing
        # the key tiles through a workgroup-wide ring) instead of a lane per key with a private ring per wavefront
        shape_rows = B.make_shape(q, k, stats_per_key=2)
        ws_rows = torch.empty((B.sablock_workspace_bytes(shape_rows, 0, 0),), dtype=torch.uint8, device=path.dev)
        out["score_two_passes"]["statistics_by_window_query_kernel_ms"] = timed(
            lambda: B.sablock_score(shape_rows, q, k, buf.s, buf.ent, ws_rows, w.eps), reps)
    for n in (2, 4, 8):
        if w.n_kv_heads % n:
            continue
        calls = []
        for b in range(w.n_seq):
            for l in range(w.n_layers):
                for h0 in range(0, w.n_kv_heads, n):
                    qg, kg = q[b:b + 1, l:l + 1, h0 * G:(h0 + n) * G], k[b:b + 1, l:l + 1, h0:h0 + n]
                    p0 = (b * w.n_layers + l) * w.n_kv_heads + h0
                    calls.append((B.make_shape(qg, kg), qg, kg, buf.s[p0:p0 + n], buf.ent[p0:p0 + n]))

        def groups():
            for sg, qg, kg, so, eo in calls:
                B.sablock_score(sg, qg, kg, so, eo, buf.ws, w.eps)
        ms = timed(groups, 3)
        out["score_two_passes"]["groups"][f"{n}_problems_{(n * w.seq_len * w.head_dim * elt) >> 20}_MiB"] = {
            "calls": len(calls), "ms": ms}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--budget-index", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count (profiling runs only)")
    ap.add_argument("--cpu-layers", type=int, default=4, help="layers of the oracle sample (0: skip)")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the oracle sample (0: every host CPU)")
    ap.add_argument("--no-row-lse", action="store_true",
                    help="skip the extra timing of scoring when it is handed the rows' log-sum-exp")
    ap.add_argument("--row-lse-only", action="store_true",
                    help="only the steps that are handed the rows' log-sum-exp (profiling runs of that mode)")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the timed steps and the stage breakdown (profiling runs: keeps the other entries' "
                         "launches of the same kernels out of the per-kernel averages)")
    ap.add_argument("--layer-by-layer-only", action="store_true",
                    help="only the per-layer calls on one stream (profiling runs: the kernels of that mode alone)")
    ap.add_argument("--yardstick", action="store_true",
                    help="only the memory-system yardsticks of the scoring kernels (key stream alone, cache-resident "
                         "groups, scoring on cache-sized groups of problems)")
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
    path = Path(torch, B, synth, w, args.budget_index, dev)
    budget, q, k, v, seg, shape, buf = path.budget, path.q, path.k, path.v, path.seg, path.shape, path.buf
    off, ptr = path.off, path.ptr
    torch.cuda.synchronize()

    if args.calibrate_copy > 0:
        src = torch.empty((args.calibrate_copy << 20,), dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # elementwise copy kernel: reads and writes calibrate_copy MiB each
        torch.cuda.synchronize()
        del src, dst
    names = ["score", "refine", "search_select", "compact"]

    if args.yardstick:
        print(json.dumps(yardstick(torch, B, path)))
        return

    if args.row_lse_only:
        lse, lse_from, _ = path.row_lse()
        dt2, sms2, _ = path.timed(args.steps, args.warmup, row_lse=lse)
        print(json.dumps({"workload": w.name, "step_with_row_lse": {"row_lse_from": lse_from, "ms_per_step": dt2 * 1e3,
                                                                    "score_ms": sms2}}))
        return

    def layer_calls(shape_l, bufs, streams=None):
        for l in range(w.n_layers):
            bl = bufs[l % len(bufs)]
            st = streams[l % len(streams)] if streams else None
            ql, kl, vl = q[:, l:l + 1], k[:, l:l + 1], v[:, l:l + 1]
            B.sablock_score(shape_l, ql, kl, bl.s, bl.ent, bl.ws, w.eps, stream=st)
            B.sablock_refine(shape_l, bl.s, bl.ent, seg, bl.s_tilde, bl.ws, w.alpha, w.eta, bl.omega, stream=st)
            B.sablock_search_select(shape_l, bl.s_tilde, seg, w.cand, budget, w.tau, bl.seg_budget, bl.block_size,
                                    bl.idx, bl.n_sel, bl.ws, stream=st, topb_out=bl.topb)
            B.sablock_compact(shape_l, kl, vl, bl.idx, bl.n_sel, budget, True, bl.k_out, bl.v_out, stream=st)

    if args.layer_by_layer_only:
        shape_l = B.make_shape(q[:, :1], k[:, :1], v[:, :1])
        buf_l = [B.Buffers(shape_l, seg, budget, dev, append_window=True)]
        for _ in range(args.warmup):
            layer_calls(shape_l, buf_l)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            layer_calls(shape_l, buf_l)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"workload": w.name, "layer_by_layer": {"ms_per_step": dt * 1e3, "ms_per_layer": dt * 1e3 / w.n_layers,
                                                                 "value": w.n_seq * w.seq_len * w.n_layers / dt}}))
        return

    # the timed region: exactly `steps` steps (see Path.timed)
    dt_step, score_ms, score_per_step = path.timed(args.steps, args.warmup)
    ms_per_step = dt_step * 1e3
    # per-stage breakdown from a second, untimed loop with an event after every call (the extra events cost a
    # few per cent, so they stay out of the timed region)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for i in range(args.steps):
        path.step(evs[i])
    torch.cuda.synchronize()
    stage_ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(names)}
    per_step = sorted(e[0].elapsed_time(e[4]) for e in evs)      # whole steps of that second loop, by their events

    alg = algorithmic_bytes(w, budget)
    score_gbs = alg["score"] / (score_ms * 1e-3) / 1e9
    head = mode_entry(w, alg, dt_step, score_ms, 2)
    traffic, traffic_source = MEASURED_TRAFFIC.get(w.name, (None, None))
    result = {
        "metric": "compressed context tokens/sec per layer (score+select+compact); % HBM roofline",
        "value": w.n_seq * w.seq_len * w.n_layers / dt_step,
        "unit": "tokens/s per layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n_seq": w.n_seq, "n_layers": w.n_layers, "seq_len": w.seq_len,
                   "window": w.window, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "cand": list(w.cand), "cache_budget": path.cache_budget,
                   "budget_B": budget, "segments": int(seg.max_segments),
                   "mode": "standalone: the path computes the rows' softmax denominators itself (two passes over K)"},
        "end_to_end": {"algorithmic_GB": sum(alg.values()) / 1e9,
                       "GBps": sum(alg.values()) / dt_step / 1e9,
                       "frac_hbm_peak": sum(alg.values()) / dt_step / 1e9 / HBM_PEAK_GBS},
        "stages_ms": stage_ms,
        "step_events_ms": {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]},
        "score_events_ms": {"median": score_per_step[len(score_per_step) // 2], "min": score_per_step[0],
                            "max": score_per_step[-1]},
        "roofline": {"kernel": "sablock_score (all kernels of the scoring step: row statistics + column pass)",
                     "bound": head["bound"], "achieved": score_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": score_gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": alg["score"], "ms": score_ms,
                     "TFLOPs": head["score_TFLOPs"], "frac_mfma_peak": head["score_frac_compute_peak"],
                     "flop_per_algorithmic_byte": head["flop_per_algorithmic_byte"]},
    }
    if args.headline_only:
        print(json.dumps(result))
        return
    # the same work issued layer by layer, the way a prefill loop would call it: n_layers x 4 calls on per-layer
    # views (outputs of all layers land in one per-layer set of buffers, which is enough for timing)
    if w.n_layers > 1:
        shape_l = B.make_shape(q[:, :1], k[:, :1], v[:, :1])
        buf_l = [B.Buffers(shape_l, seg, budget, dev, append_window=True)]
        layer_calls(shape_l, buf_l)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(5):
            layer_calls(shape_l, buf_l)
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
        torch.cuda.synchronize()
        layer_calls(shape_l, bufs, streams)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        for _ in range(5):
            layer_calls(shape_l, bufs, streams)
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
        # The values are an INPUT of the path in this mode: their producer's time (the `window_attention` entry
        # when it is this library's own kernel) is NOT inside `step_with_row_lse`.
        lse, lse_from, wa = path.row_lse()
        if wa is not None:
            result["window_attention"] = wa
        dt2, ms, _ = path.timed(args.steps, args.warmup, row_lse=lse)
        result["score_with_row_lse"] = {"ms": ms, "GBps": alg["score"] / (ms * 1e-3) / 1e9,
                                        "frac": alg["score"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        result["step_with_row_lse"] = {"row_lse_from": lse_from,
                                       "note": "row_lse is an input here: the time of its producer is outside this step",
                                       "ms_per_step": dt2 * 1e3, "value": w.n_seq * w.seq_len * w.n_layers / dt2,
                                       "GBps": sum(alg.values()) / dt2 / 1e9,
                                       "frac_hbm_peak": sum(alg.values()) / dt2 / 1e9 / HBM_PEAK_GBS}
    threads = args.cpu_threads if args.cpu_threads > 0 else (os.cpu_count() or 1)
    if args.cpu_layers > 0:
        result["cpu_baseline"] = cpu_baseline(w, q, k, v, off, ptr, budget, min(args.cpu_layers, w.n_layers), threads)
    # free the headline workload before the other configurations come in
    del path, q, k, v, buf, seg, shape, kc, vc, qn
    torch.cuda.empty_cache()
    if not args.no_configs and args.layers == 0:
        others = [n for n in ("tiny", "llama8b_8k", "llama8b_32k_heavy", "llama8b_128k", "llama8b_4x64k",
                              "paper_defaults_32k", "gqa7_32k") if n != w.name]
        result["configs"] = {n: config_entries(torch, B, synth, dev, n, max(5, args.steps // 2), args.warmup)
                             for n in others}
    if args.cpu_layers > 0:
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
