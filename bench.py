#!/usr/bin/env python3
"""Benchmark of the RefreshKV decode-attention hot path on one MI355X.

A "step" is one decode step of the whole hot path over all layers of the workload: per layer
the query-similarity bookkeeping, then either full attention + top-K selection + gather
(every S-th step) or partial attention over the small cache.  K/V are synthetic and already
resident in HBM; the rows that later steps "append" are pre-written, so a step only advances
seq_lens (the append itself is the caller's 4 KB copy, outside this library).

Prints ONE JSON line (see the keys below).  Beside the headline it carries
  roofline          achieved HBM GB/s of the dominant HBM-bound kernel (the split full-attention
                    kernel) = algorithmic bytes per launch / its average duration, measured here
                    with HIP events on the launch stream around back-to-back launches of that
                    kernel alone (rk_full_attn_scores), one per layer;
  roofline_partial  the same for the kernel of the partial step, which most of `value` is made of;
  copy_GBps         what a plain copy kernel of known size reaches in the same run (read + written
                    bytes per second): the yardstick beside the 8 TB/s peak;
  other_workloads   the other single-GPU workloads of the benchmark spec at their own layer counts, a
                    few steps each (value, roofline fraction of the first kernel of a full step,
                    full / partial ratio);
  cpu_baseline      the CPU oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_llama_32k")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = workload's)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--launch", choices=["graph", "native", "eager", "hybrid"], default="native",
                    help="native: one call of the library's step driver (rk_decode_step_batched) per step launches the "
                         "kernels of all layers back to back from C; graph: replay one HIP graph per step; hybrid: "
                         "partial steps native, full steps as a replayed HIP graph; eager: one Python call per library call")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the selection and the gather of a full step per layer on the main stream (default: see "
                         "--refresh)")
    ap.add_argument("--overlap-workspaces", type=int, default=3, help="workspaces the overlapped refresh rotates (0: one per layer)")
    ap.add_argument("--refresh", choices=["batched", "second-stream"], default="batched",
                    help="how a full step of the layer stack does its pooling, selections and gathers: all layers at once "
                         "after the last layer's attention (rk_full_attn_deferred + rk_refresh_batched), or per layer on a "
                         "second stream beside the full attention of the following layers")
    ap.add_argument("--run-ahead", type=int, default=1,
                    help="steps that may still be pending when a two-stream (full) step is submitted (-1: no limit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=4, help="layers of the oracle sample")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other workloads that the default invocation appends")
    return ap.parse_args()


def cost_model(w, lens0, eff_stride, achieved_gbps, measured_us):
    per_token = 2 * w.n_kv_heads * w.head_dim * 2
    stride = (eff_stride or {}).get("mean") or (w.stride if w.stride > 0 else float("inf"))
    rows = float(lens0.sum()) / stride + w.k_small * w.batch
    model_bytes = per_token * rows
    return {"bytes_per_step_layer": int(model_bytes), "stride": stride,
            "us_at_hbm_peak": round(model_bytes / 8000e9 * 1e6, 2),
            "us_at_achieved_rate": round(model_bytes / (achieved_gbps * 1e9) * 1e6, 2),
            "measured_us": round(measured_us, 2)}


def profile_traffic(w_name, key):
    """HBM bytes per launch of a kernel from the committed profiler summary of this workload (None if
    there is none), and where the figure comes from: it is a measurement of the commit named there,
    not of this run."""
    path = os.path.join(ROOT, "profiles", "bench_%s_pmc.json" % w_name)
    if not os.path.exists(path):
        return None, None
    with open(path) as f:
        pmc = json.load(f)
    if key not in pmc:
        return None, None
    k = pmc[key]
    traffic = int(k["fetch_kib"] * 1024 * pmc["fetch_scale"] + k["write_kib"] * 1024 * pmc["write_scale"])
    return traffic, {"file": "profiles/bench_%s_pmc.json" % w_name, "commit": pmc.get("commit"), "layers": pmc.get("layers")}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no multi-GPU part); got --gpus %d" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    result = run_workload(args, args.workload, light=False)
    if args.workload == "cfg2_llama_32k" and not args.no_other_workloads and not args.layers:
        import copy
        import gc
        import gen
        others = {}
        for name in ("cfg3_qwen_64k_dynamic", "cfg4_llama_batch16_ragged", "cfg5_llama_128k"):
            a = copy.copy(args)
            a.no_cpu_baseline = True
            a.steps, a.warmup = 4 * max(gen.WORKLOADS[name].stride, 1), max(gen.WORKLOADS[name].stride, 1)
            if gen.WORKLOADS[name].dynamic:
                a.steps, a.warmup = 60, 20          # long enough for the trigger to have fired in every layer
            gc.collect(); torch.cuda.empty_cache()      # the previous workload's caches go before the next is set up
            r = run_workload(a, name, light=True)
            others[name] = {"value": r["value"], "unit": r["unit"], "layers": r["config"]["layers"], "steps": a.steps,
                            "step_us_per_layer": r["step_us_per_layer"], "effective_stride": r["effective_stride"],
                            "full_attn_us": r["call_us_per_layer"]["full_attn"],
                            "partial_attn_us": r["call_us_per_layer"]["partial_attn"],
                            "full_over_partial": r["full_over_partial"],
                            "roofline_frac": r["roofline"]["frac"], "roofline_avg_launch_us": r["roofline"]["avg_launch_us"],
                            "roofline_traffic": r["roofline"]["traffic"], "traffic_source": r["roofline"]["traffic_source"],
                            "roofline_partial_frac": r["roofline_partial"]["frac"]}
        result["other_workloads"] = others
    print(json.dumps(result))


def run_workload(args, workload, light):
    """One workload: the timed steps, the per-kind and per-call figures, the two roofline blocks.
    light: only what `other_workloads` reports (no comparison policies, no CPU oracle)."""
    import numpy as np
    import torch
    import gen
    import paper_2411_05787_amd as rk

    dev = "cuda"
    w = gen.WORKLOADS[workload]
    n_layers = args.layers or w.n_layers
    # after the timed steps, a few more with an event pair around each give the per-kind figures: the
    # events cost about 4 us each on the stream, so the timed region itself carries none
    n_kind_steps = 3 * w.stride if w.stride > 0 else 20
    T = args.warmup + args.steps + n_kind_steps
    L0 = w.context
    # rows for every future step are pre-written: context' = L0 + T, seq_lens starts at L0
    w_alloc = gen.shrink(w, context=L0 + T + 8, n_steps=0)
    geom = rk.Geom(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.scale)
    B, Hq, Hkv, D = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim

    t_setup = time.time()
    kv = [gen.make_kv(w_alloc, l, device=dev) for l in range(n_layers)]
    cap = kv[0][0].shape[2]
    lens0 = gen.seq_lens(w)
    seq_lens = lens0.to(dev)
    wq = gen.shrink(w, n_steps=T)
    q_steps = torch.stack([gen.make_queries(wq, l) for l in range(n_layers)], dim=1).to(dev)   # [T+1, nl, B, Hq, D]
    q_cur = torch.empty(n_layers, B, Hq, D, dtype=torch.bfloat16, device=dev)
    max_len_bound = int(lens0.max()) + T + 1
    ws = rk.Workspace(geom, cap, w.k_small)
    weights = torch.empty(B, Hq, cap, dtype=torch.float32, device=dev)
    layers = [rk.RefreshKVLayer(geom, kv[l][0], kv[l][1], seq_lens, int(lens0.max()), w.k_small, w.stride,
                                pool_w=w.pool_w, dynamic=w.dynamic, threshold=w.threshold,
                                workspace=ws) for l in range(n_layers)]
    for lay in layers:
        lay.use_static_bounds(max_len_bound, max(w.stride, 1))
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    launch = "eager" if args.no_graph else args.launch
    if w.dynamic and launch in ("graph", "hybrid"):
        launch = "native"      # trigger test steps enqueue both branches; the native driver also counts refreshes
    model = None
    if launch == "native":
        model = rk.RefreshKVModel(geom, kv, seq_lens, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w,
                                  dynamic=w.dynamic, threshold=w.threshold, workspace=ws)
        if not args.no_overlap:
            if args.refresh == "batched":
                model.batched_refresh()
            else:
                model.overlap_refresh(args.overlap_workspaces)

    # hybrid: partial steps through the native driver (one foreign call, kernels launched back to back
    # from C: smaller gaps between kernels than between the nodes of a HIP graph), full steps as the
    # two-stream HIP graph.  Both act on the same per-layer state, which the native driver owns.
    partial_driver = None
    if launch == "hybrid":
        partial_driver = rk.RefreshKVModel(geom, kv, seq_lens, int(lens0.max()), w.k_small, w.stride, pool_w=w.pool_w,
                                           dynamic=False, workspace=ws)
        partial_driver.use_static_bounds(max_len_bound, max(w.stride, 1))
        for l, lay in enumerate(layers):
            lay.small_K, lay.small_V, lay.idx = partial_driver.small_K[l], partial_driver.small_V[l], partial_driver.idx[l]
            lay.tail_start, lay.out = partial_driver.tail_start[l], partial_driver.out[l]

    overlap = not args.no_overlap and model is None
    stack = rk.RefreshKVStack(layers, n_workspaces=args.overlap_workspaces, batched=args.refresh == "batched") if overlap else None

    def enqueue_step(t: int, q=None):
        """Everything of decode step t on the current stream (q_cur already holds the queries, unless
        the native driver is given the step's own queries: it takes pointers, so they need no staging)."""
        if t >= 1:
            seq_lens.add_(1)
        if model is not None:
            if t >= 1:
                model.advance()
            return model.step(t, q_cur if q is None else q)
        if partial_driver is not None and not is_full(t):
            return partial_driver.step(t, q_cur)
        if stack is not None:
            return stack.step(t, q_cur)
        kind = None
        for l, lay in enumerate(layers):
            kind = lay.step(t, q_cur[l])
        return kind

    def is_full(t):       # a step at which every layer takes a full step by schedule (the trigger's test steps are "both")
        return t == 0 or (w.stride > 0 and t % w.stride == 0 and not w.dynamic)

    # t = 0: prefill-equivalent initialisation (full step everywhere), eager
    q_cur.copy_(q_steps[0])
    enqueue_step(0)
    if model is not None:          # the per-layer objects serve the per-call timings below: initialise them too
        for l, lay in enumerate(layers):
            lay.step(0, q_cur[l])
    torch.cuda.synchronize()

    graphs = {}
    if launch in ("graph", "hybrid"):
        # capture one full-style and one partial-style step; the device-side seq_lens/tail_start
        # make a replay do the right thing at any later step.  Capturing advances seq_lens like a
        # real step would not (nothing runs during capture), so no state is disturbed.
        side = torch.cuda.Stream()
        for kind, t_like in (("partial", 1), ("full", w.stride if w.stride > 0 else 0)):
            if (kind == "full" and w.stride <= 0) or (kind == "partial" and partial_driver is not None):
                continue
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                enqueue_step(t_like)
            graphs[kind] = g
        torch.cuda.synchronize()

    def run_step(t: int):
        kind = "both" if (w.dynamic and t >= 1 and w.stride > 0 and t % w.stride == 0) else ("full" if is_full(t) else "partial")
        if model is not None:                  # pointers to the step's queries: no copy into a static buffer
            reported = enqueue_step(t, q_steps[t])
            assert reported == kind, (t, reported, kind)      # what the driver says it enqueued
            return kind
        q_cur.copy_(q_steps[t], non_blocking=True)
        if graphs and kind in graphs:
            graphs[kind].replay()
        else:
            enqueue_step(t)
        return kind

    for t in range(1, args.warmup + 1):
        run_step(t)
    torch.cuda.synchronize()

    kinds = []
    two_streams = (stack is not None and not stack.batched) or (model is not None and not args.no_overlap and args.refresh != "batched")
    done = [torch.cuda.Event() for _ in range(args.steps)] if two_streams else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # A step that uses the second stream is submitted late: the host first waits until at most
    # `--run-ahead` earlier steps are still pending.  Submitted far ahead, its second queue sits
    # blocked on a barrier behind all of them, and a blocked queue slows every dispatch of the
    # first one meanwhile (measured: +0.9 us per layer on every partial step of the period).
    t_first = args.warmup + 1
    for i, t in enumerate(range(t_first, t_first + args.steps)):
        if two_streams and args.run_ahead >= 0 and is_full(t) and i - 1 - args.run_ahead >= 0:
            done[i - 1 - args.run_ahead].synchronize()
        kinds.append(run_step(t))
        if two_streams:
            done[i].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    per_kind = {}
    for t in range(t_first + args.steps, T + 1):        # untimed: the same steps, one event pair around each
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); k = run_step(t); b.record()
        per_kind.setdefault(k, []).append((a, b))
    torch.cuda.synchronize()
    per_kind = {k: [a.elapsed_time(b) * 1e3 for a, b in v] for k, v in per_kind.items()}
    med = {k: float(np.median(v)) / n_layers for k, v in per_kind.items()}      # us per layer
    spread = {k: [round(float(np.percentile(v, q)) / n_layers, 2) for q in (10, 90)] for k, v in per_kind.items()}
    final_len = int(seq_lens.max().item())
    assert final_len == int(lens0.max()) + T, (final_len, int(lens0.max()) + T)

    # ---- per-call-class GPU time (graph of n_layers calls each), cold last-level cache ----
    def graph_us(fn, reps=3):
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            for l in range(min(2, n_layers)):
                fn(l)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for l in range(n_layers):
                fn(l)
        g.replay(); torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for _ in range(reps):
            a.record(); g.replay(); b.record(); torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / n_layers)
        return float(np.median(ts))

    out = layers[0].out
    Lb = max_len_bound
    partial_call = lambda l: rk.rk_partial_attn(geom, q_cur[l], layers[l].small_K, layers[l].small_V, w.k_small, *kv[l],
                                                layers[l].tail_start, seq_lens, max(w.stride, 1), out, workspace=ws)
    klass = {
        "full_attn": graph_us(lambda l: rk.rk_full_attn(geom, q_cur[l], *kv[l], seq_lens, Lb, out, weights=weights, workspace=ws)),
        "partial_attn": graph_us(partial_call),
    }
    if not light:
        gw = torch.Generator(device="cuda").manual_seed(4242)
        q_win = torch.randn(w.batch, 32, w.n_q_heads, w.head_dim, generator=gw, device="cuda").to(torch.bfloat16)
        q_win1 = q_win[:, -1:].contiguous()
        # the H2O comparison policy at the same budget K (K/2 recent): one state per layer, caches full
        h2o_cap = w.k_small + 1
        h2o = []
        for l in range(n_layers):
            cK = torch.randn(B, Hkv, h2o_cap, D, generator=gw, device="cuda").to(torch.bfloat16)
            cV = torch.randn(B, Hkv, h2o_cap, D, generator=gw, device="cuda").to(torch.bfloat16)
            tot = torch.rand(B, Hkv, h2o_cap, generator=gw, device="cuda")
            hpos = torch.arange(h2o_cap, dtype=torch.int32, device="cuda").expand(B, Hkv, h2o_cap).contiguous()
            n_rows = torch.full((B,), w.k_small, dtype=torch.int32, device="cuda")
            keep = (cK, cV, tot, hpos, n_rows, torch.zeros(B, dtype=torch.int32, device="cuda"))
            h2o.append((rk.h2o_state(geom, *keep), keep))
        h2o_lens = torch.full((B,), h2o_cap, dtype=torch.int32, device="cuda")
        h2o_new = torch.randn(2, B, Hkv, D, generator=gw, device="cuda").to(torch.bfloat16)

        def h2o_call(l):
            if l == 0:
                h2o_lens.add_(1)                  # one decoding step further: a new position for the new token
            rk.rk_h2o_step(geom, h2o[l][0], q_cur[l], h2o_new[0], h2o_new[1], h2o_lens, w.k_small, w.k_small // 2, out,
                           workspace=ws)

        klass.update({
            "full_attn_no_weights": graph_us(lambda l: rk.rk_full_attn(geom, q_cur[l], *kv[l], seq_lens, Lb, out, workspace=ws)),
            "h2o_step": graph_us(h2o_call),
            "full_attn_select": graph_us(lambda l: rk.rk_full_attn_select(geom, q_cur[l], *kv[l], seq_lens, Lb, out, w.k_small, w.pool_w,
                                                                           layers[l].idx, workspace=ws)),
            "score_select": graph_us(lambda l: rk.rk_score_select(geom, q_cur[l], kv[l][0], seq_lens, Lb, w.k_small, w.pool_w,
                                                                   layers[l].idx, workspace=ws)),
            # prefill-side initialisation from an observation window of 1 and of 32 prompt tokens (the queries
            # are synthetic; the window ends at the current length)
            "window_select_w1": graph_us(lambda l: rk.rk_window_select(geom, q_win1, kv[l][0], seq_lens, Lb, w.k_small, w.pool_w,
                                                                       layers[l].idx, workspace=ws)),
            "window_select_w32": graph_us(lambda l: rk.rk_window_select(geom, q_win, kv[l][0], seq_lens, Lb, w.k_small, w.pool_w,
                                                                        layers[l].idx, workspace=ws)),
            "topk_select": graph_us(lambda l: rk.rk_topk_select(geom, weights, seq_lens, Lb, w.k_small, w.pool_w, layers[l].idx, workspace=ws)),
            "gather_small_kv": graph_us(lambda l: rk.rk_gather_small_kv(geom, *kv[l], layers[l].idx, w.k_small, layers[l].small_K, layers[l].small_V)),
            "query_sim": graph_us(lambda l: rk.rk_query_sim(geom, q_cur[l], layers[l].q_ref, w.threshold, False, layers[l].sim, layers[l].need_full)),
        })
        del h2o

    # ---- roofline of the split full-attention kernel ----
    # rk_full_attn_scores launches that kernel alone.  One launch per layer (round-robin, so the
    # 256 MB last-level cache never holds the rows about to be read) is captured in a HIP graph;
    # HIP events on the launch stream bracket each replay; average = elapsed / launches.
    scores_buf = weights
    def roof_call(l):
        rk.rk_full_attn_scores(geom, q_cur[l], *kv[l], seq_lens, Lb, None, workspace=ws)      # as a full step launches it
    roof_reps = 4
    per_replay = []
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        roof_call(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_roof = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_roof):
        for l in range(n_layers):
            roof_call(l)
    g_roof.replay(); torch.cuda.synchronize()
    ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(roof_reps):
        ea.record(); g_roof.replay(); eb.record(); torch.cuda.synchronize()
        per_replay.append(ea.elapsed_time(eb) * 1e3 / n_layers)
    split_us = float(np.mean(per_replay))
    n_roof_launches = roof_reps * n_layers
    # one plain copy of known size: the kernel against which profiler byte counters are scaled, and, timed, what a
    # copy reaches on this machine in this run (bytes read + bytes written per second)
    cal_src = kv[0][0].view(-1)                          # K of layer 0: B * Hkv * capacity * 256 bytes
    cal_dst = torch.empty_like(cal_src)
    calibration_bytes = rk.rk_calibration_copy(cal_dst, cal_src)
    torch.cuda.synchronize()
    g_copy = torch.cuda.CUDAGraph()                      # other layers' rows as sources: nothing of them is in a cache
    n_copies = min(n_layers, 4)
    with torch.cuda.graph(g_copy):
        for l in range(n_copies):
            rk.rk_calibration_copy(cal_dst, kv[l][0].view(-1))
    g_copy.replay(); torch.cuda.synchronize()
    copy_us = []
    for _ in range(4):
        ea.record(); g_copy.replay(); eb.record(); torch.cuda.synchronize()
        copy_us.append(ea.elapsed_time(eb) * 1e3 / n_copies)
    copy_gbps = round(2 * calibration_bytes / (float(np.median(copy_us)) * 1e-6) / 1e9, 1)
    del cal_dst
    rows = int(seq_lens.sum().item())                    # rows streamed per launch (all sequences)
    bytes_kv = 2 * Hkv * D * 2 * rows                    # K and V rows, bf16
    # what a kernel that only reads reaches here (rk_calibration_read: streaming 16-byte loads, nothing kept): over
    # a buffer far larger than the caches in one launch, and in launches of the size of one launch of the
    # full-cache kernel (its K and V bytes), one after the other over different parts of that buffer
    read_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    launch_bytes = min(bytes_kv // 16 * 16, read_buf.numel())
    windows = min(max(read_buf.numel() // launch_bytes, 1), 16)
    read_gbps = {}
    for key, n_bytes, n_launch in (("one_launch_1GiB", read_buf.numel(), 2), ("launches_of_full_attn_kv_bytes", launch_bytes, windows)):
        g_read = torch.cuda.CUDAGraph()
        rk.rk_calibration_read(read_buf, sink, n_bytes); torch.cuda.synchronize()
        with torch.cuda.graph(g_read):
            for i in range(n_launch):
                rk.rk_calibration_read(read_buf, sink, n_bytes, offset=(i % windows) * launch_bytes if n_bytes == launch_bytes else 0)
        g_read.replay(); torch.cuda.synchronize()
        us = []
        for _ in range(4):
            ea.record(); g_read.replay(); eb.record(); torch.cuda.synchronize()
            us.append(ea.elapsed_time(eb) * 1e3 / n_launch)
        read_gbps[key] = round(n_bytes / (float(np.median(us)) * 1e-6) / 1e9, 1)
        del g_read
    read_gbps["bytes_per_launch"] = int(launch_bytes)
    del read_buf
    bytes_w = 4 * Hq * rows                              # raw scores written by the same kernel
    algo_bytes = bytes_kv + bytes_w
    achieved = algo_bytes / (split_us * 1e-6) / 1e9
    # HBM traffic of that kernel from profiler byte counters, when a committed PMC summary exists
    traffic, traffic_source = profile_traffic(w.name, "attn_split")
    roofline = {"bound": "hbm", "kernel": "rk::attn_split_kernel<%d, 4, true, false, false, false, false> (first kernel of rk_full_attn when weights are returned)" % w.group,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_us": round(split_us, 2), "launches": n_roof_launches, "algorithmic_bytes": algo_bytes}
    # ---- the same for the kernel of the partial step (one launch: rk_partial_attn) ----
    # rows it reads: the K selected rows and the rows decoded since the refresh, per sequence
    recent_rows = int((seq_lens - layers[0].tail_start).clamp(min=0, max=max(w.stride, 1)).sum().item())   # (max_recent of the call)
    sel_rows = int(torch.minimum(layers[0].tail_start, torch.full_like(seq_lens, w.k_small)).sum().item())
    partial_bytes = 2 * Hkv * D * 2 * (sel_rows + recent_rows)
    partial_us = graph_us(partial_call, reps=8)
    p_traffic, p_source = profile_traffic(w.name, "partial_attn")
    # which hand-over the library picks for this shape: tagged partial results (merged by slices) for launches over few
    # (sequence, KV head) pairs and for groups of up to 4 heads; ticketed for larger groups in launches over many pairs
    pairs = B * Hkv
    tagged = pairs <= 16 or w.group <= 4
    roofline_partial = {"bound": "hbm", "kernel": "rk::attn_split_kernel<%d, 4, false, true, false, %s, false> (rk_partial_attn)" % (w.group, "true" if tagged else "false"),
                        "achieved": round(partial_bytes / (partial_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(partial_bytes / (partial_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                        "traffic": p_traffic, "traffic_source": p_source, "avg_launch_us": round(partial_us, 2),
                        "launches": 9 * n_layers, "algorithmic_bytes": partial_bytes,
                        "rows": {"selected": sel_rows, "decoded_since_refresh": recent_rows}}

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline and not light:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = 1
        n_cpu = min(args.cpu_layers, n_layers)
        period = max(w.stride, 1)
        tot = {"full": 0.0, "refresh": 0.0, "partial": 0.0}
        lens_np = lens0.numpy().astype(np.int64)
        for l in range(n_cpu):
            Kb, Vb = gen.bf16_bits(kv[l][0]), gen.bf16_bits(kv[l][1])
            qb = gen.bf16_bits(q_steps[:period + 1, l])
            c0 = time.perf_counter()
            o, wts, _ = oracle.full_attn(qb[0], Kb, Vb, lens_np, w.scale)
            c1 = time.perf_counter()
            idx, _ = oracle.topk_select(wts.astype(np.float32), lens_np, Hkv, w.k_small, w.pool_w)
            sk = np.zeros((B, Hkv, w.k_small, D), dtype=np.uint16); sv = sk.copy()
            oracle.gather_small_kv(Kb, Vb, idx, sk, sv)
            c2 = time.perf_counter()
            for r in range(1, period):
                oracle.partial_attn(qb[r], sk, sv, w.k_small, Kb, Vb, lens_np, lens_np + r, w.scale)
            c3 = time.perf_counter()
            tot["full"] += c1 - c0; tot["refresh"] += c2 - c1; tot["partial"] += c3 - c2
            del Kb, Vb
        steps_cpu = n_cpu * period
        cpu_us = (tot["full"] + tot["refresh"] + tot["partial"]) / steps_cpu * 1e6
        cpu = {"value": round(cpu_us, 1), "unit": "us/step/layer", "cores": int(threads), "kind": "oracle",
               "host_cpus": os.cpu_count(),
               "sample": "%d layers x one stride period (1 full step + selection + gather, %d partial steps) of %s"
                         % (n_cpu, period - 1, w.name),
               "full_us": round(tot["full"] / n_cpu * 1e6, 1), "refresh_us": round(tot["refresh"] / n_cpu * 1e6, 1),
               "partial_us": round(tot["partial"] / max(n_cpu * (period - 1), 1) * 1e6, 1)}

    # dynamic schedule: how often a full step was taken, per layer (refresh counters kept on the GPU)
    eff_stride = None
    if model is not None and w.dynamic:
        fired = (model.n_full.float().mean(dim=1) - 1.0).clamp(min=1e-9).cpu().numpy()      # minus the initialisation
        per_layer = T / fired
        eff_stride = {"mean": round(float(per_layer.mean()), 2), "min": round(float(per_layer.min()), 2),
                      "max": round(float(per_layer.max()), 2), "qc_stride": w.stride, "threshold": w.threshold}
    us_per_step_layer = ms_per_step * 1e3 / n_layers
    n_full = sum(k == "full" for k in kinds)
    n_both = sum(k == "both" for k in kinds)
    result = {
        "metric": "decode attention us/step/layer (full vs partial) + achieved HBM GB/s vs peak",
        "value": round(us_per_step_layer, 3), "unit": "us/step/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers": n_layers, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "context": L0, "k_small": w.k_small, "stride": w.stride, "pool_w": w.pool_w,
                   "schedule": "dynamic" if w.dynamic else "fixed", "full_steps": n_full,
                   "partial_steps": args.steps - n_full - n_both, "trigger_test_steps": n_both, "launch": {"graph": "hip_graph", "native": "rk_decode_step_batched" if args.refresh == "batched" and not args.no_overlap else "rk_decode_step", "eager": "eager",
                                                                      "hybrid": "rk_decode_step (partial steps) + hip_graph (full steps)"}[launch],
                   "refresh": ("serial per layer" if args.no_overlap else
                               "batched over the layers (rk_refresh_batched)" if args.refresh == "batched" else
                               "per layer on a second stream")},
        "step_us_per_layer": {k: round(v, 2) for k, v in med.items()},
        "step_us_per_layer_p10_p90": spread,
        "call_us_per_layer": {k: round(v, 2) for k, v in klass.items()},
        # attention time per (step, layer) of the paper's comparison systems at kernel level (Table 1, "Time"):
        # vanilla = full attention at every step; StreamingLLM and SnapKV = the partial step at every step;
        # H2O = attention over K + 1 rows with the scores returned + its bookkeeping; RefreshKV = `value`
        "policy_us_per_layer": None if light else {"vanilla": round(klass["full_attn_no_weights"], 2),
                                                   "streaming_llm_or_snapkv": round(klass["partial_attn"], 2),
                                                   "h2o": round(klass["h2o_step"], 2), "refreshkv": round(us_per_step_layer, 2)},
        "full_over_partial": round(klass["full_attn"] / klass["partial_attn"], 2),
        "full_attn_GBps": round((bytes_kv + bytes_w) / (klass["full_attn"] * 1e-6) / 1e9, 1),
        "partial_attn_GBps": round(2 * Hkv * D * 2 * (w.k_small + 1) * B / (klass["partial_attn"] * 1e-6) / 1e9, 1),
        "effective_stride": eff_stride,
        # Appendix A.2's cost model: K/V bytes moved per step and layer, averaged over a stride period
        # = bytes per token x (L / S + K), here with the true sum of lengths, beside what it would
        # take at the rate the first kernel of a full step reaches and what a step takes
        "cost_model": cost_model(w, lens0, eff_stride, roofline["achieved"], us_per_step_layer),
        "roofline": roofline,
        "roofline_partial": roofline_partial,
        "copy_GBps": copy_gbps,
        "read_GBps": read_gbps,
        "cpu_baseline": cpu,
        "calibration_copy_bytes": calibration_bytes,
        "setup_s": round(setup_s, 1),
    }
    return result


if __name__ == "__main__":
    main()
