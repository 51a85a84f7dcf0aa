#!/usr/bin/env python3
"""Benchmark of the retrieval-attention hot path on one MI355X.

Prefill (the headline).  A step is one whole single-layer windowed prefill of the
workload's context: for every window, actqkv_build_probe -> actqkv_score_blocks ->
actqkv_select -> actqkv_retrieval_attention, in order, on one stream, with all inputs
resident in HBM.  The default workload is the benchmark's configs[2] (LLaMA3-8B layer,
128K tokens, window 512, top-k 32 with the dynamic cut-off): the one its metric
"tokens/s per layer @128K" is quoted on.  The step's launches are captured once in a HIP
graph (checked against the eager result on several replays) and the timed region replays
it; then one eager pass of the same step brackets every attention launch with HIP events
on its stream for the roofline figure (a graph cannot hold timing events).

Decode (second part of the metric).  configs[3]: 16 sequences x 32 layers x 64K cached
tokens, one new token per sequence per step, per-layer dynamic cut-off; a step is all 32
layers; reported as us/step with the HBM roofline of the decode attention kernel.

Prints ONE JSON line.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0
PEAK_FP32_TFLOPS = 157.3    # fp32 vector arithmetic (the fp32 workload's attention runs in row kernels)


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def attention_flops(shape, w0: int, rows: int, n_sel: int, l0: int) -> float:
    """Algorithmic flops of one window's attention: 4*D per (query, visible key) pair, the
    causal part of the window counted once."""
    i0 = min(shape.n_init, w0)
    past = i0 + n_sel * shape.block_size + (w0 - l0)
    pairs = rows * past + rows * (rows + 1) / 2
    return 4.0 * shape.head_dim * shape.n_q_heads * pairs


def cpu_baseline(w, q, k, v, rep, cutoffs, sample):
    """Times the oracle, as it stands, on a few whole windows of the same workload."""
    import numpy as np
    from oracle import actqkv_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sh = w.shape
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    kf, vf, repf = f(k), f(v), f(rep)
    t_total = 0.0
    tokens = 0
    for t in sample:
        w0 = t * w.window
        qw = f(q[w0:w0 + w.window])
        t0 = time.perf_counter()
        flat = qw.reshape(qw.shape[0], -1)
        st = orc.RunningStats(flat.shape[1])
        z, s2 = st.update(flat)
        phi = orc.activation_bias(flat, z, s2)
        probe, _ = orc.probe_query(flat, phi)
        res = orc.retrieve(probe, repf, w0, sh.n_init, sh.n_local, sh.block_size, sh.group, w.k_cap,
                           None if cutoffs is None else cutoffs[t])
        orc.retrieval_attention_window(qw, kf, vf, w0, res["idx"], sh.n_init, sh.n_local,
                                       sh.block_size, sh.group)
        t_total += time.perf_counter() - t0
        tokens += qw.shape[0]
    return {"value": tokens / t_total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{len(sample)} windows spread evenly over the {w.n_windows} (first {sample[0]}, last "
                      f"{sample[-1]}; all steps of the path, all rows), {t_total:.1f} s of numpy fp64"}


def capture_graph(torch, step_fn, check_tensor, log_name):
    """Captures step_fn in a HIP graph and checks three replays, with eager work in between,
    against the eager result.  Returns the graph, or None if capture or the check failed."""
    try:
        step_fn()
        torch.cuda.synchronize()
        want = check_tensor.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step_fn()
        for i in range(3):
            check_tensor.zero_()
            g.replay()
            torch.cuda.synchronize()
            if not torch.equal(check_tensor, want):
                log(f"{log_name}: graph replay {i} differs from the eager result; timing eagerly")
                return None
            step_fn()                      # eager work between replays
            torch.cuda.synchronize()
        return g
    except Exception as e:  # capture not possible: time the eager loop instead
        log(f"{log_name}: graph capture failed ({e}); timing eagerly")
        return None


PMC_COPY_BYTES = 256 << 20


def pmc_pass(torch, B, one_step, info, after=None, info_dir="."):
    """One eager pass of the step for a hardware-counter run (rocprofv3 --pmc FETCH_SIZE or
    WRITE_SIZE), after a plain copy of known size that calibrates the counter.  `after()` adds
    what is only known once the pass has run (the blocks it selected, its algorithmic bytes);
    the description of the pass goes to <info_dir>/pmc_pass_<workload>.json (--pmc-info-dir), from
    where bench_traffic.py copies it next to the counter bytes."""
    src = torch.ones(PMC_COPY_BYTES, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros_like(src)
    torch.cuda.synchronize()
    B.copy_bytes(dst, src)
    torch.cuda.synchronize()
    one_step()
    torch.cuda.synchronize()
    info = dict(info, pmc_pass=True, copy_bytes=PMC_COPY_BYTES)
    if after is not None:
        info.update(after())
    out_dir = os.path.abspath(info_dir)
    os.makedirs(out_dir, exist_ok=True)
    with open(os.path.join(out_dir, f"pmc_pass_{info['workload']}.json"), "w") as f:
        json.dump(info, f, indent=1, sort_keys=True)
    return info


def measured_traffic(workload):
    """HBM bytes per attention launch from the committed counter runs (bench_traffic.json,
    written by bench_traffic.py), or None."""
    try:
        with open(os.path.join(ROOT, "bench_traffic.json")) as f:
            return json.load(f).get(workload)
    except (OSError, ValueError):
        return None


def traffic_fields(workload, mean_blocks_selected=None):
    """roofline.traffic: the stored counter bytes, as long as they were taken on the kernels that
    are being timed (same hash of csrc/) and on a pass that selected about as many blocks."""
    t = measured_traffic(workload)
    if not t:
        return {"traffic": None, "traffic_note": "no counter run stored for this workload"}
    import bench_traffic
    now = bench_traffic.source_hash()
    if t.get("source_hash") != now:
        return {"traffic": None,
                "traffic_note": f"stored counters were taken on other kernel sources ({t.get('source_hash')}, "
                                f"now {now}): re-run the counter passes (profiles/ names the commands)"}
    e_pass = (t.get("pass") or {}).get("mean_blocks_selected")
    if mean_blocks_selected is not None and e_pass is not None and abs(e_pass - mean_blocks_selected) > 0.5:
        return {"traffic": None,
                "traffic_note": f"stored counters come from a pass that selected {e_pass:.2f} blocks on average, "
                                f"this run {mean_blocks_selected:.2f}"}
    return {"traffic": t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"],
            "traffic_detail": dict(t, unit="bytes per attention launch",
                                   source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py --pmc-pass, "
                                          "scaled by a 256 MiB copy kernel; summaries under profiles/")}


def bench_prefill(args, torch, B, H, synth):
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    if args.n_ctx:
        w = synth.scaled(w, n_ctx=args.n_ctx)
    sh = w.shape
    log(f"prefill {w.name}: generating inputs on the device")
    q, k, v = synth.gen_layer(w, dev)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    kc, vc = H.blocked_k(k, sh, w.n_blocks), H.blocked_vt(v, sh, w.n_blocks)
    repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=dev)
    repd[: rep.shape[0]] = rep
    cutoffs = None
    if w.cutoff:
        cutoffs = []
        for t in range(w.n_windows):
            b, e = H.eligible_range(sh, t * w.window)
            cutoffs.append(synth.cutoff_state(w, e - b, t, 0))
    runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, dev)
    plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, dev)
    bud0 = None if plan.budget is None else plan.budget.clone()
    out = torch.zeros_like(q)
    n_win = plan.n_windows

    # Two dependency chains (see PrefillPipeline): with overlap, the attention of window t runs
    # on a second stream beside the probe / score / select chain of window t+1.
    pipe = H.PrefillPipeline(runner, plan)
    nsel_log = pipe.n_sel

    def one_step(events=None, overlap=False, prelude_events=None):
        runner.stats.zero_()
        if bud0 is not None:
            plan.budget.copy_(bud0)
        pipe.run(q, kc, vc, repd, out, overlap, events, args.chunk, args.score_chunk, not args.per_window_selection,
                 args.attention_late_cus if overlap else 0, args.attention_cus if overlap else 256, prelude_events)

    if args.pmc_pass:
        def after():
            ns = nsel_log.cpu().tolist()
            elem = 4 if sh.dtype == "fp32" else 2
            # per window: its queries and outputs once, and every visible key and value once
            byt = 0.0
            for t in range(n_win):
                w0, rows = plan.w0[t], plan.rows[t]
                keys = min(sh.n_init, w0) + ns[t] * sh.block_size + (w0 - H.local_start(sh, w0)) + rows
                byt += (2 * rows * sh.n_q_heads + 2 * keys * sh.n_kv_heads) * sh.head_dim * elem
            n_launch = max(len(pipe.chunk_starts), 1)
            return {"mean_blocks_selected": sum(ns) / max(n_win, 1), "attention_launches": n_launch,
                    "algorithmic_bytes_per_launch": byt / n_launch}
        return pmc_pass(torch, B, lambda: one_step(overlap=not args.no_overlap),
                        {"workload": w.name, "windows": n_win, "windows_per_launch": args.chunk,
                         "attention_cus": args.attention_cus, "attention_late_cus": args.attention_late_cus},
                        after, args.pmc_info_dir)
    def timed(run, steps):
        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    # strictly in window order (one stream): reported beside the headline number
    graph_serial = None if args.eager else capture_graph(torch, one_step, out, "prefill (window order)")
    serial_s = timed(graph_serial.replay if graph_serial is not None else one_step, min(args.steps, 3))
    overlap = not args.no_overlap
    if overlap:
        step_fn = lambda: one_step(overlap=True)
        graph = None if args.eager else capture_graph(torch, step_fn, out, "prefill (two streams)")
        run = graph.replay if graph is not None else step_fn
        elapsed = timed(run, args.steps) * args.steps
    else:
        graph, elapsed = graph_serial, serial_s * args.steps
        if args.steps > 3:
            elapsed = timed(graph_serial.replay if graph_serial is not None else one_step, args.steps) * args.steps

    # ---- roofline of the dominant kernel: the prefill attention launches of one eager pass in
    # the schedule that was timed, events on the stream the attention runs on
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_win)]
    batched = overlap and not args.per_window_selection
    pre = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_win)]
    one_step(ev, overlap, pre if batched else None)
    torch.cuda.synchronize()
    n_sel = nsel_log.cpu().tolist()
    flops = sum(attention_flops(sh, plan.w0[t], plan.rows[t], n_sel[t], H.local_start(sh, plan.w0[t]))
                for t in range(n_win))
    starts = list(pipe.chunk_starts)
    attn_ms = sum(ev[t][0].elapsed_time(ev[t][1]) for t in starts)
    n_launch = len(starts)
    achieved = flops / (attn_ms * 1e-3) / 1e12
    res = {
        "metric": "prefill retrieval-attn tokens/s per layer @128K" if not args.n_ctx and
                  args.workload == "c3_128k" else f"prefill retrieval-attn tokens/s per layer ({w.name})",
        "value": w.n_ctx * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: 1 sequence, 1 layer, H{sh.n_q_heads}/Hk{sh.n_kv_heads}/D{sh.head_dim}, "
                               f"{w.n_ctx} tokens, window {w.window}, block {sh.block_size} x {sh.n_rep} rep keys, "
                               f"n_init {sh.n_init}, n_local {sh.n_local}, k_cap {w.k_cap}, "
                               f"cut-off {'on' if w.cutoff else 'off'}",
                   "windows": n_win, "mean_blocks_selected": sum(n_sel) / max(n_win, 1),
                   "launch": ("hip graph replay" if graph is not None else "eager") +
                             (f", two streams, {args.chunk} windows per call: probes, scores and selection of chunk "
                              f"c + 1 beside the attention of chunk c ({args.attention_cus} of 256 CUs" +
                              (f", {args.attention_late_cus} more once chunk c + 1 is prepared)"
                               if args.attention_late_cus else ")")
                              if overlap and not args.per_window_selection else
                              f", three streams: probes, then scoring and selection ({args.score_chunk} windows per "
                              f"hand-over), then attention ({args.attention_cus} of 256 CUs, up to {args.chunk} "
                              "windows per launch)" if overlap and args.score_chunk > 0 else
                              f", attention on a second stream ({args.attention_cus} of 256 CUs, up to {args.chunk} "
                              "windows per hand-over) beside the probe/score/select chain of the following windows"
                              if overlap
                              else ", one stream, window order"),
                   "ms_per_step_window_order": serial_s * 1e3},
        "roofline": {"bound": "mfma" if sh.dtype == "bf16" else "alu", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS if sh.dtype == "bf16" else PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / (PEAK_BF16_TFLOPS if sh.dtype == "bf16" else PEAK_FP32_TFLOPS),
                     **traffic_fields(w.name, sum(n_sel) / max(n_win, 1)),
                     "kernel": ("actqkv_retrieval_attention launches of up to %d windows "
                                "(attn_prefill_mfma_queued_kernel%s)" %
                                (args.chunk, "; timed: the first team's launch of %d workgroups, with which the "
                                             "second team of %d ends" % (args.attention_cus, args.attention_late_cus)
                                 if args.attention_late_cus and not args.per_window_selection else "")) if overlap else
                               "actqkv_retrieval_attention launch (attn_prefill_mfma_kernel)",
                     "avg_launch_us": attn_ms * 1e3 / n_launch,
                     "windows_per_launch": n_win / n_launch,
                     "algorithmic_gflop_per_launch": flops / n_launch / 1e9,
                     "timing": "HIP events, on the stream the attention runs on, around every attention "
                               "launch of one eager pass of the step in the timed schedule"},
    }
    if batched:
        # The other chain: probes, scores and selections of a chunk of windows (actqkv_build_probe,
        # actqkv_score_blocks, actqkv_select: 6 launches), timed on the stream they run on, beside the
        # attention of the chunk before.  Algorithmic bytes: every window's queries once and the
        # representative keys of its eligible blocks once.
        starts_all = list(pipe.chunk_starts)
        pre_us = [pre[t][0].elapsed_time(pre[t][1]) * 1e3 for t in starts_all]
        elem = 4 if sh.dtype == "fp32" else 2
        pre_bytes = []
        for i, t0 in enumerate(starts_all):
            t1 = starts_all[i + 1] if i + 1 < len(starts_all) else n_win
            byt = 0
            for t in range(t0, t1):
                b, e = H.eligible_range(sh, plan.w0[t])
                byt += plan.rows[t] * sh.n_q_heads * sh.head_dim * elem
                byt += (e - b) * sh.n_rep * sh.n_kv_heads * sh.head_dim * elem
            pre_bytes.append(byt)
        tot_us, tot_b = sum(pre_us), float(sum(pre_bytes))
        res["prelude"] = {"bound": "hbm", "achieved": tot_b / (tot_us * 1e-6) / 1e9, "peak": PEAK_HBM_GBS,
                          "unit": "GB/s", "frac": tot_b / (tot_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                          "kernels": "probe_rows_moments, probe_chain_stats, probe_rows_bias_weigh, "
                                     "probe_chain_finish, score_blocks, select (one call of each per chunk)",
                          "us_per_chunk": [round(u, 1) for u in pre_us],
                          "algorithmic_mb_per_chunk": [round(b / 1e6, 1) for b in pre_bytes],
                          "timing": "HIP events on the stream of the chain, around the three calls of every chunk, "
                                    "in the same eager pass as the attention's; the chain shares the chip with "
                                    "the attention of the chunk before (%d of 256 CUs)" % args.attention_cus}
    if not args.no_cpu_baseline:
        T = n_win
        stride = max(T // 48, 1)                  # about 48 windows, 10-20 s of oracle time
        sample = sorted(set(range(stride // 2, T, stride)) | {T - 1})
        log("cpu_baseline: timing the oracle on sampled windows")
        res["cpu_baseline"] = cpu_baseline(w, q, k, v, rep, cutoffs, sample)
    return res


def bench_other_configs(args, torch, B, H, synth):
    """The workloads beside the headline one, each as a short run of the same schedule, reduced to
    the figures of a bench line: c1_8k_fp32 and c2_32k (one layer), c5_200k (32 layers, every
    layer with its own inputs)."""
    import copy
    out = {}
    for name in ("c1_8k_fp32", "c2_32k"):
        a = copy.copy(args)
        a.workload, a.n_ctx, a.steps, a.warmup, a.no_cpu_baseline, a.pmc_pass = name, 0, 5, 1, True, False
        r = bench_prefill(a, torch, B, H, synth)
        torch.cuda.empty_cache()
        out[name] = {"parity": {"c1_8k_fp32": "tests/test_gpu_parity.py::test_c1_fp32_full_parity (every window, every "
                                              "row against the oracle; bar 1e-4)",
                                "c2_32k": "tests/test_gpu_parity.py::test_c2_32k_full_size_sampled_windows (every "
                                          "window's probe, scores, density, selection; sampled windows' outputs; "
                                          "bar 2e-2)"}[name],
                     "metric": r["metric"], "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                     "steps": r["steps"], "dtype": r["dtype"], "workload": r["config"]["workload"],
                     "windows": r["config"]["windows"], "mean_blocks_selected": r["config"]["mean_blocks_selected"],
                     "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac",
                                                                "avg_launch_us", "windows_per_launch")}}
    a = copy.copy(args)
    a.workload, a.n_ctx, a.steps, a.warmup, a.layers = "c5_200k", 0, 2, 1, synth.WORKLOADS["c5_200k"].n_layers
    r = bench_prefill_layers(a, torch, B, H, synth)
    torch.cuda.empty_cache()
    out["c5_200k"] = {k: r[k] for k in ("metric", "value", "unit", "ms_per_step", "steps", "dtype", "roofline_of_the_pass")}
    out["c5_200k"].update(parity="tests/test_gpu_parity.py::test_c5_200k_full_size_sampled_windows (the last layer "
                                 "at full size against the oracle; bar 2e-2)",
                          workload=r["config"]["workload"], ms_per_layer=r["config"]["ms_per_layer"],
                          mean_blocks_selected_per_layer=[round(x, 2) for x in
                                                          r["config"]["mean_blocks_selected_per_layer"]])
    return out


def bench_recall(args, torch, B, H, synth, workload="c3_128k"):
    """Synthetic stand-in for the ablation of Sec. 5.3 / Table 3: how many of the blocks that the input
    recipe planted (keys shifted toward the direction the outlier queries carry) each variant of
    the retrieval recalls, over every window of the workload, all through the library's calls:
    probe-Query (Eq. 9) against mean pooling; a fixed k against the dynamic cut-off (Eq. 11, 12)
    at the same mean number of blocks; the density over all eligible blocks against over the
    top-k only; one selection for all heads against one per KV head."""
    base = synth.WORKLOADS[workload]
    out = {}
    # the workload's own recipe, then the same with the planted keys and the outlier queries further out:
    # where the variants part depends on how strong the planted relation is
    for alpha, shift in ((base.alpha, base.shift), (base.alpha, 4 * base.shift), (4 * base.alpha, 4 * base.shift)):
        w = synth.scaled(base, alpha=alpha, shift=shift)
        r = _recall_of(w, torch, B, H, synth)
        out[f"outlier queries + {alpha:g} u, planted keys + {shift:g} u" +
            (" (the workload's recipe)" if (alpha, shift) == (base.alpha, base.shift) else "")] = r
    T = base.n_ctx // base.window
    return {"workload": base.name, "windows": T, "planted_blocks": base.n_planted, "k_cap": base.k_cap,
            "what": "over all windows with a planted block among the eligible ones: recall = planted blocks "
                    "selected / planted blocks eligible, precision = planted blocks selected / blocks selected; "
                    "the cut-off rows use the workload's seeded budget per window",
            "by_planted_signal": out}


def _recall_of(w, torch, B, H, synth, selections=None):
    """selections: an optional dict that receives, per variant, the lists (idx rows, counts)."""
    dev = "cuda:0"
    sh = w.shape
    cs = B.c_shape(sh)
    q, k, _ = synth.gen_layer(w, dev)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    del k
    repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=dev)
    repd[: rep.shape[0]] = rep
    planted = set(synth.planted_blocks(w))
    m, hk, kc = w.window, sh.n_kv_heads, w.k_cap
    T = w.n_ctx // m
    runs = {"probe": H.LayerRunner(sh, 1, m, w.n_blocks, kc, dev), "mean": H.LayerRunner(sh, 1, m, w.n_blocks, kc, dev)}
    stride = runs["probe"].score_stride
    nb_begin = sh.n_init // sh.block_size
    sc = {n: torch.zeros(T, stride, device=dev) for n in ("probe", "mean")}
    sc_ph = torch.zeros(T, hk, stride, device=dev)
    ends = [H.eligible_range(sh, t * m)[1] for t in range(T)]
    nb_end = torch.tensor(ends, dtype=torch.int32, device=dev)
    nb_end_ph = nb_end[:, None].expand(T, hk).contiguous()
    for t in range(T):
        for name, r in runs.items():
            flags = B.STATS_UPDATE | (B.PROBE_MEAN_POOLING if name == "mean" else 0)
            B.build_probe(cs, 1, m, q[t * m:(t + 1) * m], r.stats, flags, r.probe, r.probe_kv, r.probe_norm, None,
                          r.workspace)           # (every window enters the running statistics)
            if ends[t] <= nb_begin:
                continue
            B.score_blocks(cs, 1, r.probe_kv, r.probe_norm, repd, 0, ends[t], nb_begin, nb_end[t:t + 1],
                           sc[name][t:t + 1], stride)
        if ends[t] > nb_begin:
            B.score_blocks_per_head(cs, 1, runs["probe"].probe, repd, 0, ends[t], nb_begin, nb_end_ph[t:t + 1],
                                    sc_ph[t:t + 1], stride)
    nb_max = max(ends)
    cut = [synth.cutoff_state(w, max(ends[t] - nb_begin, 0), t, 0) for t in range(T)]
    bud = torch.tensor([c[0] for c in cut], dtype=torch.float32, device=dev)
    rest = torch.tensor([c[1] for c in cut], dtype=torch.float32, device=dev)

    def select(scores, rows, ends_t, k, cutoff, flags=0):
        idx = torch.full((rows, k), -1, dtype=torch.int32, device=dev)
        n = torch.zeros(rows, dtype=torch.int32, device=dev)
        b = r_ = None
        if cutoff:
            per = rows // T
            b = bud.repeat_interleave(per).contiguous()
            r_ = rest.repeat_interleave(per).contiguous()
        sc2, e2 = scores.view(rows, stride), ends_t.reshape(rows).contiguous()
        for r0 in range(0, rows, 1024):                    # the library takes at most 1024 rows a call
            r1 = min(r0 + 1024, rows)
            B.select(r1 - r0, sc2[r0:r1], stride, nb_max, nb_begin, e2[r0:r1], k, None if b is None else b[r0:r1],
                     None if r_ is None else r_[r0:r1], idx[r0:r1], n[r0:r1], None, None, None, flags)
        return idx.cpu().tolist(), n.cpu().tolist()

    def tally(idx, n, per=1):
        if selections is not None:
            selections[len(selections)] = (idx, n)
        hit = sel = tot = 0
        for row in range(len(n)):
            t = row // per
            p = {b for b in planted if nb_begin <= b < ends[t]}
            if not p:
                continue
            got = set(idx[row][:n[row]])
            hit += len(got & p)
            sel += n[row]
            tot += len(p)
        return {"recall": hit / max(tot, 1), "precision": hit / max(sel, 1),
                "mean_blocks_selected": sel / max(sum(1 for t in range(T) if any(nb_begin <= b < ends[t]
                                                                                  for b in planted)) * per, 1)}

    out = {}
    out["probe_query_fixed_k"] = tally(*select(sc["probe"], T, nb_end, kc, False))
    out["mean_pooling_fixed_k"] = tally(*select(sc["mean"], T, nb_end, kc, False))
    out["per_kv_head_fixed_k"] = tally(*select(sc_ph, T * hk, nb_end_ph, kc, False), per=hk)
    out["probe_query_cutoff"] = tally(*select(sc["probe"], T, nb_end, kc, True))
    out["probe_query_cutoff_density_over_top_k"] = tally(*select(sc["probe"], T, nb_end, kc, True,
                                                                 B.SELECT_ENTROPY_TOPK))
    out["mean_pooling_cutoff"] = tally(*select(sc["mean"], T, nb_end, kc, True))
    k_same = max(1, min(kc, round(out["probe_query_cutoff"]["mean_blocks_selected"])))
    out[f"probe_query_fixed_k_at_the_cutoffs_mean_of_{k_same}"] = tally(*select(sc["probe"], T, nb_end, k_same, False))
    out[f"mean_pooling_fixed_k_of_{k_same}"] = tally(*select(sc["mean"], T, nb_end, k_same, False))
    return {name: {k_: round(v_, 4) for k_, v_ in r.items()} for name, r in out.items()}


def bench_prefill_layers(args, torch, B, H, synth):
    """configs[4]-style run: all `--layers` layers of one sequence, every layer with its own
    seeded inputs, outlier rate, statistics and cut-off profile, in the benchmarked schedule
    (one call per step and chunk of windows, attention on a second stream), layer after layer
    in one HIP graph.  Reported in token-layers per second, i.e. the per-layer rate."""
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    if args.n_ctx:
        w = synth.scaled(w, n_ctx=args.n_ctx)
    sh, L = w.shape, args.layers
    layers = []
    out = None
    for l in range(L):
        log(f"prefill {w.name}: generating layer {l + 1} of {L} on the device")
        q, k, v = synth.gen_layer(w, dev, l)
        rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
        kc, vc = H.blocked_k(k, sh, w.n_blocks), H.blocked_vt(v, sh, w.n_blocks)
        del k, v
        repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=dev)
        repd[: rep.shape[0]] = rep
        cutoffs = None
        if w.cutoff:
            cutoffs = []
            for t in range(w.n_windows):
                b, e = H.eligible_range(sh, t * w.window)
                cutoffs.append(synth.cutoff_state(w, e - b, t, l))
        runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, dev)
        plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, dev)
        bud0 = None if plan.budget is None else plan.budget.clone()
        if out is None:
            out = torch.zeros_like(q)          # one output buffer: the layers run one after the other
        layers.append((q, kc, vc, repd, runner, plan, bud0, H.PrefillPipeline(runner, plan)))
    torch.cuda.empty_cache()

    def one_step():
        for q, kc, vc, repd, runner, plan, bud0, pipe in layers:
            runner.stats.zero_()
            if bud0 is not None:
                plan.budget.copy_(bud0)
            pipe.run(q, kc, vc, repd, out, True, None, args.chunk, args.score_chunk, True, args.attention_late_cus,
                     args.attention_cus)

    graph = None if args.eager else capture_graph(torch, one_step, out, f"prefill ({L} layers)")
    run = graph.replay if graph is not None else one_step
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    n_sel = [sum(pipe.n_sel.cpu().tolist()) / plan.n_windows for *_, plan, _, pipe in layers]
    # the attention's algorithmic flops of the whole pass over the whole pass's time: a lower bound of
    # what the attention launches reach (the pass also holds the other chain's first chunk per layer)
    flops = 0.0
    for *_, plan, _, pipe in layers:
        ns = pipe.n_sel.cpu().tolist()
        flops += sum(attention_flops(sh, plan.w0[t], plan.rows[t], ns[t], H.local_start(sh, plan.w0[t]))
                     for t in range(plan.n_windows))
    return {"metric": f"prefill retrieval-attn tokens/s per layer ({w.name}, {L} layers)",
            "roofline_of_the_pass": {"bound": "mfma", "achieved": flops / dt / 1e12, "peak": PEAK_BF16_TFLOPS,
                                     "unit": "TFLOP/s", "frac": flops / dt / 1e12 / PEAK_BF16_TFLOPS,
                                     "what": "attention flops of all layers / time of the whole pass"},
            "value": w.n_ctx * L / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": sh.dtype, "data": "synthetic",
            "config": {"workload": f"{w.name}: 1 sequence, {L} layers, {w.n_ctx} tokens, window {w.window}, "
                                   f"k_cap {w.k_cap}, cut-off {'on' if w.cutoff else 'off'}, per-layer outlier "
                                   f"rates {synth.layer_outlier_rate(w, 0):.3f} .. {synth.layer_outlier_rate(w, L - 1):.3f}",
                       "ms_per_layer": dt * 1e3 / L, "mean_blocks_selected_per_layer": n_sel,
                       "launch": ("hip graph replay" if graph is not None else "eager") +
                                 f", {args.chunk} windows per call, attention on {args.attention_cus} of 256 CUs"}}


def bench_prefill_host_cache(args, torch, B, H, synth):
    """The same layer pass with the cache of the whole context in pinned host memory and a
    working cache of a few dozen blocks in HBM (harness.HostCachePrefill): what the blocks a
    window selects cost when they come over the host link.  Window order, one stream, eager."""
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    if args.n_ctx:
        w = synth.scaled(w, n_ctx=args.n_ctx)
    sh = w.shape
    log(f"prefill {w.name}, cache in pinned host memory: generating inputs")
    q, k, v = synth.gen_layer(w, dev)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=dev)
    repd[: rep.shape[0]] = rep
    k_store = H.blocked_k(k, sh, w.n_blocks).cpu().pin_memory()
    v_store = H.blocked_vt(v, sh, w.n_blocks).cpu().pin_memory()
    cutoffs = None
    if w.cutoff:
        cutoffs = []
        for t in range(w.n_windows):
            b, e = H.eligible_range(sh, t * w.window)
            cutoffs.append(synth.cutoff_state(w, e - b, t, 0))
    runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, dev)
    plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, dev)
    bud0 = None if plan.budget is None else plan.budget.clone()
    host = H.HostCachePrefill(runner, plan)
    out = torch.zeros_like(q)
    block_bytes = 2 * sh.n_kv_heads * sh.block_size * sh.head_dim * (4 if sh.dtype == "fp32" else 2)

    def timed(fn, steps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    # ---- window order on one stream, eager (the store filled beforehand)
    def in_order():
        runner.stats.zero_()
        if bud0 is not None:
            plan.budget.copy_(bud0)
        return host.run(q, k, v, k_store, v_store, repd, out, record=range(plan.n_windows))

    gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(plan.n_windows)]
    runner.stats.zero_()
    if bud0 is not None:
        plan.budget.copy_(bud0)
    rec = host.run(q, k, v, k_store, v_store, repd, out, record=range(plan.n_windows), gather_events=gev)
    torch.cuda.synchronize()
    blocks = sum(int(r["n_sel"]) for r in rec.values())
    # the gather launches on their own: HIP events around every one of them in this pass
    g_with = [t for t in range(plan.n_windows) if int(rec[t]["n_sel"]) > 0]
    g_us = sum(gev[t][0].elapsed_time(gev[t][1]) for t in g_with) * 1e3
    steps = min(args.steps, 3)
    dt_order = timed(in_order, steps)
    out_order = out.clone()

    # ---- the overlapped schedule: selection chain ahead, data movement, write-back and attention on
    # streams of their own; the host store starts EMPTY and is filled by the write-back
    k_store.zero_()
    v_store.zero_()

    def overlapped():
        runner.stats.zero_()
        if bud0 is not None:
            plan.budget.copy_(bud0)
        host.run_overlapped(q, k, v, k_store, v_store, repd, out)

    # (eager: capturing this four-stream schedule in a HIP graph crashed on the host inside the
    # runtime's end-of-capture call, so it is not captured)
    graph = None
    dt = timed(overlapped, steps)
    same = bool(torch.equal(out, out_order))
    wb_bytes = (w.n_ctx // sh.block_size) * block_bytes
    return {"metric": "prefill retrieval-attn tokens/s per layer, cache in pinned host memory",
            "value": w.n_ctx / dt, "unit": "tokens/s", "ms_per_step": dt * 1e3, "steps": steps,
            "config": {"workload": w.name, "working_cache_blocks": host.nb_work, "working_caches": host.N_WORK,
                       "context_blocks": w.n_blocks,
                       "launch": ("hip graph replay" if graph is not None else "eager") +
                                 ", four streams: selection chain, data movement (local span, append, gather), "
                                 "write-back, attention",
                       "ms_per_step_window_order_one_stream": dt_order * 1e3,
                       "output_equals_window_order": same},
            "gather": {"bound": "host link (pinned host memory -> HBM)", "kernel": "gather_blocks_kernel "
                       "(actqkv_gather_blocks: the blocks one window selected, K and V)",
                       "achieved": blocks * block_bytes / max(g_us, 1e-9) / 1e3, "unit": "GB/s",
                       "launches_with_blocks": len(g_with), "avg_launch_us": g_us / max(len(g_with), 1),
                       "bytes_per_launch": blocks * block_bytes / max(len(g_with), 1),
                       "timing": "HIP events around every gather launch of one in-order pass"},
            "host_link": {"blocks_gathered_per_pass": blocks, "gather_bytes_per_pass": blocks * block_bytes,
                          "write_back_bytes_per_pass": wb_bytes,
                          "gather_GBps_over_the_whole_pass": blocks * block_bytes / dt / 1e9,
                          "both_directions_GBps_over_the_whole_pass": (blocks * block_bytes + wb_bytes) / dt / 1e9}}


def bench_decode(args, torch, B, H, synth):
    """configs[3]: batch 16 x 32 layers x 64K cached tokens, `decode_steps` steps."""
    dev = "cuda:0"
    w = synth.WORKLOADS["c4_decode"]
    if args.decode_layers:
        w = synth.scaled(w, n_layers=args.decode_layers)
    sh, L, bt = w.shape, w.n_layers, w.batch
    steps = args.decode_steps
    n0 = w.n_ctx                                     # cached tokens before the first step
    nb_cap = (n0 + steps + sh.block_size - 1) // sh.block_size
    hk, D, bs = sh.n_kv_heads, sh.head_dim, sh.block_size
    gb = 2 * L * bt * nb_cap * hk * bs * D * 2 / 1e9
    log(f"decode {w.name}: generating {gb:.0f} GB of KV cache on the device")
    kc = torch.empty(L, bt, nb_cap, hk, bs, D, dtype=torch.bfloat16, device=dev)
    vc = torch.empty(L, bt, nb_cap, hk, D, bs, dtype=torch.bfloat16, device=dev)
    rep = torch.empty(L, bt, nb_cap, sh.n_rep, hk, D, dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    u = synth.direction(w, 0, 0, dev)                # [Hk][D]
    for l in range(L):
        kc[l].normal_(generator=gen)
        vc[l].normal_(generator=gen)
        planted = torch.stack([torch.tensor(synth.planted_blocks(w, l, s)) for s in range(bt)]).to(dev)
        sidx = torch.arange(bt, device=dev)[:, None].expand_as(planted)
        kc[l][sidx, planted] += (w.shift * u)[None, None, :, None, :].to(torch.bfloat16)
        rep[l] = synth.pick_rep_keys_blocked(kc[l], sh.n_rep)
    u_hat = u.repeat_interleave(sh.group, dim=0)
    q_all = torch.randn(steps, L, bt, 1, sh.n_q_heads, D, generator=gen, device=dev) + w.alpha * u_hat
    q_all = q_all.to(torch.bfloat16)
    # keys and values of the tokens generated during the run, appended layer by layer (Eq. (4))
    k_all = torch.randn(steps, L, bt, 1, hk, D, generator=gen, device=dev).to(torch.bfloat16)
    v_all = torch.randn(steps, L, bt, 1, hk, D, generator=gen, device=dev).to(torch.bfloat16)
    out = torch.zeros(L, bt, 1, sh.n_q_heads, D, dtype=torch.bfloat16, device=dev)
    runner = H.LayerRunner(sh, bt, 1, nb_cap, w.k_cap, dev)
    nb_begin = sh.n_init // bs
    # per-step device scalars
    n_ctx_all = torch.tensor([[n0 + 1 + t] * bt for t in range(steps)], dtype=torch.int32, device=dev)
    nb_end_host = [H.eligible_range(sh, n0 + t)[1] for t in range(steps)]
    nb_end_all = torch.tensor([[e] * bt for e in nb_end_host], dtype=torch.int32, device=dev)
    # Alg. 1 across layers and steps: the history of the layers' densities lives on the device
    b_init, _ = synth.decode_cutoff_profile(w, nb_end_host[0] - nb_begin)
    k_mean, theta_prior = b_init / L, math.log(max(nb_end_host[0] - nb_begin, 2))
    theta_sum = torch.zeros(bt, L, dtype=torch.float32, device=dev)
    hist_steps = torch.zeros(bt, dtype=torch.float32, device=dev)
    theta_step = torch.zeros(L, bt, dtype=torch.float32, device=dev)
    rest_all = torch.zeros(L, bt, dtype=torch.float32, device=dev)
    budget = torch.zeros(bt, dtype=torch.float32, device=dev)
    # the launch that selects inside the attention reads B_kv from one array and writes the rest to another
    budgets = [budget, torch.zeros(bt, dtype=torch.float32, device=dev)]
    nsel_log = torch.zeros(L, bt, dtype=torch.int32, device=dev)
    q_step = torch.zeros(L, bt, 1, sh.n_q_heads, D, dtype=torch.bfloat16, device=dev)
    step_no = torch.zeros(1, dtype=torch.int64, device=dev)
    n_ctx_cur = torch.zeros(bt, dtype=torch.int32, device=dev)
    pos_cur = torch.zeros(bt, dtype=torch.int32, device=dev)
    k_step = torch.zeros(L, bt, 1, hk, D, dtype=torch.bfloat16, device=dev)
    v_step = torch.zeros(L, bt, 1, hk, D, dtype=torch.bfloat16, device=dev)
    nb_end_cur = torch.zeros(bt, dtype=torch.int32, device=dev)
    cache_stride, rep_stride = kc[0].stride(0), rep[0].stride(0)

    def load_step(t):
        """Per-step inputs (new queries, lengths): device copies outside the library."""
        q_step.copy_(q_all[t])
        k_step.copy_(k_all[t])
        v_step.copy_(v_all[t])
        n_ctx_cur.copy_(n_ctx_all[t])
        torch.sub(n_ctx_cur, 1, out=pos_cur)
        nb_end_cur.copy_(nb_end_all[t])

    # The sequences of a batch do not depend on each other: with --decode-streams 2 the batch is cut
    # into two halves whose layer chains run on two streams, so that one half streams keys and values
    # while the other is in a latency-bound stretch (selection, merge of partials, launch boundary).
    n_streams = max(1, args.decode_streams)
    assert bt % n_streams == 0
    hb = bt // n_streams
    side_streams = [torch.cuda.Stream(device=dev) for _ in range(n_streams - 1)]
    runners = [runner] + [H.LayerRunner(sh, hb, 1, nb_cap, w.k_cap, dev) for _ in range(n_streams - 1)]

    def layer_chain(part, events, launches):
        lo, hi = part * hb, (part + 1) * hb
        r = runners[part]
        sl = slice(lo, hi)
        for l in range(L):
            if launches == 1:
                # the whole layer in one launch
                if events is not None:
                    events[l][0].record()
                B.decode_layer(r.cs, hb, q_step[l][sl], k_step[l][sl].view(hb, hk, D), v_step[l][sl].view(hb, hk, D),
                               kc[l][sl], vc[l][sl], cache_stride, rep[l][sl], rep_stride, nb_cap, n_ctx_cur[sl],
                               nb_begin, nb_end_cur[sl], r.scores, r.score_stride, w.k_cap, budgets[l % 2][sl],
                               rest_all[l][sl], budgets[(l + 1) % 2][sl], r.idx, nsel_log[l][sl], theta_step[l][sl],
                               None, out[l][sl], None, r.workspace)
                if events is not None:
                    events[l][1].record()
                continue
            if launches == 2:
                # cache update, probe and scores in one launch, selection and attention in the other
                B.decode_retrieve(r.cs, hb, q_step[l][sl], k_step[l][sl], v_step[l][sl], pos_cur[sl], kc[l][sl],
                                  vc[l][sl], cache_stride, rep[l][sl], rep_stride, nb_cap, nb_begin, nb_end_cur[sl],
                                  None, None, None, r.scores, r.score_stride, w.k_cap, None, None, None, None,
                                  None, None, None, flags=B.DECODE_SCORES_ONLY)
                if events is not None:
                    events[l][0].record()
                B.decode_select_attention(r.cs, hb, q_step[l][sl], kc[l][sl], vc[l][sl], cache_stride, nb_cap,
                                          n_ctx_cur[sl], r.scores, r.score_stride, nb_begin, nb_end_cur[sl],
                                          w.k_cap, budgets[l % 2][sl], rest_all[l][sl], budgets[(l + 1) % 2][sl],
                                          r.idx, nsel_log[l][sl], theta_step[l][sl], None, out[l][sl], None,
                                          r.workspace)
                if events is not None:
                    events[l][1].record()
                continue
            if launches == 3:
                # cache update, probe and scores in one launch, then the selection
                B.decode_retrieve(r.cs, hb, q_step[l][sl], k_step[l][sl], v_step[l][sl], pos_cur[sl], kc[l][sl],
                                  vc[l][sl], cache_stride, rep[l][sl], rep_stride, nb_cap, nb_begin, nb_end_cur[sl],
                                  None, None, None, r.scores, r.score_stride, w.k_cap, budget[sl], rest_all[l][sl],
                                  r.idx, nsel_log[l][sl], theta_step[l][sl], None)
            else:
                B.append_kv_probe(r.cs, hb, q_step[l][sl], k_step[l][sl], v_step[l][sl], pos_cur[sl], kc[l][sl],
                                  vc[l][sl], cache_stride, rep[l][sl], rep_stride, nb_cap, r.probe, r.probe_kv,
                                  r.probe_norm)
                B.score_blocks(r.cs, hb, r.probe_kv, r.probe_norm, rep[l][sl], rep_stride,
                               nb_end_host[-1], nb_begin, nb_end_cur[sl], r.scores, r.score_stride)
                B.select(hb, r.scores, r.score_stride, nb_end_host[-1], nb_begin, nb_end_cur[sl],
                         w.k_cap, budget[sl], rest_all[l][sl], r.idx, nsel_log[l][sl], theta_step[l][sl], None)
            if events is not None:
                events[l][0].record()
            B.retrieval_attention(r.cs, hb, 1, q_step[l][sl], kc[l][sl], vc[l][sl], cache_stride, nb_cap,
                                  n_ctx_cur[sl], r.idx, nsel_log[l][sl], w.k_cap, out[l][sl], None,
                                  r.workspace)
            if events is not None:
                events[l][1].record()

    def one_step(events=None, launches=None):
        launches = args.decode_launches if launches is None else launches
        # folds the step before into the history; B_kv = L * k again; R^l for every layer
        B.cutoff_next_step(bt, L, k_mean, theta_prior, theta_step, theta_sum, hist_steps, budget, rest_all)
        cur = torch.cuda.current_stream()
        for st in side_streams:
            st.wait_stream(cur)
        for part in range(n_streams - 1, 0, -1):
            with torch.cuda.stream(side_streams[part - 1]):
                layer_chain(part, None, launches)
        layer_chain(0, events, launches)
        for st in side_streams:
            cur.wait_stream(st)

    load_step(0)
    # the first step has no history: the prior stands in for every layer's mean density
    B.cutoff_next_step(bt, L, k_mean, theta_prior, None, theta_sum, hist_steps, budget, rest_all)
    for l in range(L):
        B.build_probe(runner.cs, bt, 1, q_step[l], None, False, runner.probe, runner.probe_kv,
                      runner.probe_norm, None, runner.workspace)
        B.score_blocks(runner.cs, bt, runner.probe_kv, runner.probe_norm, rep[l], rep_stride,
                       nb_end_host[-1], nb_begin, nb_end_cur, runner.scores, runner.score_stride)
        B.select(bt, runner.scores, runner.score_stride, nb_end_host[-1], nb_begin, nb_end_cur,
                 w.k_cap, budget, rest_all[l], runner.idx, nsel_log[l], theta_step[l], None)
    if args.pmc_pass:
        def after():
            ns = nsel_log.cpu()
            n_ctx_now = int(n_ctx_cur[0])
            keys = min(sh.n_init, n_ctx_now - 1) + (n_ctx_now - H.local_start(sh, n_ctx_now - 1))
            byt = float((ns.sum().item() * bs + keys * L * bt) * hk * D * 2 * 2)
            return {"mean_blocks_selected": float(ns.float().mean()), "layers": L, "batch": bt,
                    "launches_per_layer": args.decode_launches,
                    "algorithmic_bytes_per_launch": byt / L,
                    "scoring_bytes_per_launch": float((nb_end_host[0] - nb_begin) * sh.n_rep * hk * D * 2 * bt)}
        return pmc_pass(torch, B, one_step, {"workload": w.name, "launches": L}, after, args.pmc_info_dir)
    graph = None if args.eager else capture_graph(torch, one_step, out, "decode")
    run = graph.replay if graph is not None else one_step
    for t in range(min(8, steps)):
        load_step(t)
        run()
    torch.cuda.synchronize()
    times = []
    nsel_sum = torch.zeros(L, bt, dtype=torch.int64, device=dev)      # blocks recalled per layer, over the steps
    t_all0 = time.perf_counter()
    for t in range(steps):
        load_step(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        nsel_sum += nsel_log
    t_all = time.perf_counter() - t_all0
    times.sort()
    # roofline of the decode attention kernel: one eager step with events
    load_step(steps - 1)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
    one_step(ev)
    torch.cuda.synchronize()
    n_sel = nsel_log.cpu()
    n_ctx_last = n0 + steps
    l0 = H.local_start(sh, n_ctx_last - 1)
    keys = min(sh.n_init, n_ctx_last - 1) + (n_ctx_last - l0)
    byt = float(((n_sel.sum().item() * bs) + keys * L * bt) * hk * D * 2 * 2)       # K and V, bf16
    attn_ms = sum(a.elapsed_time(b) for (a, b) in ev)
    # the attention launch without the selection inside it (selection as a launch of its own)
    alone_ms, alone_byt = attn_ms, byt
    if args.decode_launches <= 2:
        one_step(ev, launches=3)
        torch.cuda.synchronize()
        alone_ms = sum(a.elapsed_time(b) for (a, b) in ev)
        alone_byt = float(((nsel_log.sum().item() * bs) + keys * L * bt) * hk * D * 2 * 2)
    score_bytes = float((nb_end_host[-1] - nb_begin) * sh.n_rep * hk * D * 2 * L * bt)
    launch_byt = byt + score_bytes if args.decode_launches == 1 else byt    # the one launch also scores
    achieved = launch_byt / (attn_ms * 1e-3) / 1e9
    per_layer_e = (nsel_sum.double().sum(dim=1) / (steps * bt)).cpu().tolist()
    mean_us = sum(times) / len(times) * 1e6
    return {
        "metric": "decode step us", "value": mean_us, "unit": "us/step", "p50_us": times[len(times) // 2] * 1e6,
        "higher_is_better": False, "steps": steps, "wall_s_incl_input_copies": t_all,
        "config": {"workload": f"{w.name}: batch {bt}, {L} layers, {n0} cached tokens, k_cap {w.k_cap}, "
                               f"dynamic cut-off with the density history on the device, new token appended per layer, KV cache {gb:.0f} GB bf16 in HBM",
                   "mean_blocks_selected": float(n_sel.float().mean()),
                   # the synthetic analogue of the paper's blocks-recalled-per-layer figure (Sec. 5.4):
                   # mean E^l over all steps and sequences, layer 0 first
                   "mean_blocks_selected_per_layer": [round(e, 3) for e in per_layer_e],
                   "launch": "hip graph replay" if graph is not None else "eager",
                   "launches_per_layer": args.decode_launches},
        "algorithmic_bytes_per_step": byt + score_bytes,
        "hbm_frac_of_step": (byt + score_bytes) / (mean_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS,
                     **traffic_fields(w.name, float(n_sel.float().mean())),
                     "kernel": ("actqkv_decode_layer launch (decode_layer_kernel: cache update + probe + scores + "
                                "selection + attention of one layer)" if args.decode_launches == 1 else
                                "actqkv_decode_select_attention launch (attn_decode_select_kernel: selection + attention)"
                                if args.decode_launches == 2 else
                                "actqkv_retrieval_attention launch, m = 1 (attn_decode_kernel)"),
                     "avg_launch_us": attn_ms * 1e3 / L, "algorithmic_mb_per_launch": launch_byt / L / 1e6,
                     "timing": "HIP events around every attention launch of one eager step",
                     "attention_alone": {"avg_launch_us": alone_ms * 1e3 / L,
                                         "achieved": alone_byt / (alone_ms * 1e-3) / 1e9,
                                         "frac": alone_byt / (alone_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                         "kernel": "actqkv_retrieval_attention launch, m = 1 (attn_decode_kernel), "
                                                   "with actqkv_select as a launch of its own"}},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3_128k")
    ap.add_argument("--n-ctx", type=int, default=0, help="override the context length (testing)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="do not use HIP graphs")
    ap.add_argument("--skip-decode", action="store_true")
    ap.add_argument("--skip-prefill", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--decode-layers", type=int, default=0, help="override the layer count (testing)")
    ap.add_argument("--decode-launches", type=int, default=2, choices=(1, 2, 3, 4),
                    help="launches per layer of a decode step: 1 = the whole layer (actqkv_decode_layer); "
                         "2 = (cache update + probe + scores), (selection + "
                         "attention); 3 = (cache update + probe + scores), selection, attention; "
                         "4 = (cache update + probe), scores, selection, attention")
    ap.add_argument("--decode-streams", type=int, default=1,
                    help="decode: the batch in this many parts, each part's layer chain on a stream of its own")
    ap.add_argument("--no-overlap", action="store_true",
                    help="prefill: one stream, strictly in window order")
    ap.add_argument("--chunk", type=int, default=32,
                    help="prefill, two streams: windows per hand-over between the streams")
    ap.add_argument("--score-chunk", type=int, default=16,
                    help="prefill: > 0 puts scoring and selection on a stream of their own, this many "
                         "windows behind the probe chain per hand-over")
    ap.add_argument("--per-window-selection", action="store_true",
                    help="prefill, with overlap: probe, score and select calls of one window each (three "
                         "streams) instead of one call per chunk of windows")
    ap.add_argument("--attention-late-cus", type=int, default=32,
                    help="compute units that join a chunk's attention once the next chunk is prepared "
                         "(a second launch that drains the same queue); 0: none")
    ap.add_argument("--attention-cus", type=int, default=224,
                    help="prefill, two streams: compute units the attention may fill")
    ap.add_argument("--layers", type=int, default=1,
                    help="prefill: > 1 runs that many layers of the workload (configs[4]: --workload c5_200k "
                         "--layers 32), each with its own inputs, and reports only that run")
    ap.add_argument("--host-cache", action="store_true",
                    help="also time the prefill pass with the cache in pinned host memory (reported as "
                         "\"host_cache\" beside the headline line)")
    ap.add_argument("--no-configs", action="store_true",
                    help="leave out the short runs of c1_8k_fp32, c2_32k and c5_200k (\"configs\" of the line)")
    ap.add_argument("--no-recall", action="store_true",
                    help="leave out the planted-block recall of the retrieval variants (\"recall\" of the line)")
    ap.add_argument("--pmc-info-dir", default=".",
                    help="--pmc-pass: folder that receives pmc_pass_<workload>.json, the description of the pass")
    ap.add_argument("--pmc-pass", action="store_true",
                    help="one calibration copy and one eager pass, for a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives, no sharding in this build).", file=sys.stderr)
        return 2

    import torch
    from paper_2502_13542_amd import binding as B
    from paper_2502_13542_amd import harness as H
    from paper_2502_13542_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.load_library()
    torch.cuda.set_device(0)
    res = {}
    if args.layers > 1:
        print(json.dumps(bench_prefill_layers(args, torch, B, H, synth)))
        return 0
    if not args.skip_prefill:
        res = bench_prefill(args, torch, B, H, synth)
        torch.cuda.empty_cache()
    if args.host_cache and not args.pmc_pass:
        hc = bench_prefill_host_cache(args, torch, B, H, synth)
        torch.cuda.empty_cache()
        if res:
            res["host_cache"] = hc
        else:
            res = hc
    if not args.skip_decode:
        dec = bench_decode(args, torch, B, H, synth)
        torch.cuda.empty_cache()
        if res:
            res["decode"] = dec
        else:
            res = dec
    headline = args.workload == "c3_128k" and not args.n_ctx and not args.pmc_pass and not args.skip_prefill
    if headline and not args.no_recall:
        log("recall of planted blocks per retrieval variant")
        res["recall"] = bench_recall(args, torch, B, H, synth)
        torch.cuda.empty_cache()
    if headline and not args.no_configs:
        res["configs"] = bench_other_configs(args, torch, B, H, synth)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
