#!/usr/bin/env python3
"""Benchmark of the retrieval-attention hot path on one MI355X.

A step is one whole single-layer windowed prefill of the workload's context: for every
window, actqkv_build_probe -> actqkv_score_blocks -> actqkv_select ->
actqkv_retrieval_attention, in order, on one stream, with all inputs resident in HBM.
The default workload is the benchmark's configs[2] (LLaMA3-8B layer, 128K tokens, window
512, top-k 32 with the dynamic cut-off): the one its metric "tokens/s per layer @128K"
is quoted on.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0


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
            "sample": f"windows {list(sample)} of {w.n_windows} (all steps of the path, all rows), "
                      f"{t_total:.1f} s of numpy fp64"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3_128k")
    ap.add_argument("--n-ctx", type=int, default=0, help="override the context length (testing)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    if args.n_ctx:
        w = synth.scaled(w, n_ctx=args.n_ctx)
    sh = w.shape

    # ---- inputs, generated on the device and resident in HBM before timing starts
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
    cut0 = None if plan.cutoff is None else plan.cutoff.clone()
    out = torch.zeros_like(q)
    n_win = plan.n_windows
    nsel_log = torch.zeros(n_win, dtype=torch.int32, device=dev)

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_win)] for _ in range(args.steps)]

    def one_step(events=None):
        runner.reset()
        if cut0 is not None:
            plan.cutoff.copy_(cut0)
        nb_begin = sh.n_init // sh.block_size
        for t in range(n_win):
            w0, rows = plan.w0[t], plan.rows[t]
            qw = q[w0:w0 + rows]
            cut = None if plan.cutoff is None else plan.cutoff[t:t + 1]
            nb_cap = min(max(plan.nb_end_host[t], nb_begin), runner.nb_capacity)
            B.build_probe(runner.cs, 1, rows, qw, runner.stats, True, runner.probe, runner.probe_kv,
                          runner.probe_norm, None, runner.workspace)
            B.score_blocks(runner.cs, 1, runner.probe_kv, runner.probe_norm, repd, 0, nb_cap, nb_begin,
                           plan.nb_end[t:t + 1], runner.scores, runner.score_stride)
            B.select(1, runner.scores, runner.score_stride, nb_cap, nb_begin, plan.nb_end[t:t + 1],
                     w.k_cap, cut, runner.idx, nsel_log[t:t + 1], None, None)
            if events is not None:
                events[t][0].record()
            B.retrieval_attention(runner.cs, 1, rows, qw, kc, vc, 0, runner.nb_capacity,
                                  plan.n_ctx[t:t + 1], runner.idx, nsel_log[t:t + 1], w.k_cap,
                                  out[w0:w0 + rows], None, runner.workspace)
            if events is not None:
                events[t][1].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- roofline of the dominant kernel: the prefill attention launch
    n_sel = nsel_log.cpu().tolist()
    flops = 0.0
    for t in range(n_win):
        flops += attention_flops(sh, plan.w0[t], plan.rows[t], n_sel[t], H.local_start(sh, plan.w0[t]))
    attn_ms = sum(a.elapsed_time(b) for step in ev for (a, b) in step)
    n_launch = args.steps * n_win
    avg_us = attn_ms * 1e3 / n_launch
    achieved = (flops * args.steps) / (attn_ms * 1e-3) / 1e12
    tokens_per_s = w.n_ctx * args.steps / elapsed
    res = {
        "metric": "prefill retrieval-attn tokens/s per layer @128K" if not args.n_ctx and
                  args.workload == "c3_128k" else f"prefill retrieval-attn tokens/s per layer ({w.name})",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: 1 sequence, 1 layer, H{sh.n_q_heads}/Hk{sh.n_kv_heads}/D{sh.head_dim}, "
                               f"{w.n_ctx} tokens, window {w.window}, block {sh.block_size} x {sh.n_rep} rep keys, "
                               f"n_init {sh.n_init}, n_local {sh.n_local}, k_cap {w.k_cap}, "
                               f"cut-off {'on' if w.cutoff else 'off'}",
                   "windows": n_win, "mean_blocks_selected": sum(n_sel) / max(n_win, 1)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
                     "kernel": "actqkv_retrieval_attention launch (attn_prefill_mfma_kernel + split combine)",
                     "avg_launch_us": avg_us, "algorithmic_gflop_per_launch": flops / n_win / 1e9,
                     "attention_share_of_step": attn_ms / 1e3 / elapsed},
    }
    if not args.no_cpu_baseline:
        T = n_win
        sample = sorted({max(T // 4, 0), T // 2, (3 * T) // 4, T - 1})
        res["cpu_baseline"] = cpu_baseline(w, q, k, v, rep, cutoffs, sample)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
