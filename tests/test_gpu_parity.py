"""GPU parity: every entry point of libactqkv.so against the CPU oracle, element by
element, on the same seeded inputs.  All calls go through the C ABI (ctypes binding)."""
import ctypes
import math

import numpy as np
import pytest
import torch

from oracle import actqkv_oracle as orc
from paper_2502_13542_amd import binding as B
from paper_2502_13542_amd import harness as H
from paper_2502_13542_amd import synth
from paper_2502_13542_amd.synth import LayerShape

from parity_utils import (TOL_BUDGET, TOL_OUT, TOL_PROBE, TOL_SCORE, TOL_THETA, TOL_WEIGHT,
                          check_selection, f64, oracle_windows, out_error, rel_to_max)

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def run_prefill_case(w: synth.Workload, attend=None, use_cutoff=None, layer=0):
    """Runs a whole single-sequence prefill on the GPU and in the oracle and compares
    every window's probe, weights, scores, density, budget and selection, and the
    attention output of the windows in `attend` (all if None)."""
    sh = w.shape
    _say(f"[case] {w.name} N={w.n_ctx} m={w.window} k_cap={w.k_cap} dtype={sh.dtype} seed={w.seed}")
    q, k, v = synth.gen_layer(w, "cpu", layer)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    n_win = w.n_windows
    use_cutoff = w.cutoff if use_cutoff is None else use_cutoff
    cutoffs = None
    if use_cutoff:
        cutoffs = []
        for t in range(n_win):
            b, e = H.eligible_range(sh, t * w.window)
            cutoffs.append(synth.cutoff_state(w, e - b, t, layer))
    nb_cap = w.n_blocks
    qd, kc, vc = q.to(DEV), H.blocked_k(k.to(DEV), sh, nb_cap), H.blocked_vt(v.to(DEV), sh, nb_cap)
    repd = torch.zeros(nb_cap, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=DEV)
    repd[: rep.shape[0]] = rep.to(DEV)
    runner = H.LayerRunner(sh, 1, w.window, nb_cap, w.k_cap, DEV)
    plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, DEV)
    out = torch.zeros_like(qd)
    rec = H.prefill_layer(runner, plan, qd, kc, vc, repd, out, record=range(n_win))
    torch.cuda.synchronize()
    want = oracle_windows(q, k, v, rep, sh, w.window, w.k_cap, cutoffs, attend)
    n_exact = 0
    worst = 0.0
    for t, res in enumerate(want):
        g = rec[t]
        assert rel_to_max(g["probe"], res["probe"]) < TOL_PROBE, f"probe, window {t}"
        assert rel_to_max(g["weights"], res["weights"]) < TOL_WEIGHT, f"weights, window {t}"
        assert abs(float(g["weights"].sum()) - 1.0) < 1e-4
        pn = float(np.linalg.norm(res["probe"]))
        assert abs(float(g["probe_norm"]) - pn) < TOL_PROBE * pn
        elig = res["eligible"]
        if elig:
            gs = f64(g["scores"])[elig]
            assert np.abs(gs - res["scores"]).max() < TOL_SCORE, f"scores, window {t}"
            assert abs(float(g["theta"]) - res["theta"]) < TOL_THETA, f"theta, window {t}"
            assert abs(float(g["budget"]) - res["budget"]) <= TOL_BUDGET * max(1.0, abs(res["budget"]))
            if cutoffs is not None:
                assert abs(float(g["budget_after"]) - res["b_kv_after"]) <= TOL_BUDGET * max(
                    1.0, abs(cutoffs[t][0]))
        gi = g["idx"].cpu().tolist()
        gn = int(g["n_sel"])
        same = check_selection(gi, gn, res, w.k_cap)
        n_exact += int(same)
        if "out" in res:
            w0 = res["w0"]
            ref = res["out"]
            if not same:  # a legitimate near-tie swap: compare against the oracle on the GPU's set
                ref = orc.retrieval_attention_window(f64(q[w0:w0 + w.window]), f64(k), f64(v), w0,
                                                     gi[:gn], sh.n_init, sh.n_local, sh.block_size,
                                                     sh.group)
            err = out_error(out[w0:w0 + ref.shape[0]], ref)
            worst = max(worst, err)
            assert err < TOL_OUT[sh.dtype], f"attention output, window {t}: {err}"
    _say(f"[case] {w.name}: {n_win} windows, {n_exact} identical selections, worst out err {worst:.3e}")
    return n_exact, n_win


def test_c1_fp32_full_parity():
    # configs[0] as it is: every window, every row
    n_exact, n_win = run_prefill_case(synth.WORKLOADS["c1_8k_fp32"])
    assert n_exact >= n_win - 2


def test_c1_fp32_with_cutoff_and_ragged_tail():
    w = synth.scaled(synth.WORKLOADS["c1_8k_fp32"], n_ctx=4096 + 77, cutoff=True, k_cap=8)
    run_prefill_case(w)


def test_llama_shape_bf16_small():
    w = synth.scaled(synth.WORKLOADS["c2_32k"], n_ctx=6144, name="c2_reduced")
    run_prefill_case(w, attend=[0, 1, 5, 11])


def test_llama_shape_bf16_cutoff_ragged():
    w = synth.scaled(synth.WORKLOADS["c3_128k"], n_ctx=8192 + 300, k_cap=32, name="c3_reduced")
    run_prefill_case(w, attend=[0, 3, 16])


def test_c2_32k_full_size_sampled_windows():
    # configs[1] at full size, in the launch configuration bench.py uses; the oracle checks the
    # probe and the selection of every window and the attention of a spread of windows
    run_prefill_case(synth.WORKLOADS["c2_32k"], attend=[0, 1, 7, 31, 63])


def test_c3_128k_full_size_sampled_windows():
    # configs[2] (the benchmarked workload) at full size with the dynamic cut-off
    run_prefill_case(synth.WORKLOADS["c3_128k"], attend=[2, 64, 255])


def test_c5_200k_full_size_sampled_windows():
    # configs[4] at full size in its ragged form (200,000 tokens: the last window has 320 rows),
    # its last layer (3 % outlier tokens): every window's probe, scores, density, budget and
    # selection, and the attention of a spread of windows
    run_prefill_case(synth.scaled(synth.WORKLOADS["c5_200k"], n_ctx=200000), attend=[5, 211, 390], layer=31)


def test_c3_128k_two_stream_pipeline_as_benchmarked():
    """configs[2] at full size in the schedules of PrefillPipeline, the last one being the one
    bench.py times: (1) three streams, calls of one window each: probes, then scoring and
    selection 16 windows behind them, then the attention of up to 32 windows per launch with 224
    of the 256 compute units; (2) the same with scoring and selection on the probes' stream;
    (3) one probe, one score, one select and one attention call per 32 windows; (4) the same with a
    second team of attention workgroups per chunk.  Every window's
    selection must equal the one found in window order; the attention of sampled windows is
    checked against the oracle and all rows against the window-order result."""
    w = synth.WORKLOADS["c3_128k"]
    sh = w.shape
    _say(f"[case] {w.name} two streams N={w.n_ctx} seed={w.seed}")
    q, k, v = synth.gen_layer(w, "cpu", 0)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    cutoffs = []
    for t in range(w.n_windows):
        b, e = H.eligible_range(sh, t * w.window)
        cutoffs.append(synth.cutoff_state(w, e - b, t, 0))
    qd, kc, vc = q.to(DEV), H.blocked_k(k.to(DEV), sh, w.n_blocks), H.blocked_vt(v.to(DEV), sh, w.n_blocks)
    repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=DEV)
    repd[: rep.shape[0]] = rep.to(DEV)
    runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, DEV)
    plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, DEV)
    bud0 = plan.budget.clone()
    pipe = H.PrefillPipeline(runner, plan)
    out_order, out_two = torch.zeros_like(qd), torch.zeros_like(qd)
    pipe.run(qd, kc, vc, repd, out_order, overlap=False)
    torch.cuda.synchronize()
    idx_order, nsel_order = pipe.idx.clone(), pipe.n_sel.clone()
    runner.reset()
    plan.budget.copy_(bud0)
    pipe.idx.fill_(-1)
    pipe.run(qd, kc, vc, repd, out_two, overlap=True, attention_cus=224)
    torch.cuda.synchronize()
    assert torch.equal(pipe.idx, idx_order) and torch.equal(pipe.n_sel, nsel_order)
    # the same with scoring and selection kept on the probes' stream
    out_b = torch.zeros_like(qd)
    runner.reset()
    plan.budget.copy_(bud0)
    pipe.idx.fill_(-1)
    pipe.run(qd, kc, vc, repd, out_b, overlap=True, score_chunk=0, attention_cus=224)
    torch.cuda.synchronize()
    assert torch.equal(pipe.idx, idx_order) and torch.equal(pipe.n_sel, nsel_order)
    assert torch.equal(out_b, out_two)
    diff = (out_two.float() - out_order.float()).abs().max().item()
    scale = out_order.float().abs().max().item()
    assert diff <= TOL_OUT["bf16"] * scale, f"two streams vs window order: {diff}"
    # the benchmarked schedule: one probe, one score, one select and one attention call per 32
    # windows.  The statistics are merged from per-window moments, so probes differ from the
    # window-order ones in rounding; selections may differ only where blocks all but tie.
    out_c = torch.zeros_like(qd)
    runner.reset()
    plan.budget.copy_(bud0)
    pipe.idx.fill_(-1)
    pipe.run(qd, kc, vc, repd, out_c, overlap=True, batched=True, attention_cus=224)
    torch.cuda.synchronize()
    assert torch.equal(pipe.n_sel, nsel_order)
    differ = [t for t in range(w.n_windows) if not torch.equal(pipe.idx[t], idx_order[t])]
    assert len(differ) <= w.n_windows // 50, f"{len(differ)} windows select differently: {differ[:8]}"
    same_rows = torch.ones(w.n_ctx, dtype=torch.bool)
    for t in differ:
        same_rows[plan.w0[t]:plan.w0[t] + plan.rows[t]] = False
    diff_c = (out_c.float() - out_order.float()).abs().amax(dim=(1, 2)).cpu()[same_rows].max().item()
    assert diff_c <= TOL_OUT["bf16"] * scale, f"chunked calls vs window order: {diff_c}"
    # (4) the same with a second team of 32 attention workgroups that joins each chunk's queue
    # once the next chunk is prepared: the same items, whoever takes them, so the same bits;
    # twice in a row, so that a queue left dirty would show
    for rep_run in range(2):
        out_d = torch.zeros_like(qd)
        runner.reset()
        plan.budget.copy_(bud0)
        idx_c = pipe.idx.clone()
        pipe.idx.fill_(-1)
        pipe.run(qd, kc, vc, repd, out_d, overlap=True, batched=True, late_cus=32, attention_cus=224)
        torch.cuda.synchronize()
        assert torch.equal(pipe.idx, idx_c) and torch.equal(pipe.n_sel, nsel_order)
        assert torch.equal(out_d, out_c), f"two teams of attention workgroups, run {rep_run}"
        assert not pipe.ws_attn[:8192].any() and not pipe.ws_attn_b[:8192].any()   # tickets and queue back at zero
    out_two = out_c
    attend = [3, 130, 255]
    want = oracle_windows(q, k, v, rep, sh, w.window, w.k_cap, cutoffs, attend)
    worst = 0.0
    for t in attend:
        res = want[t]
        gi, gn = pipe.idx[t].cpu().tolist(), int(pipe.n_sel[t])
        ref = res["out"]
        if not check_selection(gi, gn, res, w.k_cap):
            ref = orc.retrieval_attention_window(f64(q[res["w0"]:res["w0"] + w.window]), f64(k), f64(v),
                                                 res["w0"], gi[:gn], sh.n_init, sh.n_local,
                                                 sh.block_size, sh.group)
        err = out_error(out_two[res["w0"]:res["w0"] + ref.shape[0]], ref)
        worst = max(worst, err)
        assert err < TOL_OUT["bf16"], f"attention output, window {t}: {err}"
    _say(f"[case] {w.name} two streams: selections equal, max |two - order| {diff:.3e}; chunked calls: "
         f"{len(differ)} windows with a near-tie swap, max |chunked - order| {diff_c:.3e}, worst out err {worst:.3e}")


@pytest.mark.parametrize("hq,hkv,d,dtype", [(28, 4, 128, "bf16"), (6, 2, 64, "fp32"), (12, 4, 128, "bf16")])
def test_group_sizes_that_do_not_divide_eight(hq, hkv, d, dtype):
    """7 query heads per KV head (the second model of Sec. 5.1 has 28 and 4), and 3."""
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    w = synth.Workload(f"group_{hq // hkv}", sh, 3072 + 100, 512 if dtype == "bf16" else 256, 6, True,
                       4242 + hq, outlier_rate=0.02, outlier_kind="boost" if dtype == "fp32" else "student_t",
                       n_planted=4)
    run_prefill_case(w, attend=[0, 2, 6])


@pytest.mark.parametrize("n_init,n_local", [(0, 256), (128, 0), (256, 128), (0, 0), (512, 1024)])
def test_geometry_variants(n_init, n_local):
    sh = LayerShape(4, 2, 64, 128, 2, n_init, n_local, "fp32")
    w = synth.Workload(f"geom_{n_init}_{n_local}", sh, 2048 + 50, 128, 4, False, 99 + n_init + n_local,
                       outlier_rate=0.03, outlier_kind="boost", n_planted=3)
    run_prefill_case(w)


@pytest.mark.parametrize("m,n_ctx,attend", [(2048, 3 * 2048 + 300, [1, 3]), (4096, 2 * 4096 + 128, [1, 2])])
def test_windows_larger_than_the_benchmarked_one(m, n_ctx, attend):
    """Windows of 2048 tokens (16 key tiles of the window itself: still the matrix-core kernel) and
    of 4096 (more tiles than its tile table holds: the row kernel), bf16, ragged last window;
    probes, scores and selections of every window, attention of the windows in `attend`."""
    sh = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    w = synth.Workload(f"window_{m}", sh, n_ctx, m, 6, True, 4242 + m, n_planted=4)
    run_prefill_case(w, attend=attend)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_probe_with_statistics_used_as_they_are(dtype):
    """actqkv_build_probe without ACTQKV_STATS_UPDATE: the bias of a window against the statistics
    of the windows before it only, and the record left untouched."""
    m, hq, hkv, d = 256, 8, 2, 64
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(5)
    q = (torch.randn(2 * m, hq, d, generator=g) * 1.2 + 0.4).to(td)
    q[m + 7, :, 3] *= 10.0
    qd = q.to(DEV)
    runner = H.LayerRunner(sh, 1, m, 8, 4, DEV)
    wts = torch.zeros(1, m, device=DEV)
    B.build_probe(cs, 1, m, qd[:m], runner.stats, True, runner.probe, runner.probe_kv, runner.probe_norm, None,
                  runner.workspace)
    torch.cuda.synchronize()
    before = runner.stats.clone()
    B.build_probe(cs, 1, m, qd[m:], runner.stats, False, runner.probe, runner.probe_kv, runner.probe_norm, wts,
                  runner.workspace)
    torch.cuda.synchronize()
    assert torch.equal(runner.stats, before)
    stats = orc.RunningStats(hq * d)
    z_bar, sigma2 = stats.update(f64(q[:m]).reshape(m, -1))
    qw = f64(q[m:]).reshape(m, -1)
    probe, weights = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2))
    assert rel_to_max(runner.probe[0], probe) < TOL_PROBE and rel_to_max(wts[0], weights) < TOL_WEIGHT
    assert int(torch.argmax(wts[0])) == 7


def test_probe_of_the_largest_window():
    """actqkv_build_probe with m = 8192, the largest window the library takes, against the oracle
    (statistics of two windows, bias, weights, probe)."""
    m, hq, hkv, d = 8192, 4, 2, 64
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, "fp32")
    cs = B.c_shape(sh)
    g = torch.Generator().manual_seed(8192)
    q = torch.randn(2 * m, hq, d, generator=g) * 1.3 + 0.2
    q[torch.randperm(2 * m, generator=g)[:200], :, 5] *= 9.0                    # outlier tokens
    qd = q.to(DEV)
    runner = H.LayerRunner(sh, 1, m, 8, 4, DEV)
    wts = torch.zeros(1, m, device=DEV)
    stats = orc.RunningStats(hq * d)
    for t in range(2):
        B.build_probe(cs, 1, m, qd[t * m:(t + 1) * m], runner.stats, True, runner.probe, runner.probe_kv,
                      runner.probe_norm, wts, runner.workspace)
        torch.cuda.synchronize()
        qw = f64(q[t * m:(t + 1) * m]).reshape(m, -1)
        z_bar, sigma2 = stats.update(qw)
        probe, weights = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2))
        assert rel_to_max(runner.probe[0], probe) < TOL_PROBE, f"probe, window {t}"
        assert rel_to_max(wts[0], weights) < TOL_WEIGHT, f"weights, window {t}"
        assert abs(float(wts.sum()) - 1.0) < 1e-4
    assert lib_rejects_window(cs, m + 1)


def lib_rejects_window(cs, m):
    lib = B.load_library()
    rc = lib.actqkv_build_probe(ctypes.byref(cs), 1, m, 16, 16, 1, 16, 16, 16, None, 16, 1 << 30, None)
    return rc == -2


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 64)])
def test_attention_over_the_largest_selection(dtype, d):
    """A window that retrieves 64 blocks (the largest k_cap), in a batch of two windows of one
    sequence with different selections; the second one's idx holds out-of-range and negative
    entries, which count as empty blocks (device-side values cannot cause an access out of bounds)."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    m, k_cap, n_tok = 256, 64, 80 * 128 + 2 * 256
    nb = n_tok // 128
    g = torch.Generator().manual_seed(64 + d)
    q = torch.randn(2 * m, 8, d, generator=g).to(td)
    k = torch.randn(n_tok, 2, d, generator=g).to(td)
    v = torch.randn(n_tok, 2, d, generator=g).to(td)
    w0 = [n_tok - 2 * m, n_tok - m]
    kc, vc = H.blocked_k(k.to(DEV), sh, nb), H.blocked_vt(v.to(DEV), sh, nb)
    b, e = H.eligible_range(sh, w0[0])
    sel = (torch.randperm(e - b, generator=g)[:k_cap] + b).tolist()
    idx = torch.full((2, k_cap), -1, dtype=torch.int32)
    idx[0] = torch.tensor(sel, dtype=torch.int32)
    idx[1, :5] = torch.tensor([3, 10 ** 6, -7, 2, nb + 1], dtype=torch.int32)      # only blocks 3 and 2 exist
    n_sel = torch.tensor([k_cap, 5], dtype=torch.int32)
    n_ctx = torch.tensor([w0[0] + m, w0[1] + m], dtype=torch.int32)
    out = torch.zeros(2 * m, 8, d, dtype=td, device=DEV)
    ws = torch.zeros(B.workspace_bytes(cs, 2, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    B.retrieval_attention(cs, 2, m, q.to(DEV), kc, vc, 0, nb, n_ctx.to(DEV), idx.to(DEV), n_sel.to(DEV), k_cap, out,
                          None, ws)
    torch.cuda.synchronize()
    for i, chosen in enumerate((sel, [3, 2])):
        ref = orc.retrieval_attention_window(f64(q[i * m:(i + 1) * m]), f64(k), f64(v), w0[i], chosen, sh.n_init,
                                             sh.n_local, 128, sh.group)
        err = out_error(out[i * m:(i + 1) * m], ref)
        assert err < TOL_OUT[dtype], f"window {i}: {err}"


@pytest.mark.parametrize("dtype,d,m,n_ctx", [("bf16", 128, 2, 700), ("bf16", 128, 33, 1500), ("fp32", 64, 3, 500)])
def test_tiny_windows(dtype, d, m, n_ctx):
    """Windows of 2, 3 and 33 tokens (most rows of a query tile idle, a ragged last window)."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    w = synth.Workload(f"tiny_window_{m}", sh, n_ctx, m, 2, True, 77 + m, n_planted=2)
    run_prefill_case(w, attend=[0, w.n_windows // 2, w.n_windows - 1])


@pytest.mark.parametrize("per_head", [False, True])
def test_queued_attention_equals_one_call_per_window(per_head):
    """32 windows of one sequence in ONE attention call (work items drawn from a queue, longest
    first) against 32 calls of one window each, with a selection per sequence and with one per
    (sequence, KV head); two runs in a row on one workspace give the same bits."""
    sh = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    m, nw, k_cap = 512, 32, 8
    n_tok = (nw + 1) * m
    nb = n_tok // 128
    g = torch.Generator().manual_seed(31 + per_head)
    q = torch.randn(nw * m, 8, 128, generator=g).to(torch.bfloat16).to(DEV)
    kc = torch.randn(nb, 2, 128, 128, generator=g).to(torch.bfloat16).to(DEV)
    vc = torch.randn(nb, 2, 128, 128, generator=g).to(torch.bfloat16).to(DEV)
    rows = nw * (2 if per_head else 1)
    idx = torch.full((rows, k_cap), -1, dtype=torch.int32)
    n_sel = torch.randint(0, k_cap + 1, (rows,), generator=g, dtype=torch.int32)
    n_ctx = torch.tensor([(i + 2) * m for i in range(nw)], dtype=torch.int32)
    for r in range(rows):
        w0 = (r // (2 if per_head else 1) + 1) * m
        b, e = H.eligible_range(sh, w0)
        idx[r, : int(n_sel[r])] = (torch.randperm(e - b, generator=g)[: int(n_sel[r])] + b).int()
    idx, n_sel, n_ctx = idx.to(DEV), n_sel.to(DEV), n_ctx.to(DEV)
    ws = torch.zeros(B.workspace_bytes(cs, nw, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    step = 2 if per_head else 1
    ref = torch.zeros_like(q)
    for i in range(nw):
        B.retrieval_attention(cs, 1, m, q[i * m:(i + 1) * m], kc, vc, 0, nb, n_ctx[i:i + 1],
                              idx[i * step:(i + 1) * step], n_sel[i * step:(i + 1) * step], k_cap,
                              ref[i * m:(i + 1) * m], None, ws, per_head=per_head)
    # on 192 of the chip's compute units: the windows' items go through the queue
    side = torch.cuda.Stream(device=DEV)
    outs = []
    for run in range(2):
        out = torch.zeros_like(q)
        if per_head:
            B.retrieval_attention(cs, nw, m, q, kc, vc, 0, nb, n_ctx, idx, n_sel, k_cap, out, None, ws,
                                  per_head=per_head)
        else:
            B.retrieval_attention_teams(cs, nw, m, q, kc, vc, 0, nb, n_ctx, idx, n_sel, k_cap, out, None, ws,
                                        192, 0)
        torch.cuda.synchronize()
        # (a one-window call cuts its key tiles into pieces and merges partial results: another
        # summation order, so the last bits of a bf16 output may differ)
        err = ((out.float() - ref.float()).abs().amax(dim=-1) / ref.float().abs().amax(dim=-1)).max().item()
        assert err < 1e-2, f"run {run}: {err}"
        assert not ws[:8192].any()
        outs.append(out)
    assert torch.equal(outs[0], outs[1])              # whoever takes an item, the same bits
    if not per_head:
        # two teams of workgroups, the second one on the same stream (it then finds the queue empty)
        # and on a stream of its own (it then draws beside the first team): the same bits, and the
        # queue back at zero
        for late_stream in (None, side):
            out = torch.zeros_like(q)
            if late_stream is not None:
                late_stream.wait_stream(torch.cuda.current_stream())
            B.retrieval_attention_teams(cs, nw, m, q, kc, vc, 0, nb, n_ctx, idx, n_sel, k_cap, out, None, ws,
                                        192, 32, None, late_stream)
            torch.cuda.synchronize()
            assert torch.equal(out, outs[0]) and not ws[:8192].any()


def _lse_reference(q_row, k, pos, group):
    """log sum exp of the scaled logits of one query row [H][D] over the keys at `pos`, per head."""
    q_row, pos = f64(q_row), np.asarray(pos)
    out = np.zeros(q_row.shape[0])
    for h in range(q_row.shape[0]):
        z = f64(k[pos, h // group]) @ q_row[h] / math.sqrt(q_row.shape[1])
        out[h] = z.max() + math.log(np.exp(z - z.max()).sum())
    return out


@pytest.mark.parametrize("dtype,d,m,nw", [("bf16", 128, 512, 1),     # key tiles cut into pieces, merged
                                          ("bf16", 128, 512, 8),     # whole query tiles per workgroup
                                          ("fp32", 64, 256, 2),      # row kernel
                                          ("bf16", 128, 1, 3),       # decode, several workgroups per pair
                                          ("bf16", 128, 1, 200),     # decode, one workgroup per pair
                                          ("fp32", 64, 1, 3)])       # decode, row kernel
def test_log_sum_exp_output(dtype, d, m, nw):
    """The optional lse output [batch][H][m] of every attention kernel: the natural-log sum of the
    exponentials of the scaled logits over exactly the keys a row sees."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    k_cap, base = 4, 9 * 128 + 40
    n_tok = base + nw * m
    nb = (n_tok + 127) // 128
    g = torch.Generator().manual_seed(m + nw)
    q = torch.randn(nw * m, 8, d, generator=g).to(td)
    k = torch.randn(nb * 128, 2, d, generator=g).to(td)
    v = torch.randn(nb * 128, 2, d, generator=g).to(td)
    kc, vc = H.blocked_k(k.to(DEV), sh, nb), H.blocked_vt(v.to(DEV), sh, nb)
    w0 = [base + i * m for i in range(nw)]
    idx = torch.full((nw, k_cap), -1, dtype=torch.int32)
    n_sel = torch.zeros(nw, dtype=torch.int32)
    for i in range(nw):
        b, e = H.eligible_range(sh, w0[i])
        n_sel[i] = min(k_cap, e - b, 1 + i % k_cap)
        idx[i, : int(n_sel[i])] = (torch.randperm(e - b, generator=g)[: int(n_sel[i])] + b).int()
    n_ctx = torch.tensor([w + m for w in w0], dtype=torch.int32)
    out = torch.zeros(nw * m, 8, d, dtype=td, device=DEV)
    lse = torch.full((nw, 8, m), float("nan"), device=DEV)
    ws = torch.zeros(B.workspace_bytes(cs, nw, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    B.retrieval_attention(cs, nw, m, q.to(DEV), kc, vc, 0, nb, n_ctx.to(DEV), idx.to(DEV), n_sel.to(DEV), k_cap,
                          out, lse, ws)
    torch.cuda.synchronize()
    lse = lse.cpu().numpy()
    assert np.isfinite(lse).all()
    tol = 2e-5 if dtype == "fp32" else 2e-3            # bf16 inputs are exact; the logits are fp32 sums either way
    for i in range(0, nw, max(nw // 5, 1)):
        chosen = idx[i, : int(n_sel[i])].tolist()
        for r in sorted({0, m // 3, m - 1}):
            pos = orc.key_positions(w0[i], w0[i] + r, chosen, sh.n_init, sh.n_local, 128)
            ref = _lse_reference(q[i * m + r], k, pos, sh.group)
            assert np.abs(lse[i, :, r] - ref).max() < tol * max(1.0, np.abs(ref).max()), f"window {i} row {r}"


@pytest.mark.parametrize("dtype,d,m,nw", [("bf16", 128, 256, 1), ("bf16", 128, 256, 40), ("fp32", 64, 128, 2),
                                          ("bf16", 128, 1, 4), ("fp32", 64, 1, 2)])
def test_softmax_scale_of_the_caller(dtype, d, m, nw):
    """shape.softmax_scale other than 1/sqrt(D), in every attention kernel."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    scale = 0.031
    cs = B.c_shape(sh, softmax_scale=scale)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    k_cap, base = 3, 7 * 128 + 19
    n_tok = base + nw * m
    nb = (n_tok + 127) // 128
    g = torch.Generator().manual_seed(3 * m + nw)
    q = (torch.randn(nw * m, 8, d, generator=g) * 2.0).to(td)
    k = torch.randn(nb * 128, 2, d, generator=g).to(td)
    v = torch.randn(nb * 128, 2, d, generator=g).to(td)
    kc, vc = H.blocked_k(k.to(DEV), sh, nb), H.blocked_vt(v.to(DEV), sh, nb)
    w0 = [base + i * m for i in range(nw)]
    idx = torch.tensor([[2, 4, 5]] * nw, dtype=torch.int32)
    n_sel = torch.full((nw,), 3, dtype=torch.int32)
    n_ctx = torch.tensor([w + m for w in w0], dtype=torch.int32)
    out = torch.zeros(nw * m, 8, d, dtype=td, device=DEV)
    ws = torch.zeros(B.workspace_bytes(cs, nw, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    B.retrieval_attention(cs, nw, m, q.to(DEV), kc, vc, 0, nb, n_ctx.to(DEV), idx.to(DEV), n_sel.to(DEV), k_cap,
                          out, None, ws)
    torch.cuda.synchronize()
    for i in sorted({0, nw // 2, nw - 1}):
        for r in sorted({0, m - 1}):
            pos = orc.key_positions(w0[i], w0[i] + r, [2, 4, 5], sh.n_init, sh.n_local, 128)
            ref = orc.attention_rows(f64(q[i * m + r])[None], f64(k), f64(v), pos, sh.group, scale)[0]
            default = orc.attention_rows(f64(q[i * m + r])[None], f64(k), f64(v), pos, sh.group)[0]
            assert out_error(out[i * m + r], ref) < TOL_OUT[dtype], f"window {i} row {r}"
            assert out_error(default, ref) > 5 * TOL_OUT[dtype]       # the scale matters on these inputs


def test_variance_floor_of_the_caller():
    """shape.var_eps: a channel that never varies has variance 0, floored at var_eps (Eq. (7))."""
    m, hq, hkv, d = 128, 4, 2, 64
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, "fp32")
    eps = 0.25
    cs = B.c_shape(sh, var_eps=eps)
    g = torch.Generator().manual_seed(12)
    q = torch.randn(2 * m, hq, d, generator=g)
    q[:m, 1, 9] = 0.75                                      # constant in the first window: variance 0 after it
    qd = q.to(DEV)
    runner = H.LayerRunner(sh, 1, m, 8, 4, DEV)
    wts = torch.zeros(1, m, device=DEV)
    B.build_probe(cs, 1, m, qd[:m], runner.stats, True, runner.probe, runner.probe_kv, runner.probe_norm, None,
                  runner.workspace)
    B.build_probe(cs, 1, m, qd[m:], runner.stats, False, runner.probe, runner.probe_kv, runner.probe_norm, wts,
                  runner.workspace)
    torch.cuda.synchronize()
    stats = orc.RunningStats(hq * d)
    z_bar, sigma2 = stats.update(f64(q[:m]).reshape(m, -1))
    assert sigma2[1 * d + 9] < 1e-12
    qw = f64(q[m:]).reshape(m, -1)
    probe, weights = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2, eps))
    other, _ = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2, 1e-12))
    assert rel_to_max(runner.probe[0], probe) < TOL_PROBE and rel_to_max(wts[0], weights) < TOL_WEIGHT
    assert rel_to_max(other, probe) > 100 * TOL_PROBE       # the floor matters on these inputs


@pytest.mark.parametrize("n_rep,dtype,d", [(1, "bf16", 128), (6, "bf16", 128), (16, "fp32", 64)])
def test_other_numbers_of_representative_keys(n_rep, dtype, d):
    """1, 6 and 16 representative keys per block (the scoring kernels walk them four at a time):
    a prefill against the oracle, the decode scoring launch against the scoring kernel, and the
    cache update's choice of representatives."""
    sh = LayerShape(8, 2, d, 128, n_rep, 128, 256, dtype)
    w = synth.Workload(f"rep_{n_rep}", sh, 2048 + 60, 256, 4, True, 600 + n_rep, n_planted=3)
    run_prefill_case(w, attend=[w.n_windows - 1])
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(n_rep)
    n, nb = 1000, 9
    k = torch.randn(n, 2, d, generator=g).to(td)
    v = torch.randn(n, 2, d, generator=g).to(td)
    kc = torch.zeros(1, nb, 2, 128, d, dtype=td, device=DEV); vc = torch.zeros(1, nb, 2, d, 128, dtype=td, device=DEV)
    rep = torch.zeros(1, nb, n_rep, 2, d, dtype=td, device=DEV)
    B.append_kv(cs, 1, n, k.to(DEV), v.to(DEV), torch.zeros(1, dtype=torch.int32, device=DEV), kc, vc, 0, rep, 0, nb)
    torch.cuda.synchronize()
    want = orc.representative_keys(k.float().numpy(), 128, n_rep)
    assert np.array_equal(rep[0, : want.shape[0]].float().cpu().numpy(), want)
    q = torch.randn(1, 1, 8, d, generator=g).to(td).to(DEV)
    nb_end = torch.tensor([7], dtype=torch.int32, device=DEV)
    r = H.LayerRunner(sh, 1, 1, nb, 4, DEV)
    B.build_probe(cs, 1, 1, q, None, False, r.probe, r.probe_kv, r.probe_norm, None, r.workspace)
    B.score_blocks(cs, 1, r.probe_kv, r.probe_norm, rep, 0, nb, 1, nb_end, r.scores, r.score_stride)
    torch.cuda.synchronize()
    a = r.scores[0, 1:7].clone()
    r.scores.zero_()
    B.decode_retrieve(cs, 1, q, None, None, None, None, None, 0, rep, 0, nb, 1, nb_end, None, None, None, r.scores,
                      r.score_stride, 4, None, None, r.idx, r.n_sel, None, None)
    torch.cuda.synchronize()
    assert torch.allclose(r.scores[0, 1:7], a, rtol=2e-6, atol=1e-7)
    ref = orc.block_scores(f64(q[0, 0].cpu()).reshape(-1), want[1:7].astype(np.float64), sh.group)
    assert np.abs(f64(a.cpu()) - ref).max() < TOL_SCORE


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("fp32", 128)])
def test_the_other_storage_and_head_size_pairs(dtype, d):
    """bf16 with 64 channels per head and fp32 with 128 (the benchmarked pairs are bf16 / 128 and
    fp32 / 64): a prefill, and a decode step through the separate and the fused calls."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    w = synth.Workload(f"{dtype}_{d}", sh, 2048 + 33, 256, 4, True, 900 + d, n_planted=3,
                       outlier_kind="boost" if dtype == "fp32" else "student_t")
    run_prefill_case(w, attend=[2, w.n_windows - 1])
    n = 1500
    q, k, v = synth.gen_layer(w, "cpu", 0, 0, n_ctx=2048)
    rep = synth.pick_rep_keys(k[:n - 1], 128, sh.n_rep)
    nb = 12
    kc = H.blocked_k(k[:n - 1].to(DEV), sh, nb).unsqueeze(0).contiguous()
    vc = H.blocked_vt(v[:n - 1].to(DEV), sh, nb).unsqueeze(0).contiguous()
    repd = torch.zeros(1, nb, sh.n_rep, 2, d, dtype=sh.torch_dtype, device=DEV)
    repd[0, : rep.shape[0]] = rep.to(DEV)
    qd = q[n - 1][None, None].contiguous().to(DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    runner = H.LayerRunner(sh, 1, 1, nb, w.k_cap, DEV)
    out = torch.zeros_like(qd)
    nb_end_h = H.eligible_range(sh, n - 1)[1]
    runner.decode_step(qd, kc, vc, repd, torch.tensor([n], **i32), torch.tensor([nb_end_h], **i32), nb_end_h, out,
                       None, None, k[n - 1][None, None].contiguous().to(DEV), v[n - 1][None, None].contiguous().to(DEV),
                       torch.tensor([n - 1], **i32))
    torch.cuda.synchronize()
    res = orc.decode_step(f64(q[n - 1]), f64(k[:n]), f64(v[:n]), f64(rep), n, sh.n_init, sh.n_local, 128, w.k_cap, None)
    gi, gn = runner.idx[0].cpu().tolist(), int(runner.n_sel[0])
    assert check_selection(gi, gn, res, w.k_cap)
    assert out_error(out[0, 0], res["out"]) < TOL_OUT[dtype]


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 64)])
def test_prefill_of_three_sequences_in_one_batch(dtype, d):
    """Three independent sequences (own statistics, caches, representative keys, budgets) window by
    window in one batch; the third is 5 windows ahead of the others, so every per-sequence
    length (n_ctx, nb_end) differs within a call.  Every window of every sequence against the oracle."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    m, k_cap, n_win, lead = 256, 4, 6, [0, 0, 5]
    bt = 3
    n_tok = (n_win + max(lead)) * m
    nb = n_tok // 128
    seqs = []
    for s_ in range(bt):
        w = synth.Workload(f"batch_seq_{s_}", sh, n_tok, m, k_cap, True, 3100 + 17 * s_, n_planted=3,
                           outlier_kind="boost" if dtype == "fp32" else "student_t")
        q, k, v = synth.gen_layer(w, "cpu", 0, s_)
        seqs.append((w, q, k, v, synth.pick_rep_keys(k, 128, sh.n_rep)))
    kc = torch.stack([H.blocked_k(x[2].to(DEV), sh, nb) for x in seqs])
    vc = torch.stack([H.blocked_vt(x[3].to(DEV), sh, nb) for x in seqs])
    repd = torch.stack([x[4].to(DEV) for x in seqs])
    runner = H.LayerRunner(sh, bt, m, nb, k_cap, DEV)
    cut = [[synth.cutoff_state(x[0], max(H.eligible_range(sh, t * m)[1] - 1, 0), t, 0) for t in range(n_win + max(lead))]
           for x in seqs]
    want = [oracle_windows(x[1], x[2], x[3], x[4], sh, m, k_cap, cut[s_], attend=range(n_win + lead[s_]))
            for s_, x in enumerate(seqs)]
    i32 = dict(dtype=torch.int32, device=DEV)
    # the third sequence runs its first `lead` windows alone (a batch of one on the same record)
    solo = H.LayerRunner(sh, 1, m, nb, k_cap, DEV)
    for t in range(lead[2]):
        o = torch.zeros(m, 8, d, dtype=sh.torch_dtype, device=DEV)
        bud = torch.tensor([cut[2][t][0]], dtype=torch.float32, device=DEV)
        rest = torch.tensor([cut[2][t][1]], dtype=torch.float32, device=DEV)
        solo.step(seqs[2][1][t * m:(t + 1) * m].to(DEV), kc[2], vc[2], repd[2], torch.tensor([(t + 1) * m], **i32),
                  torch.tensor([H.eligible_range(sh, t * m)[1]], **i32), nb, o, bud, rest, True, m)
    runner.stats[2].copy_(solo.stats[0])
    for t in range(n_win):
        ts = [t + lead[s_] for s_ in range(bt)]
        qw = torch.stack([seqs[s_][1][ts[s_] * m:(ts[s_] + 1) * m] for s_ in range(bt)]).to(DEV)
        out = torch.zeros_like(qw)
        bud = torch.tensor([cut[s_][ts[s_]][0] for s_ in range(bt)], dtype=torch.float32, device=DEV)
        rest = torch.tensor([cut[s_][ts[s_]][1] for s_ in range(bt)], dtype=torch.float32, device=DEV)
        ends = [H.eligible_range(sh, ts[s_] * m)[1] for s_ in range(bt)]
        runner.step(qw, kc, vc, repd, torch.tensor([(x + 1) * m for x in ts], **i32), torch.tensor(ends, **i32),
                    max(ends), out, bud, rest, True, m)
        torch.cuda.synchronize()
        for s_ in range(bt):
            res = want[s_][ts[s_]]
            assert rel_to_max(runner.probe[s_], res["probe"]) < TOL_PROBE, f"probe, sequence {s_} window {ts[s_]}"
            gi, gn = runner.idx[s_].cpu().tolist(), int(runner.n_sel[s_])
            ref = res["out"]
            if not check_selection(gi, gn, res, k_cap):
                ref = orc.retrieval_attention_window(f64(seqs[s_][1][res["w0"]:res["w0"] + m]), f64(seqs[s_][2]),
                                                     f64(seqs[s_][3]), res["w0"], gi[:gn], sh.n_init, sh.n_local,
                                                     128, sh.group)
            assert out_error(out[s_], ref) < TOL_OUT[dtype], f"output, sequence {s_} window {ts[s_]}"


@pytest.mark.parametrize("n_init,n_local", [(0, 0), (0, 256), (384, 0), (512, 1024)])
def test_geometry_variants_on_the_matrix_core_kernels(n_init, n_local):
    """No initial tokens, no local span, neither, or more of both than the benchmarks use: a bf16
    prefill (matrix-core attention) and a decode step in two launches."""
    sh = LayerShape(8, 2, 128, 128, 4, n_init, n_local, "bf16")
    w = synth.Workload(f"geom_bf16_{n_init}_{n_local}", sh, 3072 + 50, 256, 4, True, 5150 + n_init + n_local,
                       n_planted=3)
    run_prefill_case(w, attend=[0, 5, w.n_windows - 1])
    n = 2900
    q, k, v = synth.gen_layer(w, "cpu", 0, 1, n_ctx=3072)
    rep = synth.pick_rep_keys(k[:n], 128, sh.n_rep)
    nb = 24
    kc = H.blocked_k(k[:n].to(DEV), sh, nb).unsqueeze(0).contiguous()
    vc = H.blocked_vt(v[:n].to(DEV), sh, nb).unsqueeze(0).contiguous()
    repd = torch.zeros(1, nb, sh.n_rep, 2, 128, dtype=torch.bfloat16, device=DEV)
    repd[0, : rep.shape[0]] = rep.to(DEV)
    qd = q[n - 1][None, None].contiguous().to(DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    runner = H.LayerRunner(sh, 1, 1, nb, w.k_cap, DEV)
    out = torch.zeros_like(qd)
    runner.decode_step_two_launches(qd, kc, vc, repd, torch.tensor([n], **i32),
                                    torch.tensor([H.eligible_range(sh, n - 1)[1]], **i32), out)
    torch.cuda.synchronize()
    res = orc.decode_step(f64(q[n - 1]), f64(k[:n]), f64(v[:n]), f64(rep), n, n_init, n_local, 128, w.k_cap, None)
    gi, gn = runner.idx[0].cpu().tolist(), int(runner.n_sel[0])
    assert check_selection(gi, gn, res, w.k_cap)
    assert out_error(out[0, 0], res["out"]) < TOL_OUT["bf16"]


@pytest.mark.parametrize("dtype,d,m", [("bf16", 128, 256), ("fp32", 64, 128), ("bf16", 128, 1), ("fp32", 64, 1)])
def test_device_side_values_are_clamped(dtype, d, m):
    """Lengths and counts that live in device memory are clamped against the capacities the
    host passes (every kernel does so before it forms an address): a call with absurd values
    gives exactly what the call with the clamped values gives."""
    sh = LayerShape(8, 2, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    nb, k_cap, bt = 12, 4, 3
    big, neg = 2 ** 31 - 1, -(2 ** 31)
    g = torch.Generator().manual_seed(77 + m)
    q = torch.randn(bt, m, 8, d, generator=g).to(td).to(DEV)
    kc = torch.randn(bt, nb, 2, 128, d, generator=g).to(td).to(DEV)
    vc = torch.randn(bt, nb, 2, d, 128, generator=g).to(td).to(DEV)
    rep = torch.randn(bt, nb, 4, 2, d, generator=g).to(td).to(DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    runner = H.LayerRunner(sh, bt, m, nb, k_cap, DEV)

    def run(n_ctx, nb_end, n_sel_attn):
        r = {}
        B.build_probe(cs, bt, m, q, runner.stats.zero_(), True, runner.probe, runner.probe_kv, runner.probe_norm, None,
                      runner.workspace)
        scores = torch.zeros(bt, runner.score_stride, device=DEV)
        B.score_blocks(cs, bt, runner.probe_kv, runner.probe_norm, rep, rep.stride(0), nb, 1,
                       torch.tensor(nb_end, **i32), scores, runner.score_stride)
        idx = torch.zeros(bt, k_cap, **i32); n_sel = torch.zeros(bt, **i32)
        B.select(bt, scores, runner.score_stride, nb, 1, torch.tensor(nb_end, **i32), k_cap, None, None, idx, n_sel)
        out = torch.zeros_like(q)
        bad_idx = torch.tensor([[2, big, neg, 5]] * bt, **i32)
        B.retrieval_attention(cs, bt, m, q, kc, vc, kc.stride(0), nb, torch.tensor(n_ctx, **i32), bad_idx,
                              torch.tensor(n_sel_attn, **i32), k_cap, out, None, runner.workspace)
        torch.cuda.synchronize()
        return scores, idx, n_sel, out

    cap = nb * 128
    absurd = run([big, neg, cap + 1], [big, neg, nb + 5], [big, neg, 3])
    clamped = run([cap, max(m, 1), cap], [nb, 1, nb], [k_cap, 0, 3])
    for a, b in zip(absurd, clamped):
        assert torch.equal(a, b)
    assert bool(torch.isfinite(absurd[3].float()).all())
    # a position far behind the cache: nothing is written (the cache update and the decode scoring launch)
    kc2, vc2, rep2 = kc.clone(), vc.clone(), rep.clone()
    k_new = torch.randn(bt, m, 2, d, generator=g).to(td).to(DEV)
    far = torch.tensor([big, big - 5, cap], **i32)
    B.append_kv(cs, bt, m, k_new, k_new, far, kc2, vc2, kc2.stride(0), rep2, rep2.stride(0), nb)
    if m == 1:
        B.decode_retrieve(cs, bt, q, k_new, k_new, far, kc2, vc2, kc2.stride(0), rep2, rep2.stride(0), nb, 1,
                          torch.tensor([nb, nb, nb], **i32), None, None, None, torch.zeros_like(clamped[0]),
                          runner.score_stride, k_cap, None, None, clamped[1].clone(), clamped[2].clone(), None, None)
    torch.cuda.synchronize()
    assert torch.equal(kc2, kc) and torch.equal(vc2, vc) and torch.equal(rep2, rep)
    if m == 1 and dtype == "bf16":                          # the attention launch that selects for itself
        def fused(n_ctx, nb_end):
            idx = torch.zeros(bt, k_cap, **i32); n_sel = torch.zeros(bt, **i32)
            out = torch.zeros_like(q)
            B.decode_select_attention(cs, bt, q, kc, vc, kc.stride(0), nb, torch.tensor(n_ctx, **i32), clamped[0],
                                      runner.score_stride, 1, torch.tensor(nb_end, **i32), k_cap, None, None, None,
                                      idx, n_sel, None, None, out, None, runner.workspace)
            torch.cuda.synchronize()
            return idx, n_sel, out
        for a, b in zip(fused([big, neg, cap + 1], [big, neg, nb + 5]), fused([cap, 1, cap], [nb, 1, nb])):
            assert torch.equal(a, b)


def test_context_shorter_than_init():
    sh = LayerShape(4, 2, 64, 128, 2, 128, 128, "fp32")
    w = synth.Workload("tiny", sh, 100, 128, 4, False, 5, outlier_kind="boost", n_planted=0)
    run_prefill_case(w)


def test_copy_bytes():
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    B.copy_bytes(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


# ---------------------------------------------------------------- select alone: ties, cut-off, sizes
def _select_case(scores: np.ndarray, nb_begin: int, k_cap: int, cutoff, topk: bool = False):
    n = len(scores)
    sc = torch.zeros(1, n + nb_begin, dtype=torch.float32, device=DEV)
    sc[0, nb_begin:] = torch.from_numpy(scores.astype(np.float32)).to(DEV)
    nb_end = torch.tensor([n + nb_begin], dtype=torch.int32, device=DEV)
    idx = torch.zeros(1, k_cap, dtype=torch.int32, device=DEV)
    n_sel = torch.zeros(1, dtype=torch.int32, device=DEV)
    theta = torch.zeros(1, dtype=torch.float32, device=DEV)
    budget = torch.zeros(1, dtype=torch.float32, device=DEV)
    cut = None if cutoff is None else torch.tensor([list(cutoff)], dtype=torch.float32, device=DEV)
    bud = None if cut is None else cut[0, 0:1]
    rest = None if cut is None else cut[0, 1:2]
    B.select(1, sc, n + nb_begin, n + nb_begin, nb_begin, nb_end, k_cap, bud, rest, idx, n_sel, theta,
             budget, flags=B.SELECT_ENTROPY_TOPK if topk else 0)
    torch.cuda.synchronize()
    s32 = scores.astype(np.float32).astype(np.float64)
    ids = list(range(nb_begin, nb_begin + n))
    th = (orc.information_density_topk(s32, k_cap) if topk else orc.information_density(s32)) if n else 0.0
    if cutoff is None:
        count = min(k_cap, n)
    else:
        count = orc.cutoff_count(orc.layer_budget(th, cutoff[1], cutoff[0]), k_cap, n) if n else 0
    want = orc.select_blocks(s32, ids, count)
    return idx[0].cpu().tolist(), int(n_sel), float(theta), float(budget), want, th, cut


@pytest.mark.parametrize("n,k_cap", [(1, 4), (5, 8), (63, 8), (64, 64), (65, 32), (1000, 32),
                                     (1025, 16), (4097, 64), (8192, 32)])
def test_select_exact_with_ties(n, k_cap):
    rng = np.random.default_rng(n * 131 + k_cap)
    scores = rng.integers(-6, 7, size=n) / 8.0            # many exact ties, exactly representable
    scores[rng.integers(0, n)] = -0.0
    _say(f"[select] n={n} k_cap={k_cap}")
    got, n_sel, theta, budget, want, th, _ = _select_case(scores, 3, k_cap, None)
    assert n_sel == len(want) and got[:n_sel] == want and all(x == -1 for x in got[n_sel:])
    assert abs(theta - th) < TOL_THETA


def test_select_cutoff_bookkeeping_and_monotonicity():
    rng = np.random.default_rng(3)
    base = rng.normal(size=500) * 0.05
    counts = []
    for spread in (4.0, 2.0, 1.0, 0.5, 0.1):               # density rises as the spread shrinks
        scores = np.clip(base * spread, -1, 1)
        got, n_sel, theta, budget, want, th, cut = _select_case(scores, 1, 32, (200.0, 60.0))
        b = orc.layer_budget(th, 60.0, 200.0)
        assert abs(budget - b) < TOL_BUDGET * b and abs(float(cut[0, 0]) - (200.0 - b)) < 1e-2
        assert got[:n_sel] == want
        counts.append(n_sel)
    assert counts == sorted(counts)
    # nothing eligible: nothing selected, budget untouched
    got, n_sel, theta, budget, want, th, cut = _select_case(np.zeros(0), 2, 8, (50.0, 10.0))
    assert n_sel == 0 and got == [-1] * 8 and float(cut[0, 0]) == 50.0


@pytest.mark.parametrize("n,k_cap", [(1, 4), (5, 8), (64, 64), (65, 32), (1000, 32), (1025, 16), (5000, 64)])
def test_select_density_over_the_best_blocks(n, k_cap):
    """ACTQKV_SELECT_ENTROPY_TOPK: the density of Eq. (11) over the k_cap best blocks only, then
    the same budget, count and selection; without cut-off state the selection does not change."""
    rng = np.random.default_rng(n * 17 + k_cap)
    scores = np.clip(rng.normal(size=n) * 0.2, -1, 1)
    _say(f"[select, density over the best] n={n} k_cap={k_cap}")
    cut = (3.0 * k_cap, 2.5 * math.log(max(min(n, k_cap), 2)))
    got, n_sel, theta, budget, want, th, state = _select_case(scores, 2, k_cap, cut, topk=True)
    assert abs(theta - th) < TOL_THETA
    b = orc.layer_budget(th, cut[1], cut[0])
    assert abs(budget - b) <= TOL_BUDGET * max(1.0, b) and abs(float(state[0, 0]) - (cut[0] - b)) < 1e-2
    assert n_sel == len(want) and got[:n_sel] == want and all(x == -1 for x in got[n_sel:])
    plain = _select_case(scores, 2, k_cap, None)
    top = _select_case(scores, 2, k_cap, None, topk=True)
    assert plain[0] == top[0] and plain[1] == top[1]
    if n > k_cap:
        assert top[2] < plain[2]            # fewer terms, lower entropy


def test_scores_zero_norms_and_determinism():
    sh = LayerShape(8, 2, 64, 128, 4, 128, 128, "bf16")
    cs = B.c_shape(sh)
    g = torch.Generator().manual_seed(11)
    nb = 37
    rep = torch.randn(nb, 4, 2, 64, generator=g).to(torch.bfloat16)
    rep[5] = 0                                               # a block of zero keys scores 0
    probe = torch.randn(8, 64, generator=g)
    pk = probe.reshape(2, 4, 64).sum(1).reshape(1, -1).contiguous().to(DEV)
    pn = probe.norm().reshape(1).to(DEV)
    nb_end = torch.tensor([nb], dtype=torch.int32, device=DEV)
    outs = []
    for _ in range(2):
        sc = torch.full((1, 40), 7.0, dtype=torch.float32, device=DEV)
        B.score_blocks(cs, 1, pk, pn, rep.to(DEV), 0, nb, 1, nb_end, sc, 40)
        torch.cuda.synchronize()
        outs.append(sc.cpu())
    assert torch.equal(outs[0], outs[1])
    want = orc.block_scores(f64(probe).reshape(-1), f64(rep), 4)
    got = f64(outs[0][0])
    assert got[0] == 7.0 and (got[nb:] == 7.0).all()         # outside the range: untouched
    assert np.abs(got[1:nb] - want[1:]).max() < TOL_SCORE and got[5] == 0.0
    # zero probe: all scores 0
    sc = torch.full((1, 40), 7.0, dtype=torch.float32, device=DEV)
    B.score_blocks(cs, 1, torch.zeros_like(pk), torch.zeros_like(pn), rep.to(DEV), 0, nb, 1, nb_end, sc, 40)
    assert float(sc[0, 1:nb].abs().max()) == 0.0


# ---------------------------------------------------------------- decode
@pytest.mark.parametrize("dtype,hq,hkv,n_ctxs", [
    ("fp32", 8, 2, [3000, 2817, 1100]),                       # ragged, one just past a block boundary
    ("bf16", 8, 2, [3000, 2817, 1100]),                       # few (sequence, head) pairs: several workgroups per pair, merged by the last one
    ("bf16", 32, 8, [2900, 2817, 1100, 700, 3000, 129, 2048, 1]),  # 64 pairs: one workgroup per pair
    ("bf16", 28, 4, [2900, 1100, 129]),                       # 7 query heads per KV head
])
@pytest.mark.parametrize("launches", [4, 3, 2, 1, 0])
def test_decode_step_batch(dtype, hq, hkv, n_ctxs, launches):
    """launches 4: probe, scores, selection, attention; 3: probe and scores in one launch
    (actqkv_decode_retrieve); 2: the selection inside the attention launch as well
    (actqkv_decode_select_attention; bf16 only); 1: the whole layer in one launch
    (actqkv_decode_layer); 0: the same with ACTQKV_DECODE_NO_WAIT, i.e. every workgroup takes
    the path of a wait that ran out and scores its whole sequence itself."""
    if launches <= 2 and dtype != "bf16":
        pytest.skip("the attention that selects for itself is a bf16 kernel")
    sh = LayerShape(hq, hkv, 128 if dtype == "bf16" else 64, 128, 4, 128, 256, dtype)
    w = synth.Workload("decode_small", sh, 3000, 1, 6, True, 2024, n_planted=4, batch=len(n_ctxs))
    nb_cap = 24
    bt = len(n_ctxs)
    ks, vs, reps, qs = [], [], [], []
    for s, n in enumerate(n_ctxs):
        q, k, v = synth.gen_layer(w, "cpu", 0, s, n_ctx=4096)
        ks.append(k[:n]); vs.append(v[:n]); qs.append(q[n - 1])
        reps.append(synth.pick_rep_keys(k[:n], 128, sh.n_rep))
    kc = torch.stack([H.blocked_k(k.to(DEV), sh, nb_cap) for k in ks])
    vc = torch.stack([H.blocked_vt(v.to(DEV), sh, nb_cap) for v in vs])
    repd = torch.zeros(bt, nb_cap, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=sh.torch_dtype, device=DEV)
    for s, r in enumerate(reps):
        repd[s, : r.shape[0]] = r.to(DEV)
    qd = torch.stack(qs).unsqueeze(1).contiguous().to(DEV)    # [B][1][H][D]
    runner = H.LayerRunner(sh, bt, 1, nb_cap, w.k_cap, DEV)
    nb_ends = [H.eligible_range(sh, n - 1)[1] for n in n_ctxs]
    cuts = [synth.cutoff_state(w, e - 1, 0, 3, s) for s, e in enumerate(nb_ends)]
    bud = torch.tensor([c[0] for c in cuts], dtype=torch.float32, device=DEV)
    rest = torch.tensor([c[1] for c in cuts], dtype=torch.float32, device=DEV)
    out = torch.zeros_like(qd)
    if launches == 3:
        runner.decode_step(qd, kc, vc, repd, torch.tensor(n_ctxs, dtype=torch.int32, device=DEV),
                           torch.tensor(nb_ends, dtype=torch.int32, device=DEV), max(nb_ends), out, bud, rest)
    elif launches == 2:
        after = torch.zeros_like(bud)
        runner.decode_step_two_launches(qd, kc, vc, repd, torch.tensor(n_ctxs, dtype=torch.int32, device=DEV),
                                        torch.tensor(nb_ends, dtype=torch.int32, device=DEV), out, bud, rest, after)
        torch.cuda.synchronize()
        want_after = bud - runner.budget
        want_after[runner.n_sel == 0] = bud[runner.n_sel == 0]
        assert torch.allclose(after, want_after, rtol=1e-6, atol=1e-6)
    elif launches <= 1:
        after = torch.zeros_like(bud)
        nb_end_d = torch.tensor(nb_ends, dtype=torch.int32, device=DEV)
        for run in range(2):               # twice: the sequence counters must be back at zero
            runner.decode_step_one_launch(qd, kc, vc, repd, torch.tensor(n_ctxs, dtype=torch.int32, device=DEV),
                                          nb_end_d, out, bud, rest, after,
                                          flags=0 if launches == 1 else B.DECODE_NO_WAIT)
            torch.cuda.synchronize()
            assert not runner.workspace[:8192].any(), "counters left dirty"
        want_after = bud - runner.budget
        want_after[runner.n_sel == 0] = bud[runner.n_sel == 0]
        assert torch.allclose(after, want_after, rtol=1e-6, atol=1e-6)
        # the scores are those of the scoring call
        pkv = qd.float().reshape(bt, hkv, hq // hkv, -1).sum(dim=2).reshape(bt, -1).contiguous()
        pn = qd.float().reshape(bt, -1).norm(dim=1).contiguous()
        sc_ref = torch.zeros_like(runner.scores)
        B.score_blocks(runner.cs, bt, pkv, pn, repd, repd.stride(0), nb_cap, 1, nb_end_d, sc_ref, runner.score_stride)
        torch.cuda.synchronize()
        for s_, e in enumerate(nb_ends):
            assert torch.allclose(runner.scores[s_, 1:e], sc_ref[s_, 1:e], rtol=1e-5, atol=1e-6)
    else:
        runner.step(qd, kc, vc, repd, torch.tensor(n_ctxs, dtype=torch.int32, device=DEV),
                    torch.tensor(nb_ends, dtype=torch.int32, device=DEV), max(nb_ends), out, bud, rest,
                    update_stats=False, m=1)
    torch.cuda.synchronize()
    for s, n in enumerate(n_ctxs):
        res = orc.decode_step(f64(qs[s]), f64(ks[s]), f64(vs[s]), f64(reps[s]), n, sh.n_init, sh.n_local,
                              128, w.k_cap, cuts[s])
        gi, gn = runner.idx[s].cpu().tolist(), int(runner.n_sel[s])
        same = check_selection(gi, gn, res, w.k_cap)
        ref = res["out"]
        if not same:
            ref = orc.retrieval_attention(f64(qs[s])[None], f64(ks[s]), f64(vs[s]), n - 1, gi[:gn],
                                          sh.n_init, sh.n_local, 128, sh.group)[0]
        assert out_error(out[s, 0], ref) < TOL_OUT[dtype], f"decode output, sequence {s}"
        if launches >= 2:      # (the one-launch layer keeps the probe to itself)
            assert rel_to_max(runner.probe[s], f64(qs[s]).reshape(-1)) == 0.0   # probe is the query itself


def test_decode_full_size_layer_as_benchmarked():
    """One layer of configs[3] at full size in the launch configuration bench.py times: 16
    sequences with 65536 cached tokens each (4.3 GB of keys and values), a new token appended,
    k_cap 32 with the cut-off; the selection and the output of sampled sequences against the
    oracle, the whole batch for finiteness and for equality between two runs."""
    w = synth.WORKLOADS["c4_decode"]
    sh, bt = w.shape, w.batch
    n0 = w.n_ctx
    nb_cap = (n0 + 256 + 127) // 128
    hk, D = sh.n_kv_heads, sh.head_dim
    _say(f"[case] {w.name} one layer, batch {bt}, {n0} cached tokens")
    gen = torch.Generator(device=DEV); gen.manual_seed(w.seed)
    kc = torch.empty(bt, nb_cap, hk, 128, D, dtype=torch.bfloat16, device=DEV).normal_(generator=gen)
    vc = torch.empty(bt, nb_cap, hk, D, 128, dtype=torch.bfloat16, device=DEV).normal_(generator=gen)
    u = synth.direction(w, 0, 0, DEV)
    planted = torch.stack([torch.tensor(synth.planted_blocks(w, 0, s)) for s in range(bt)]).to(DEV)
    sidx = torch.arange(bt, device=DEV)[:, None].expand_as(planted)
    kc[sidx, planted] += (w.shift * u)[None, None, :, None, :].to(torch.bfloat16)
    cs = B.c_shape(sh)
    rep = synth.pick_rep_keys_blocked(kc, sh.n_rep).contiguous()      # the harness rule for synthetic caches
    q = (torch.randn(bt, 1, sh.n_q_heads, D, generator=gen, device=DEV) +
         w.alpha * u.repeat_interleave(sh.group, dim=0)).to(torch.bfloat16)
    k_new = torch.randn(bt, 1, hk, D, generator=gen, device=DEV).to(torch.bfloat16)
    v_new = torch.randn(bt, 1, hk, D, generator=gen, device=DEV).to(torch.bfloat16)
    pos0 = torch.full((bt,), n0, dtype=torch.int32, device=DEV)
    n_ctx = torch.full((bt,), n0 + 1, dtype=torch.int32, device=DEV)
    nb_begin, nb_end_h = H.eligible_range(sh, n0)
    nb_end = torch.full((bt,), nb_end_h, dtype=torch.int32, device=DEV)
    cut = synth.cutoff_state(w, nb_end_h - nb_begin, 0, 5, 0)
    runner = H.LayerRunner(sh, bt, 1, nb_cap, w.k_cap, DEV)
    outs = []
    for rep_run in range(4):
        bud = torch.full((bt,), cut[0], dtype=torch.float32, device=DEV)
        rest = torch.full((bt,), cut[1], dtype=torch.float32, device=DEV)
        out = torch.zeros_like(q)
        if rep_run == 0:      # five launches: update, probe, scores, selection, attention
            B.append_kv(cs, bt, 1, k_new, v_new, pos0, kc, vc, kc.stride(0), rep, rep.stride(0), nb_cap)
            runner.step(q, kc, vc, rep, n_ctx, nb_end, nb_end_h, out, bud, rest, update_stats=False, m=1)
        elif rep_run == 1:    # three launches
            runner.decode_step(q, kc, vc, rep, n_ctx, nb_end, nb_end_h, out, bud, rest, k_new, v_new, pos0)
        elif rep_run == 2:    # two launches
            after = torch.zeros_like(bud)
            runner.decode_step_two_launches(q, kc, vc, rep, n_ctx, nb_end, out, bud, rest, after, k_new, v_new, pos0)
            bud = after
        else:                 # one launch, as benchmarked
            after = torch.zeros_like(bud)
            runner.decode_step_one_launch(q, kc, vc, rep, n_ctx, nb_end, out, bud, rest, after,
                                          k_new.squeeze(1).contiguous(), v_new.squeeze(1).contiguous())
            bud = after
        torch.cuda.synchronize()
        outs.append((runner.idx.clone(), runner.n_sel.clone(), out, runner.theta.clone(), bud))
    for other in outs[1:]:      # selections bit for bit; outputs, density and budget to rounding
        for i, (a, b) in enumerate(zip(outs[0], other)):
            if i < 2:
                assert torch.equal(a, b)
            elif i == 2:
                assert float((a.float() - b.float()).abs().max()) <= 2e-2 * float(a.float().abs().max())
            else:
                assert torch.allclose(a, b, rtol=1e-5)
    assert torch.equal(outs[0][2], outs[1][2])        # the same attention kernel on the same selection
    outs = [o[2] for o in outs]
    assert bool(torch.isfinite(outs[0].float()).all())
    for s in (0, 7, 15):
        k_log, v_log = _logical_from_blocked(kc[s].cpu(), vc[s].cpu(), n0 + 1)
        assert torch.equal(k_log[n0], k_new[s, 0].cpu()) and torch.equal(v_log[n0], v_new[s, 0].cpu())
        rep_s = rep[s, : (n0 + 1) // 128].cpu()
        res = orc.decode_step(f64(q[s, 0]), k_log.float().numpy(), v_log.float().numpy(), f64(rep_s), n0 + 1,
                              sh.n_init, sh.n_local, 128, w.k_cap, cut)
        gi, gn = runner.idx[s].cpu().tolist(), int(runner.n_sel[s])
        ref = res["out"]
        if not check_selection(gi, gn, res, w.k_cap):
            ref = orc.retrieval_attention(f64(q[s, 0])[None], k_log.float().numpy(), v_log.float().numpy(), n0,
                                          gi[:gn], sh.n_init, sh.n_local, 128, sh.group)[0]
        errs = [out_error(o[s, 0], ref) for o in outs]
        err = max(errs)
        _say(f"[case] {w.name} sequence {s}: E = {gn}, output error {errs[0]:.3e} / {errs[1]:.3e} / {errs[2]:.3e} / "
             f"{errs[3]:.3e} (five, three, two launches, one launch)")
        assert err < TOL_OUT["bf16"], f"decode output, sequence {s}"


@pytest.mark.parametrize("n,k_cap,mode", [(5, 8, "cutoff"), (511, 32, "cutoff"), (513, 32, "cutoff"), (1500, 64, "topk"),
                                          (4000, 16, "plain"), (0, 8, "cutoff")])
def test_decode_attention_that_selects_for_itself(n, k_cap, mode):
    """actqkv_decode_select_attention against the oracle's selection (ties by block index,
    density, budget, count) for more eligible blocks than the 512 threads of a workgroup, and
    against actqkv_select + actqkv_retrieval_attention on the same inputs.  mode: cut-off on /
    density over the best blocks (the other reading of Eq. (11)) / no cut-off."""
    sh = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    bt, nb_begin = 2, 1
    nb = nb_begin + n + 4                                   # the local span and the new token's block behind the eligible ones
    n_ctx = (nb - 1) * 128 + 1
    rng = np.random.default_rng(7 * n + k_cap)
    g = torch.Generator().manual_seed(n + 1)
    kc = torch.randn(bt, nb, 2, 128, 128, generator=g).to(torch.bfloat16).to(DEV)
    vc = torch.randn(bt, nb, 2, 128, 128, generator=g).to(torch.bfloat16).to(DEV)
    q = torch.randn(bt, 1, 8, 128, generator=g).to(torch.bfloat16).to(DEV)
    stride = nb
    scores = np.zeros((bt, stride), dtype=np.float32)
    scores[0, nb_begin:nb_begin + n] = rng.integers(-6, 7, size=n) / 8.0      # many exact ties
    scores[1, nb_begin:nb_begin + n] = rng.normal(size=n).astype(np.float32) * 0.3
    sd = torch.from_numpy(scores).to(DEV)
    nb_end = torch.full((bt,), nb_begin + n, dtype=torch.int32, device=DEV)
    nctx = torch.full((bt,), n_ctx, dtype=torch.int32, device=DEV)
    cut = (37.0, 11.0) if mode != "plain" else None
    flags = B.SELECT_ENTROPY_TOPK if mode == "topk" else 0
    ws = torch.zeros(B.workspace_bytes(cs, bt, 1, nb, k_cap), dtype=torch.uint8, device=DEV)
    res = []
    for fused in (False, True):
        bud = torch.full((bt,), cut[0], device=DEV) if cut else None
        rest = torch.full((bt,), cut[1], device=DEV) if cut else None
        after = torch.full((bt,), -1.0, device=DEV)
        idx = torch.zeros(bt, k_cap, dtype=torch.int32, device=DEV)
        n_sel = torch.zeros(bt, dtype=torch.int32, device=DEV)
        theta = torch.zeros(bt, device=DEV); b_l = torch.zeros(bt, device=DEV)
        out = torch.zeros_like(q)
        if fused:
            B.decode_select_attention(cs, bt, q, kc, vc, kc.stride(0), nb, nctx, sd, stride, nb_begin, nb_end, k_cap,
                                      bud, rest, after if cut else None, idx, n_sel, theta, b_l, out, None, ws,
                                      flags=flags)
        else:
            B.select(bt, sd, stride, nb, nb_begin, nb_end, k_cap, bud, rest, idx, n_sel, theta, b_l, flags=flags)
            B.retrieval_attention(cs, bt, 1, q, kc, vc, kc.stride(0), nb, nctx, idx, n_sel, k_cap, out, None, ws)
            after = bud
        torch.cuda.synchronize()
        res.append((idx.cpu(), n_sel.cpu(), theta.cpu(), b_l.cpu(), after.cpu() if cut else None, out.float().cpu()))
    a, b = res
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert torch.allclose(a[2], b[2], rtol=1e-5, atol=1e-6) and torch.allclose(a[3], b[3], rtol=1e-5, atol=1e-6)
    if cut:
        assert torch.allclose(a[4], b[4], rtol=1e-5, atol=1e-5)
    assert float((a[5] - b[5]).abs().max()) <= 1e-2 * float(a[5].abs().max())
    for s_ in range(bt):                                    # and the oracle
        sc = scores[s_, nb_begin:nb_begin + n].astype(np.float64)
        ids = list(range(nb_begin, nb_begin + n))
        if n == 0:
            assert int(b[1][s_]) == 0 and all(int(x) == -1 for x in b[0][s_])
            continue
        th = orc.information_density_topk(sc, k_cap) if mode == "topk" else orc.information_density(sc)
        if cut:
            bl = orc.layer_budget(th, cut[1], cut[0])
            count = orc.cutoff_count(bl, k_cap, n)
            assert abs(float(b[3][s_]) - bl) < TOL_BUDGET * max(bl, 1.0)
        else:
            count = min(k_cap, n)
        assert abs(float(b[2][s_]) - th) < TOL_THETA
        want = orc.select_blocks(scores[s_, nb_begin:nb_begin + n], ids, count)
        assert int(b[1][s_]) == count and b[0][s_].tolist()[:count] == want


def test_largest_batch_of_a_decode_step():
    """1024 sequences (the largest batch the library takes) through the decode step in two
    launches: short ragged contexts, selections against the oracle's rule on the GPU's scores,
    outputs against a plain softmax attention over the keys each sequence sees."""
    sh = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    bt, nb, k_cap = 1024, 8, 3
    g = torch.Generator(device=DEV).manual_seed(1024)
    kc = torch.randn(bt, nb, 2, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
    vc = torch.randn(bt, nb, 2, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
    rep = torch.randn(bt, nb, 4, 2, 128, generator=g, device=DEV).to(torch.bfloat16)
    q = torch.randn(bt, 1, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
    n_ctx_h = [1 + (37 * s) % (nb * 128 - 1) for s in range(bt)]
    n_ctx = torch.tensor(n_ctx_h, dtype=torch.int32, device=DEV)
    nb_end_h = [H.eligible_range(sh, n - 1)[1] for n in n_ctx_h]
    nb_end = torch.tensor(nb_end_h, dtype=torch.int32, device=DEV)
    runner = H.LayerRunner(sh, bt, 1, nb, k_cap, DEV)
    out = torch.zeros_like(q)
    runner.decode_step_two_launches(q, kc, vc, rep, n_ctx, nb_end, out)
    torch.cuda.synchronize()
    scores, idx, n_sel = runner.scores.cpu().numpy(), runner.idx.cpu().tolist(), runner.n_sel.cpu().tolist()
    assert bool(torch.isfinite(out.float()).all())
    for s in range(0, bt, 41):
        n, e = n_ctx_h[s], nb_end_h[s]
        elig = list(range(1, e))
        want = orc.select_blocks(scores[s, 1:e], elig, min(k_cap, len(elig))) if elig else []
        assert n_sel[s] == len(want) and idx[s][:n_sel[s]] == want, f"sequence {s}"
        l0 = H.local_start(sh, n - 1)
        pos = list(range(0, min(sh.n_init, n - 1)))
        for b in want:
            pos += list(range(b * 128, b * 128 + 128))
        pos += list(range(l0, n))
        pos = torch.tensor(sorted(set(pos)), device=DEV)
        K = kc[s][pos // 128, :, pos % 128, :].float()
        V = vc[s][pos // 128, :, :, pos % 128].float()
        qq = q[s, 0].float().reshape(2, 4, 128)
        p = torch.softmax(torch.einsum("hgd,nhd->hgn", qq, K) / 128 ** 0.5, dim=-1)
        ref = torch.einsum("hgn,nhd->hgd", p, V).reshape(8, 128)
        err = ((out[s, 0].float() - ref).abs().amax(dim=-1) / ref.abs().amax(dim=-1)).max().item()
        assert err < TOL_OUT["bf16"], f"sequence {s}: {err}"


# ---------------------------------------------------------------- cache update and representatives
def _logical_from_blocked(kc, vc, n):
    """[nb][Hk][Bs][D], [nb][Hk][D][Bs] -> K, V [n][Hk][D]."""
    nb, hk, bs, d = kc.shape
    k = kc.permute(0, 2, 1, 3).reshape(nb * bs, hk, d)[:n]
    v = vc.permute(0, 3, 1, 2).reshape(nb * bs, hk, d)[:n]
    return k, v


def _check_reps(rep_gpu, k_all_cpu, sh, n_tokens):
    """Representative keys of all complete blocks against the oracle: bit-equal, unless the
    fp32 norms that decide on the GPU tie within rounding with the fp64 ones of the oracle."""
    want = orc.representative_keys(k_all_cpu.float().numpy(), sh.block_size, sh.n_rep)
    got = rep_gpu[: want.shape[0]].float().cpu().numpy()
    for b in range(want.shape[0]):
        if np.array_equal(got[b], want[b]):
            continue
        kb = f64(k_all_cpu[b * sh.block_size:(b + 1) * sh.block_size])
        norms = np.sqrt((kb ** 2).sum(axis=(1, 2)))
        order = np.sort(norms)[::-1]
        gap = order[sh.n_rep - 1] - order[sh.n_rep]
        assert gap < 1e-5 * order[0], f"block {b}: representatives differ with a norm gap of {gap}"
        rows = {tuple(r.reshape(-1)) for r in kb.astype(np.float32)}
        assert all(tuple(r.reshape(-1)) in rows for r in got[b]), f"block {b}: not keys of the block"


@pytest.mark.parametrize("dtype,hq,hkv,d,chunks", [
    ("bf16", 32, 8, 128, [512, 512, 512, 77]),          # aligned windows and a ragged tail
    ("bf16", 32, 8, 128, [100, 1, 1, 300, 27, 1]),      # unaligned pieces, single tokens
    ("fp32", 8, 2, 64, [256, 256, 130]),
    ("bf16", 8, 2, 128, [77, 8192, 3000]),              # the largest window, starting inside a block
    ("fp32", 4, 2, 64, [5000, 1]),
])
def test_append_kv_builds_the_cache_and_the_representatives(dtype, hq, hkv, d, chunks):
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    n = sum(chunks)
    nb_cap = (n + 127) // 128 + 1
    g = torch.Generator().manual_seed(1234 + n)
    k = torch.randn(n, hkv, d, generator=g).to(tdt)
    v = torch.randn(n, hkv, d, generator=g).to(tdt)
    _say(f"[append] {dtype} H{hq}/Hk{hkv}/D{d} chunks={chunks}")
    kc = torch.zeros(nb_cap, hkv, 128, d, dtype=tdt, device=DEV)
    vc = torch.zeros(nb_cap, hkv, d, 128, dtype=tdt, device=DEV)
    rep = torch.zeros(nb_cap, sh.n_rep, hkv, d, dtype=tdt, device=DEV)
    pos = 0
    for m in chunks:
        pos0 = torch.tensor([pos], dtype=torch.int32, device=DEV)
        B.append_kv(cs, 1, m, k[pos:pos + m].to(DEV), v[pos:pos + m].to(DEV), pos0, kc, vc, 0, rep, 0, nb_cap)
        pos += m
    torch.cuda.synchronize()
    # byte moves: bit-exact, and nothing written behind the last token
    assert torch.equal(kc.cpu(), H.blocked_k(k, sh, nb_cap)) and torch.equal(vc.cpu(), H.blocked_vt(v, sh, nb_cap))
    kl, vl = _logical_from_blocked(kc.cpu(), vc.cpu(), n)
    k_or, v_or = orc.append_cache(k[:0].float().numpy(), v[:0].float().numpy(), k.float().numpy(), v.float().numpy())
    assert np.array_equal(kl.float().numpy(), k_or) and np.array_equal(vl.float().numpy(), v_or)
    _check_reps(rep, k, sh, n)
    assert not rep[n // 128:].any(), "representatives of an incomplete block were written"


def test_append_kv_on_random_chunk_sequences():
    """20 random shapes and sequences of chunk lengths (single tokens, pieces that end on, just
    before and just behind block boundaries, long windows); half of the single tokens go through
    the decode scoring launch, which also updates the cache."""
    rng = np.random.default_rng(555)
    for trial in range(20):
        hkv = int(rng.choice([1, 2, 4, 8])); d = int(rng.choice([64, 128])); n_rep = int(rng.integers(1, 9))
        dtype = "bf16" if trial % 2 else "fp32"
        tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
        sh = LayerShape(hkv * 2, hkv, d, 128, n_rep, 128, 256, dtype)
        cs = B.c_shape(sh)
        chunks, total = [], 0
        while total < 900:
            c = int(rng.choice([1, 1, 1, 2, 127, 128, 129, 300, (128 - total % 128) or 1, int(rng.integers(1, 400))]))
            chunks.append(c); total += c
        n = total
        nb_cap = (n + 127) // 128 + 1
        g = torch.Generator().manual_seed(9000 + trial)
        k = torch.randn(n, hkv, d, generator=g).to(tdt)
        v = torch.randn(n, hkv, d, generator=g).to(tdt)
        kc = torch.zeros(1, nb_cap, hkv, 128, d, dtype=tdt, device=DEV)
        vc = torch.zeros(1, nb_cap, hkv, d, 128, dtype=tdt, device=DEV)
        rep = torch.zeros(1, nb_cap, n_rep, hkv, d, dtype=tdt, device=DEV)
        q = torch.zeros(1, 1, hkv * 2, d, dtype=tdt, device=DEV)
        scores = torch.zeros(1, nb_cap + 3, device=DEV)
        nb_end = torch.zeros(1, dtype=torch.int32, device=DEV)
        pos = 0
        for i, m in enumerate(chunks):
            pos0 = torch.tensor([pos], dtype=torch.int32, device=DEV)
            kn, vn = k[pos:pos + m][None].contiguous().to(DEV), v[pos:pos + m][None].contiguous().to(DEV)
            if m == 1 and i % 2:
                B.decode_retrieve(cs, 1, q, kn, vn, pos0, kc, vc, 0, rep, 0, nb_cap, 1, nb_end, None, None, None, scores,
                                  nb_cap + 3, 4, None, None, None, None, None, None, flags=B.DECODE_SCORES_ONLY)
            else:
                B.append_kv(cs, 1, m, kn, vn, pos0, kc, vc, 0, rep, 0, nb_cap)
            pos += m
        torch.cuda.synchronize()
        assert torch.equal(kc[0].cpu(), H.blocked_k(k, sh, nb_cap)), (trial, chunks)
        assert torch.equal(vc[0].cpu(), H.blocked_vt(v, sh, nb_cap)), (trial, chunks)
        want = orc.representative_keys(k.float().numpy(), 128, n_rep)
        assert np.array_equal(rep[0, : want.shape[0]].float().cpu().numpy(), want), (trial, chunks)
        assert not rep[0, n // 128:].any(), (trial, chunks)


def test_append_kv_batch_of_decode_steps():
    """Three sequences at different lengths take single tokens; two of them finish a block."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    lens = [126, 255, 300]
    steps, nb_cap = 3, 4
    g = torch.Generator().manual_seed(99)
    ks = [torch.randn(l + steps, 8, 128, generator=g).to(torch.bfloat16) for l in lens]
    vs = [torch.randn(l + steps, 8, 128, generator=g).to(torch.bfloat16) for l in lens]
    kc = torch.stack([H.blocked_k(k[:l], sh, nb_cap) for k, l in zip(ks, lens)]).to(DEV)
    vc = torch.stack([H.blocked_vt(v[:l], sh, nb_cap) for v, l in zip(vs, lens)]).to(DEV)
    rep = torch.zeros(3, nb_cap, 4, 8, 128, dtype=torch.bfloat16, device=DEV)
    for t in range(steps):
        pos0 = torch.tensor([l + t for l in lens], dtype=torch.int32, device=DEV)
        kn = torch.stack([k[l + t:l + t + 1] for k, l in zip(ks, lens)]).to(DEV)
        vn = torch.stack([v[l + t:l + t + 1] for v, l in zip(vs, lens)]).to(DEV)
        B.append_kv(cs, 3, 1, kn, vn, pos0, kc, vc, kc.stride(0), rep, rep.stride(0), nb_cap)
    torch.cuda.synchronize()
    for i, l in enumerate(lens):
        assert torch.equal(kc[i].cpu(), H.blocked_k(ks[i], sh, nb_cap))
        assert torch.equal(vc[i].cpu(), H.blocked_vt(vs[i], sh, nb_cap))
        want = orc.representative_keys(ks[i].float().numpy(), 128, 4)
        newly = [b for b in range(want.shape[0]) if b * 128 + 128 > l]     # finished during the steps
        for b in range(nb_cap):
            if b in newly:
                assert np.array_equal(rep[i, b].float().cpu().numpy(), want[b]), f"seq {i} block {b}"
            else:
                assert not rep[i, b].any()


@pytest.mark.parametrize("dtype,hq,hkv,d", [("bf16", 32, 8, 128), ("fp32", 6, 2, 64)])
def test_append_and_probe_in_one_launch(dtype, hq, hkv, d):
    """actqkv_append_kv_probe = actqkv_append_kv (m = 1) + actqkv_build_probe (m = 1), bit for
    bit, including a token that completes a block (its representatives are picked)."""
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    bt, nb = 3, 6
    g = torch.Generator().manual_seed(5 + d)
    kc0 = torch.randn(bt, nb, hkv, 128, d, generator=g).to(td).to(DEV)
    vc0 = torch.randn(bt, nb, hkv, d, 128, generator=g).to(td).to(DEV)
    rep0 = torch.randn(bt, nb, 4, hkv, d, generator=g).to(td).to(DEV)
    q = torch.randn(bt, hq, d, generator=g).to(td).to(DEV)
    kn = torch.randn(bt, 1, hkv, d, generator=g).to(td).to(DEV)
    vn = torch.randn(bt, 1, hkv, d, generator=g).to(td).to(DEV)
    pos0 = torch.tensor([300, 383, 5], dtype=torch.int32, device=DEV)      # 383 completes block 2
    res = []
    for fused in (False, True):
        kc, vc, rep = kc0.clone(), vc0.clone(), rep0.clone()
        probe = torch.zeros(bt, hq * d, device=DEV)
        pkv = torch.zeros(bt, hkv * d, device=DEV)
        pn = torch.zeros(bt, device=DEV)
        if fused:
            B.append_kv_probe(cs, bt, q, kn, vn, pos0, kc, vc, kc.stride(0), rep, rep.stride(0), nb, probe, pkv, pn)
        else:
            ws = torch.zeros(B.workspace_bytes(cs, bt, 1, nb, 4), dtype=torch.uint8, device=DEV)
            B.append_kv(cs, bt, 1, kn, vn, pos0, kc, vc, kc.stride(0), rep, rep.stride(0), nb)
            B.build_probe(cs, bt, 1, q, None, False, probe, pkv, pn, None, ws)
        torch.cuda.synchronize()
        res.append((kc, vc, rep, probe, pkv, pn))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    assert not torch.equal(res[1][2][1, 2], rep0[1, 2])                     # the representatives of block 2 were written
    assert torch.equal(res[1][3], q.float().reshape(bt, -1))                # the probe is the query


@pytest.mark.parametrize("dtype,hq,hkv,d", [("bf16", 32, 8, 128), ("fp32", 6, 2, 64)])
@pytest.mark.parametrize("update", [True, False])
def test_decode_retrieve_equals_the_four_calls(dtype, hq, hkv, d, update):
    """actqkv_decode_retrieve = actqkv_append_kv (m = 1) + actqkv_build_probe (m = 1) +
    actqkv_score_blocks + actqkv_select: caches, representatives, probe and selection bit for
    bit, norm and scores up to the order of one fp32 sum.  Ragged lengths (many scoring
    workgroups per sequence, one sequence with no eligible block, one whose token completes a
    block), the cut-off on, three steps in a row."""
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    pos = [9000, 5000, 300, 8831]                       # 8831 completes block 68
    bt, nb, k_cap = len(pos), 72, 12
    nb_begin = 1
    ends = [H.eligible_range(sh, p)[1] for p in pos]
    assert max(ends) - nb_begin > 48 and min(ends) <= nb_begin
    g = torch.Generator().manual_seed(11 + d)
    kc0 = torch.randn(bt, nb, hkv, 128, d, generator=g).to(td).to(DEV)
    vc0 = torch.randn(bt, nb, hkv, d, 128, generator=g).to(td).to(DEV)
    rep0 = torch.randn(bt, nb, 4, hkv, d, generator=g).to(td).to(DEV)
    pos0 = torch.tensor(pos, dtype=torch.int32, device=DEV)
    nb_end = torch.tensor(ends, dtype=torch.int32, device=DEV)
    stride = nb
    steps = []
    for t in range(3):
        steps.append([torch.randn(bt, hq, d, generator=g).to(td).to(DEV),
                      torch.randn(bt, 1, hkv, d, generator=g).to(td).to(DEV),
                      torch.randn(bt, 1, hkv, d, generator=g).to(td).to(DEV)])
    res = []
    for one_call in (False, True):
        kc, vc, rep = kc0.clone(), vc0.clone(), rep0.clone()
        ws = torch.zeros(B.workspace_bytes(cs, bt, 1, nb, k_cap), dtype=torch.uint8, device=DEV)
        bud = torch.full((bt,), 40.0, device=DEV)
        got = []
        for q, kn, vn in steps:
            probe = torch.zeros(bt, hq * d, device=DEV); pkv = torch.zeros(bt, hkv * d, device=DEV)
            pn = torch.zeros(bt, device=DEV)
            scores = torch.zeros(bt, stride, device=DEV)
            idx = torch.zeros(bt, k_cap, dtype=torch.int32, device=DEV)
            n_sel = torch.zeros(bt, dtype=torch.int32, device=DEV)
            theta = torch.zeros(bt, device=DEV); b_l = torch.zeros(bt, device=DEV)
            rest = torch.full((bt,), 9.0, device=DEV)
            if one_call:
                B.decode_retrieve(cs, bt, q, kn if update else None, vn if update else None,
                                  pos0 if update else None, kc, vc, kc.stride(0), rep, rep.stride(0), nb,
                                  nb_begin, nb_end, probe, pkv, pn, scores, stride, k_cap, bud, rest, idx,
                                  n_sel, theta, b_l)
            else:
                if update:
                    B.append_kv(cs, bt, 1, kn, vn, pos0, kc, vc, kc.stride(0), rep, rep.stride(0), nb)
                B.build_probe(cs, bt, 1, q, None, False, probe, pkv, pn, None, ws)
                B.score_blocks(cs, bt, pkv, pn, rep, rep.stride(0), nb, nb_begin, nb_end, scores, stride)
                B.select(bt, scores, stride, nb, nb_begin, nb_end, k_cap, bud, rest, idx, n_sel, theta, b_l)
            torch.cuda.synchronize()
            for s_, e in enumerate(ends):
                scores[s_, max(e, 0):] = 0
            got += [probe, pkv, idx, n_sel, pn, scores, theta, b_l, bud.clone()]
        res.append(got + [kc, vc, rep])
    names = ["probe", "probe_kv", "idx", "n_sel", "probe_norm", "scores", "theta", "budget", "budget_remaining"]
    for i, (a, b) in enumerate(zip(*res)):
        if i >= 27 or i % 9 < 4:
            assert torch.equal(a, b), names[i % 9] if i < 27 else "cache"
        else:
            assert torch.allclose(a, b, rtol=2e-6, atol=1e-7), names[i % 9]
    n_sel = res[1][3].cpu().tolist()
    assert n_sel[2] == 0 and min(n_sel[0], n_sel[1], n_sel[3]) >= 1
    if update:
        assert not torch.equal(res[1][-1][3, 68], rep0[3, 68])            # representatives of the completed block


def test_decode_layer_in_one_launch_equals_the_two_launches():
    """actqkv_decode_layer = actqkv_decode_retrieve (scores only) + actqkv_decode_select_attention:
    caches, representatives, scores, selection, density, budgets bit for bit, the output up to the
    order of fp32 sums.  Ragged lengths (one sequence with no eligible block, one whose token
    completes a block, one shorter than the initial tokens), the cut-off on, three steps in a row,
    with the wait for the other workgroups and with every workgroup scoring for itself."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    td = torch.bfloat16
    n_tok = [9001, 5001, 301, 8832, 100]                 # 8832: the token at 8831 completes block 68
    bt, nb, k_cap = len(n_tok), 72, 12
    nb_begin = 1
    ends = [H.eligible_range(sh, n - 1)[1] for n in n_tok]
    g = torch.Generator().manual_seed(77)
    kc0 = torch.randn(bt, nb, 8, 128, 128, generator=g).to(td).to(DEV)
    vc0 = torch.randn(bt, nb, 8, 128, 128, generator=g).to(td).to(DEV)
    rep0 = torch.randn(bt, nb, 4, 8, 128, generator=g).to(td).to(DEV)
    n_ctx = torch.tensor(n_tok, dtype=torch.int32, device=DEV)
    pos0 = n_ctx - 1
    nb_end = torch.tensor(ends, dtype=torch.int32, device=DEV)
    steps = [[torch.randn(bt, 1, 32, 128, generator=g).to(td).to(DEV),
              torch.randn(bt, 1, 8, 128, generator=g).to(td).to(DEV),
              torch.randn(bt, 1, 8, 128, generator=g).to(td).to(DEV)] for _ in range(3)]
    res = []
    for mode in ("two", "one", "one_no_wait"):
        kc, vc, rep = kc0.clone(), vc0.clone(), rep0.clone()
        runner = H.LayerRunner(sh, bt, 1, nb, k_cap, DEV)
        bud = torch.full((bt,), 40.0, device=DEV)
        got = []
        for q, kn, vn in steps:
            rest = torch.full((bt,), 9.0, device=DEV)
            after = torch.zeros_like(bud)
            out = torch.zeros_like(q)
            lse = torch.zeros(bt, 32, 1, device=DEV)
            if mode == "two":
                runner.decode_step_two_launches(q, kc, vc, rep, n_ctx, nb_end, out, bud, rest, after, kn, vn, pos0,
                                                lse=lse)
            else:
                runner.decode_step_one_launch(q, kc, vc, rep, n_ctx, nb_end, out, bud, rest, after,
                                              kn.squeeze(1).contiguous(), vn.squeeze(1).contiguous(), lse=lse,
                                              flags=0 if mode == "one" else B.DECODE_NO_WAIT)
            torch.cuda.synchronize()
            assert not runner.workspace[:8192].any(), "counters left dirty"
            sc = runner.scores.clone()
            for s_, e in enumerate(ends):
                sc[s_, max(e, 0):] = 0
                sc[s_, :nb_begin] = 0
            got += [runner.idx.clone(), runner.n_sel.clone(), sc, runner.theta.clone(), runner.budget.clone(),
                    after.clone(), out, lse]
            bud = after
        res.append(got + [kc, vc, rep])
    names = ["idx", "n_sel", "scores", "theta", "budget", "budget_after", "out", "lse"]
    for other in res[1:]:
        for i, (a, b) in enumerate(zip(res[0], other)):
            name = names[i % 8] if i < 24 else "cache"
            if i >= 24 or i % 8 < 2:
                assert torch.equal(a, b), name
            elif i % 8 < 6:
                assert torch.allclose(a, b, rtol=2e-6, atol=1e-7), name
            else:
                assert float((a.float() - b.float()).abs().max()) <= 1e-2 * float(a.float().abs().max()), name
    assert torch.equal(res[1][6], res[2][6])              # waiting or not: the same bits
    n_sel = res[1][1].cpu().tolist()
    assert n_sel[2] == 0 and n_sel[4] == 0 and min(n_sel[0], n_sel[1], n_sel[3]) >= 1
    assert not torch.equal(res[1][-1][3, 68], rep0[3, 68])            # representatives of the completed block
    # the token sits in the cache where a later step will look for it
    k_log, v_log = _logical_from_blocked(res[1][-3][4].cpu(), res[1][-2][4].cpu(), 100)
    assert torch.equal(k_log[99], steps[-1][1][4, 0].cpu()) and torch.equal(v_log[99], steps[-1][2][4, 0].cpu())


def test_two_streams_with_a_workspace_each():
    """Two independent batches of sequences decode at the same time on two streams, each with
    its own buffers and workspace, ten steps each: the same bits as one after the other."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")
    bt, nb, k_cap, steps = 4, 40, 8, 10
    n0 = 36 * 128 + 17
    i32 = dict(dtype=torch.int32, device=DEV)

    def make(seed):
        g = torch.Generator(device=DEV).manual_seed(seed)
        kc = torch.randn(bt, nb, 8, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
        vc = torch.randn(bt, nb, 8, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
        rep = torch.randn(bt, nb, 4, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
        q = torch.randn(steps, bt, 1, 32, 128, generator=g, device=DEV).to(torch.bfloat16)
        kn = torch.randn(steps, bt, 1, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
        vn = torch.randn(steps, bt, 1, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
        return dict(kc=kc, vc=vc, rep=rep, q=q, kn=kn, vn=vn, runner=H.LayerRunner(sh, bt, 1, nb, k_cap, DEV),
                    out=torch.zeros(steps, bt, 1, 32, 128, dtype=torch.bfloat16, device=DEV),
                    idx=torch.zeros(steps, bt, k_cap, **i32))

    def run(x, stream):
        with torch.cuda.stream(stream):
            for t in range(steps):
                n = n0 + t
                x["runner"].decode_step_two_launches(
                    x["q"][t], x["kc"], x["vc"], x["rep"], torch.full((bt,), n + 1, **i32),
                    torch.full((bt,), H.eligible_range(sh, n)[1], **i32), x["out"][t], None, None, None,
                    x["kn"][t], x["vn"][t], torch.full((bt,), n, **i32))
                x["idx"][t].copy_(x["runner"].idx)

    results = []
    for concurrent in (False, True):
        a, b = make(1), make(2)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        if concurrent:
            run(a, sa); run(b, sb)
        else:
            run(a, sa); torch.cuda.synchronize(); run(b, sb)
        torch.cuda.synchronize()
        results.append((a["out"], a["idx"], a["kc"], b["out"], b["idx"], b["kc"]))
    for u, v_ in zip(*results):
        assert torch.equal(u, v_)


def _replays_equal_eager(step, outputs):
    """Captures step() in a HIP graph; three replays, with eager runs and synchronisations in
    between, must each leave exactly what the eager run leaves in `outputs`."""
    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in range(3):
        for o in outputs:
            o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for o, w_ in zip(outputs, want):
            assert torch.equal(o, w_), f"replay {i}"
        step()
        torch.cuda.synchronize()


def test_graph_replays_of_a_decode_step_and_of_a_prefill_pass():
    """The benchmarked schedules inside HIP graphs: a decode step of two layers in two launches
    each, and a prefill pass in chunks of windows on two streams with the second team of
    attention workgroups."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")
    i32 = dict(dtype=torch.int32, device=DEV)
    bt, nb, k_cap, L = 4, 24, 8, 2
    g = torch.Generator(device=DEV).manual_seed(3)
    kc = torch.randn(L, bt, nb, 8, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
    vc = torch.randn(L, bt, nb, 8, 128, 128, generator=g, device=DEV).to(torch.bfloat16)
    rep = torch.randn(L, bt, nb, 4, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
    q = torch.randn(L, bt, 1, 32, 128, generator=g, device=DEV).to(torch.bfloat16)
    kn = torch.randn(L, bt, 1, 8, 128, generator=g, device=DEV).to(torch.bfloat16)
    n = 20 * 128 + 5
    n_ctx, pos0 = torch.full((bt,), n + 1, **i32), torch.full((bt,), n, **i32)
    nb_end = torch.full((bt,), H.eligible_range(sh, n)[1], **i32)
    runner = H.LayerRunner(sh, bt, 1, nb, k_cap, DEV)
    out = torch.zeros(L, bt, 1, 32, 128, dtype=torch.bfloat16, device=DEV)
    idx = torch.zeros(L, bt, k_cap, **i32)
    buds = [torch.full((bt,), 9.0, device=DEV), torch.zeros(bt, device=DEV), torch.zeros(bt, device=DEV)]
    rest = torch.full((bt,), 2.0, device=DEV)

    def decode():
        for l in range(L):
            runner.decode_step_two_launches(q[l], kc[l], vc[l], rep[l], n_ctx, nb_end, out[l], buds[l], rest,
                                            buds[l + 1], kn[l], kn[l], pos0)
            idx[l].copy_(runner.idx)
    _replays_equal_eager(decode, [out, idx, buds[2]])

    w = synth.scaled(synth.WORKLOADS["c2_32k"], n_ctx=20 * 512 + 100, name="graph_prefill", cutoff=True, k_cap=8)
    qp, k, v = synth.gen_layer(w, "cpu", 0)
    rp = synth.pick_rep_keys(k, 128, 4)
    cut = [synth.cutoff_state(w, H.eligible_range(sh, t * 512)[1] - 1, t, 0) for t in range(w.n_windows)]
    qd, kcp, vcp = qp.to(DEV), H.blocked_k(k.to(DEV), sh, w.n_blocks), H.blocked_vt(v.to(DEV), sh, w.n_blocks)
    repd = torch.zeros(w.n_blocks, 4, 8, 128, dtype=torch.bfloat16, device=DEV)
    repd[: rp.shape[0]] = rp.to(DEV)
    r2 = H.LayerRunner(sh, 1, 512, w.n_blocks, w.k_cap, DEV)
    plan = H.make_prefill_plan(sh, w.n_ctx, 512, cut, DEV)
    bud0 = plan.budget.clone()
    pipe = H.PrefillPipeline(r2, plan)
    outp = torch.zeros_like(qd)

    def prefill():
        r2.stats.zero_()
        plan.budget.copy_(bud0)
        pipe.run(qd, kcp, vcp, repd, outp, overlap=True, chunk=8, batched=True, late_cus=32, attention_cus=224)
    _replays_equal_eager(prefill, [outp, pipe.idx, pipe.n_sel])


@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_group_size_in_decode_and_prefill_attention(group):
    """1 to 8 query heads per KV head, bf16: a decode step in two launches and a prefill window on
    the matrix cores against a plain softmax attention over the keys each row sees."""
    hkv = 2
    sh = LayerShape(group * hkv, hkv, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    i32 = dict(dtype=torch.int32, device=DEV)
    g = torch.Generator().manual_seed(40 + group)
    nb, k_cap, m = 16, 4, 192
    n_tok = nb * 128
    k = torch.randn(n_tok, hkv, 128, generator=g).to(torch.bfloat16)
    v = torch.randn(n_tok, hkv, 128, generator=g).to(torch.bfloat16)
    kc, vc = H.blocked_k(k.to(DEV), sh, nb), H.blocked_vt(v.to(DEV), sh, nb)
    sel = [3, 7, 5]
    idx = torch.tensor([sel + [-1]], **i32)
    n_sel = torch.tensor([3], **i32)
    ws = torch.zeros(B.workspace_bytes(cs, 1, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    for rows, n_ctx in ((1, 1900), (m, 1800 + m)):
        q = torch.randn(rows, group * hkv, 128, generator=g).to(torch.bfloat16)
        out = torch.zeros(rows, group * hkv, 128, dtype=torch.bfloat16, device=DEV)
        B.retrieval_attention(cs, 1, rows, q.to(DEV), kc, vc, 0, nb, torch.tensor([n_ctx], **i32), idx, n_sel, k_cap,
                              out, None, ws)
        torch.cuda.synchronize()
        w0 = n_ctx - rows
        for r in sorted({0, rows // 2, rows - 1}):
            pos = orc.key_positions(w0, w0 + r, sel, sh.n_init, sh.n_local, 128)
            ref = orc.attention_rows(f64(q[r])[None], f64(k), f64(v), pos, group)[0]
            assert out_error(out[r], ref) < TOL_OUT["bf16"], f"rows {rows} row {r}"


def test_selection_on_random_cases():
    """300 random selection problems (sizes, capacities, score scales, ties, cut-off states, both
    density readings) in batches, every one against the oracle."""
    rng = np.random.default_rng(2024)
    for trial in range(10):
        bt = 30
        n_max = int(rng.choice([7, 64, 65, 600, 1100, 3000]))
        k_cap = int(rng.integers(1, 65))
        ns = rng.integers(0, n_max + 1, size=bt)
        nb_begin = int(rng.integers(0, 3))
        stride = nb_begin + n_max + 3
        scores = np.zeros((bt, stride), dtype=np.float32)
        for s_ in range(bt):
            sc = rng.normal(size=ns[s_]) * rng.choice([0.01, 0.3, 3.0])
            if s_ % 3 == 0:
                sc = np.round(sc * 4) / 4                    # exact ties
            scores[s_, nb_begin:nb_begin + ns[s_]] = sc
        use_cut, topk = bool(trial % 2), bool(trial % 3 == 0)
        bud_h = rng.uniform(0.5, 90.0, size=bt).astype(np.float32)
        rest_h = rng.uniform(0.0, 40.0, size=bt).astype(np.float32)
        bud = torch.from_numpy(bud_h.copy()).to(DEV) if use_cut else None
        rest = torch.from_numpy(rest_h).to(DEV) if use_cut else None
        idx = torch.zeros(bt, k_cap, dtype=torch.int32, device=DEV)
        n_sel = torch.zeros(bt, dtype=torch.int32, device=DEV)
        theta = torch.zeros(bt, device=DEV); b_l = torch.zeros(bt, device=DEV)
        B.select(bt, torch.from_numpy(scores).to(DEV), stride, nb_begin + n_max, nb_begin,
                 torch.tensor(nb_begin + ns, dtype=torch.int32, device=DEV), k_cap, bud, rest, idx, n_sel, theta, b_l,
                 flags=B.SELECT_ENTROPY_TOPK if topk else 0)
        torch.cuda.synchronize()
        idx_h, n_h, th_h, bl_h = idx.cpu().tolist(), n_sel.cpu().tolist(), theta.cpu().numpy(), b_l.cpu().numpy()
        for s_ in range(bt):
            n = int(ns[s_])
            if n == 0:
                assert n_h[s_] == 0 and all(x == -1 for x in idx_h[s_])
                continue
            sc = scores[s_, nb_begin:nb_begin + n].astype(np.float64)
            th = orc.information_density_topk(sc, k_cap) if topk else orc.information_density(sc)
            assert abs(th_h[s_] - th) < TOL_THETA, (trial, s_)
            if use_cut:
                bl = orc.layer_budget(th, float(rest_h[s_]), float(bud_h[s_]))
                assert abs(bl_h[s_] - bl) < TOL_BUDGET * max(bl, 1.0)
                if abs(bl + 0.5 - round(bl + 0.5)) < 1e-3:
                    continue                                 # B^l at a rounding boundary: either count is right
                count = orc.cutoff_count(bl, k_cap, n)
            else:
                count = min(k_cap, n)
            want = orc.select_blocks(scores[s_, nb_begin:nb_begin + n], list(range(nb_begin, nb_begin + n)), count)
            assert n_h[s_] == count and idx_h[s_][:count] == want, (trial, s_)
            assert all(x == -1 for x in idx_h[s_][count:])


def test_scores_on_random_shapes():
    """40 random shapes (heads, group, channels, representative keys, batch, blocks, both storage
    types; shared or per-sequence keys): block scores, head-merged and per KV head, and the
    decode scoring launch against the oracle."""
    rng = np.random.default_rng(77)
    for trial in range(40):
        hkv = int(rng.choice([1, 2, 4, 8])); group = int(rng.integers(1, 9)); d = int(rng.choice([64, 128]))
        if hkv * group * d > 16384:
            continue
        n_rep = int(rng.integers(1, 17)); bt = int(rng.integers(1, 6)); nb = int(rng.integers(2, 70))
        dtype = "bf16" if trial % 2 else "fp32"
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        sh = LayerShape(hkv * group, hkv, d, 128, n_rep, 128, 256, dtype)
        cs = B.c_shape(sh)
        shared = trial % 5 == 0
        g = torch.Generator().manual_seed(trial)
        rep = torch.randn(1 if shared else bt, nb, n_rep, hkv, d, generator=g).to(td)
        q = torch.randn(bt, 1, hkv * group, d, generator=g).to(td)
        nb_begin = 1
        ends = rng.integers(0, nb + 1, size=bt)
        repd, qd = rep.to(DEV), q.to(DEV)
        nb_end = torch.tensor(ends, dtype=torch.int32, device=DEV)
        r = H.LayerRunner(sh, bt, 1, nb, 4, DEV)
        B.build_probe(cs, bt, 1, qd, None, False, r.probe, r.probe_kv, r.probe_norm, None, r.workspace)
        B.score_blocks(cs, bt, r.probe_kv, r.probe_norm, repd, 0 if shared else repd.stride(0), nb, nb_begin, nb_end,
                       r.scores, r.score_stride)
        ph = torch.zeros(bt, hkv, r.score_stride, device=DEV)
        B.score_blocks_per_head(cs, bt, r.probe, repd, 0 if shared else repd.stride(0), nb, nb_begin,
                                nb_end.repeat_interleave(hkv).contiguous(), ph, r.score_stride)
        fused = torch.zeros_like(r.scores)
        if not shared:
            B.decode_retrieve(cs, bt, qd, None, None, None, None, None, 0, repd, repd.stride(0), nb, nb_begin, nb_end,
                              None, None, None, fused, r.score_stride, 4, None, None, None, None, None, None,
                              flags=B.DECODE_SCORES_ONLY)
        torch.cuda.synchronize()
        for s_ in range(bt):
            e = int(ends[s_])
            if e <= nb_begin:
                continue
            keys = f64(rep[0 if shared else s_, nb_begin:e])
            want = orc.block_scores(f64(q[s_, 0]).reshape(-1), keys, group)
            assert np.abs(f64(r.scores[s_, nb_begin:e]) - want).max() < TOL_SCORE, (trial, s_)
            want_ph = orc.block_scores_per_head(f64(q[s_, 0]).reshape(-1), keys, group)
            assert np.abs(f64(ph[s_, :, nb_begin:e]) - want_ph).max() < TOL_SCORE, (trial, s_)
            if not shared:
                assert np.abs(f64(fused[s_, nb_begin:e]) - want).max() < TOL_SCORE, (trial, s_)


@pytest.mark.parametrize("hkv,group,d,n_rep,bt,nb", [
    (8, 4, 128, 4, 32, 300),     # the benchmarked shape: 32 windows of one call, more than one round of tiles
    (8, 4, 128, 4, 37, 75),      # a second, ragged group of windows; blocks that are no multiple of a tile
    (4, 2, 128, 2, 5, 41),       # two keys a block, fewer windows than a tile has rows
    (2, 3, 64, 1, 9, 130),       # one key a block, short keys
    (8, 4, 128, 4, 4, 9),        # hardly a tile
])
def test_scores_of_many_windows_on_shared_keys(hkv, group, d, n_rep, bt, nb):
    """Several windows of one sequence scored in one call (seq_stride 0, bf16): the matrix-core
    kernel, every window with its own end of the eligible blocks, against the oracle window by
    window; blocks at and beyond a window's end keep what the buffer held."""
    sh = LayerShape(hkv * group, hkv, d, 128, n_rep, 128, 256, "bf16")
    cs = B.c_shape(sh)
    _say(f"[case] shared-key scores Hk{hkv} G{group} D{d} r{n_rep} windows {bt} blocks {nb}")
    g = torch.Generator().manual_seed(1000 * bt + nb)
    rep = (torch.randn(nb, n_rep, hkv, d, generator=g) * 1.3).to(torch.bfloat16)
    rep[3] = 0                                                        # a block of zero keys scores 0
    q = (torch.randn(bt, 1, hkv * group, d, generator=g) + 0.2).to(torch.bfloat16)
    q[bt - 1] = 0                                                     # and so does a zero probe
    rng = np.random.default_rng(nb)
    ends = rng.integers(0, nb + 1, size=bt)
    ends[0] = nb
    nb_begin = 1
    repd, qd = rep.to(DEV), q.to(DEV)
    nb_end = torch.tensor(ends, dtype=torch.int32, device=DEV)
    r = H.LayerRunner(sh, bt, 1, nb, 4, DEV)
    B.build_probe(cs, bt, 1, qd, None, False, r.probe, r.probe_kv, r.probe_norm, None, r.workspace)
    r.scores.fill_(-7.0)
    B.score_blocks(cs, bt, r.probe_kv, r.probe_norm, repd, 0, nb, nb_begin, nb_end, r.scores, r.score_stride)
    torch.cuda.synchronize()
    got = f64(r.scores)
    for s_ in range(bt):
        e = max(int(ends[s_]), nb_begin)
        assert (got[s_, :nb_begin] == -7.0).all() and (got[s_, e:] == -7.0).all(), s_
        if e > nb_begin:
            want = orc.block_scores(f64(q[s_, 0]).reshape(-1), f64(rep[nb_begin:e]), group)
            assert np.abs(got[s_, nb_begin:e] - want).max() < TOL_SCORE, s_
            if nb_begin <= 3 < e:
                assert got[s_, 3] == 0.0
    assert (got[bt - 1, nb_begin:max(int(ends[bt - 1]), nb_begin)] == 0.0).all()


def test_scores_of_many_windows_on_random_shapes():
    """25 random problems for the scoring of several windows on shared keys (heads, group, channels,
    keys per block, windows, blocks, first eligible block, ragged ends), against the oracle."""
    rng = np.random.default_rng(4242)
    for trial in range(25):
        hkv, d = [(8, 128), (4, 128), (2, 128), (4, 64), (8, 64), (1, 128)][int(rng.integers(0, 6))]
        group = int(rng.integers(1, 9)); n_rep = int(rng.choice([1, 2, 4])); bt = int(rng.integers(4, 70))
        nb = int(rng.integers(2, 140)); nb_begin = int(rng.integers(0, min(nb, 3)))
        if hkv * group * d > 16384:
            continue
        sh = LayerShape(hkv * group, hkv, d, 128, n_rep, 128, 256, "bf16")
        cs = B.c_shape(sh)
        _say(f"[case] shared-key scores, trial {trial}: Hk{hkv} G{group} D{d} r{n_rep} windows {bt} blocks {nb} from {nb_begin}")
        g = torch.Generator().manual_seed(trial)
        rep = (torch.randn(nb, n_rep, hkv, d, generator=g) * float(rng.uniform(0.3, 2.0))).to(torch.bfloat16)
        q = (torch.randn(bt, 1, hkv * group, d, generator=g) + float(rng.uniform(-0.5, 0.5))).to(torch.bfloat16)
        ends = rng.integers(0, nb + 1, size=bt)
        repd, qd = rep.to(DEV), q.to(DEV)
        nb_end = torch.tensor(ends, dtype=torch.int32, device=DEV)
        r = H.LayerRunner(sh, bt, 1, nb, 4, DEV)
        B.build_probe(cs, bt, 1, qd, None, False, r.probe, r.probe_kv, r.probe_norm, None, r.workspace)
        r.scores.fill_(3.0)
        B.score_blocks(cs, bt, r.probe_kv, r.probe_norm, repd, 0, nb, nb_begin, nb_end, r.scores, r.score_stride)
        torch.cuda.synchronize()
        got = f64(r.scores)
        for s_ in range(bt):
            e = max(int(ends[s_]), nb_begin)
            assert (got[s_, :nb_begin] == 3.0).all() and (got[s_, e:] == 3.0).all(), (trial, s_)
            if e > nb_begin:
                want = orc.block_scores(f64(q[s_, 0]).reshape(-1), f64(rep[nb_begin:e]), group)
                assert np.abs(got[s_, nb_begin:e] - want).max() < TOL_SCORE, (trial, s_)


def test_probe_on_random_shapes():
    """30 random shapes (heads, channels, window lengths from 2 to 700, batch, storage type, mean
    pooling or not): two windows per sequence, statistics, weights, probe, its group sum and its
    norm against the oracle."""
    rng = np.random.default_rng(99)
    for trial in range(30):
        hkv = int(rng.choice([1, 2, 4, 8])); group = int(rng.integers(1, 9)); d = int(rng.choice([64, 128]))
        if hkv * group * d > 16384:
            continue
        m = int(rng.choice([2, 3, 17, 64, 100, 255, 256, 513, 700])); bt = int(rng.integers(1, 5))
        dtype = "bf16" if trial % 2 else "fp32"
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        pooling = trial % 7 == 0
        hq, dd = hkv * group, hkv * group * d
        sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
        cs = B.c_shape(sh)
        g = torch.Generator().manual_seed(1000 + trial)
        q = (torch.randn(bt, 2 * m, hq, d, generator=g) * float(rng.uniform(0.3, 3.0)) + float(rng.normal())).to(td)
        q[:, rng.integers(0, 2 * m), :, rng.integers(0, d)] *= 12.0
        qd = q.to(DEV)
        r = H.LayerRunner(sh, bt, m, 8, 4, DEV)
        wts = torch.zeros(bt, m, device=DEV)
        flags = B.STATS_UPDATE | (B.PROBE_MEAN_POOLING if pooling else 0)
        stats = [orc.RunningStats(dd) for _ in range(bt)]
        for t in range(2):
            B.build_probe(cs, bt, m, qd[:, t * m:(t + 1) * m].contiguous(), r.stats, flags, r.probe, r.probe_kv,
                          r.probe_norm, wts, r.workspace)
            torch.cuda.synchronize()
            for s_ in range(bt):
                qw = f64(q[s_, t * m:(t + 1) * m]).reshape(m, dd)
                z_bar, sigma2 = stats[s_].update(qw)
                if pooling:
                    probe, weights = qw.mean(axis=0), np.full(m, 1.0 / m)
                else:
                    probe, weights = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2))
                assert rel_to_max(r.probe[s_], probe) < TOL_PROBE, (trial, t, s_)
                assert rel_to_max(wts[s_], weights) < TOL_WEIGHT, (trial, t, s_)
                kv = probe.reshape(hkv, group, d).sum(axis=1).reshape(-1)
                assert rel_to_max(r.probe_kv[s_], kv) < TOL_PROBE * group, (trial, t, s_)
                assert abs(float(r.probe_norm[s_]) - np.linalg.norm(probe)) < TOL_PROBE * np.linalg.norm(probe)


def test_attention_on_random_shapes():
    """40 random attention problems: heads, group, channels, storage type, window length (1 for a
    decode step up to 600), context, initial tokens and local span, batch entries with their
    own caches or sharing one, random selections; sampled rows against the oracle."""
    rng = np.random.default_rng(4242)
    for trial in range(40):
        hkv = int(rng.choice([1, 2, 4, 8])); group = int(rng.integers(1, 9)); d = int(rng.choice([64, 128]))
        dtype = "bf16" if trial % 3 else "fp32"
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        n_init, n_local = 128 * int(rng.integers(0, 3)), 128 * int(rng.integers(0, 4))
        m = int(rng.choice([1, 1, 2, 31, 64, 100, 256, 257, 600])); bt = int(rng.integers(1, 4))
        shared = bt > 1 and trial % 4 == 0
        hq = hkv * group
        sh = LayerShape(hq, hkv, d, 128, 4, n_init, n_local, dtype)
        cs = B.c_shape(sh)
        k_cap = int(rng.integers(1, 9))
        nb = int(rng.integers((m + 127) // 128 + 1, 30))
        g = torch.Generator().manual_seed(7000 + trial)
        ks = [torch.randn(nb * 128, hkv, d, generator=g).to(td) for _ in range(1 if shared else bt)]
        vs = [torch.randn(nb * 128, hkv, d, generator=g).to(td) for _ in range(1 if shared else bt)]
        kc = torch.stack([H.blocked_k(x.to(DEV), sh, nb) for x in ks])
        vc = torch.stack([H.blocked_vt(x.to(DEV), sh, nb) for x in vs])
        q = torch.randn(bt, m, hq, d, generator=g).to(td)
        n_ctx = [int(rng.integers(m, nb * 128 + 1)) for _ in range(bt)]
        idx = torch.full((bt, k_cap), -1, dtype=torch.int32)
        n_sel = torch.zeros(bt, dtype=torch.int32)
        chosen = []
        for s_ in range(bt):
            b, e = H.eligible_range(sh, n_ctx[s_] - m)
            cnt = int(rng.integers(0, min(k_cap, max(e - b, 0)) + 1))
            pick = (rng.permutation(max(e - b, 0))[:cnt] + b).tolist()
            idx[s_, :cnt] = torch.tensor(pick, dtype=torch.int32)
            n_sel[s_] = cnt
            chosen.append(pick)
        out = torch.zeros(bt, m, hq, d, dtype=td, device=DEV)
        ws = torch.zeros(B.workspace_bytes(cs, bt, m, nb, k_cap), dtype=torch.uint8, device=DEV)
        B.retrieval_attention(cs, bt, m, q.to(DEV), kc, vc, 0 if shared else kc.stride(0), nb,
                              torch.tensor(n_ctx, dtype=torch.int32, device=DEV), idx.to(DEV), n_sel.to(DEV), k_cap,
                              out, None, ws)
        torch.cuda.synchronize()
        for s_ in range(bt):
            kk, vv = (ks[0], vs[0]) if shared else (ks[s_], vs[s_])
            w0 = n_ctx[s_] - m
            for r in sorted({0, m // 2, m - 1}):
                pos = orc.key_positions(w0, w0 + r, chosen[s_], n_init, n_local, 128)
                ref = orc.attention_rows(f64(q[s_, r])[None], f64(kk), f64(vv), pos, group)[0]
                err = out_error(out[s_, r], ref)
                assert err < TOL_OUT[dtype], (trial, s_, r, err, dict(hkv=hkv, group=group, d=d, dtype=dtype, m=m,
                                                                    n_init=n_init, n_local=n_local, n_ctx=n_ctx[s_]))


def test_decode_step_on_a_cache_of_one_block():
    """The first tokens of a sequence: one cache block, nothing eligible.  The two-launch step
    writes the token, the probe and an empty selection, and attends over what is there."""
    sh = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    cs = B.c_shape(sh)
    bt, nb, k_cap = 3, 1, 4
    g = torch.Generator().manual_seed(9)
    pos = [0, 5, 127]
    k = torch.randn(bt, 128, 2, 128, generator=g).to(torch.bfloat16)
    v = torch.randn(bt, 128, 2, 128, generator=g).to(torch.bfloat16)
    q = torch.randn(bt, 1, 8, 128, generator=g).to(torch.bfloat16).to(DEV)
    kc = torch.zeros(bt, nb, 2, 128, 128, dtype=torch.bfloat16, device=DEV)
    vc = torch.zeros(bt, nb, 2, 128, 128, dtype=torch.bfloat16, device=DEV)
    for s, p_ in enumerate(pos):                           # the cache holds the tokens before the new one
        kc[s] = H.blocked_k(torch.cat([k[s, :p_], torch.zeros(128 - p_, 2, 128, dtype=torch.bfloat16)]).to(DEV), sh, nb)
        vc[s] = H.blocked_vt(torch.cat([v[s, :p_], torch.zeros(128 - p_, 2, 128, dtype=torch.bfloat16)]).to(DEV), sh, nb)
    rep = torch.zeros(bt, nb, 4, 2, 128, dtype=torch.bfloat16, device=DEV)
    k_new = torch.stack([k[s, p_] for s, p_ in enumerate(pos)]).unsqueeze(1).to(DEV)
    v_new = torch.stack([v[s, p_] for s, p_ in enumerate(pos)]).unsqueeze(1).to(DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    runner = H.LayerRunner(sh, bt, 1, nb, k_cap, DEV)
    out = torch.zeros_like(q)
    runner.idx.fill_(7)
    runner.decode_step_two_launches(q, kc, vc, rep, torch.tensor([p_ + 1 for p_ in pos], **i32),
                                    torch.tensor([1] * bt, **i32), out, None, None, None, k_new, v_new,
                                    torch.tensor(pos, **i32))
    torch.cuda.synchronize()
    assert runner.n_sel.cpu().tolist() == [0] * bt and bool((runner.idx == -1).all())
    assert torch.equal(runner.probe.cpu(), q.float().reshape(bt, -1).cpu())
    assert rep[2].any() and not rep[:2].any()              # position 127 completes the block: representatives picked
    for s, p_ in enumerate(pos):
        res = orc.decode_step(f64(q[s, 0].cpu()), f64(k[s, :p_ + 1]), f64(v[s, :p_ + 1]), np.zeros((0, 4, 2, 128)),
                              p_ + 1, sh.n_init, sh.n_local, 128, k_cap, None)
        assert out_error(out[s, 0], res["out"]) < TOL_OUT["bf16"], f"sequence {s}"


def test_append_kv_drops_tokens_behind_the_capacity():
    sh = LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32")
    cs = B.c_shape(sh)
    k = torch.randn(200, 2, 64); v = torch.randn(200, 2, 64)
    kc = torch.zeros(1, 2, 128, 64, device=DEV); vc = torch.zeros(1, 2, 64, 128, device=DEV)
    guard_k, guard_v = torch.full((4096,), 7.0, device=DEV), torch.full((4096,), 7.0, device=DEV)
    pos0 = torch.tensor([0], dtype=torch.int32, device=DEV)
    B.append_kv(cs, 1, 200, k.to(DEV), v.to(DEV), pos0, kc, vc, 0, None, 0, 1)
    torch.cuda.synchronize()
    assert torch.equal(kc.cpu(), H.blocked_k(k[:128], sh, 1)) and torch.equal(vc.cpu(), H.blocked_vt(v[:128], sh, 1))
    assert bool((guard_k == 7).all()) and bool((guard_v == 7).all())


# ---------------------------------------------------------------- cut-off across layers and steps
def test_cutoff_history_across_layers_and_steps():
    """Alg. 1 with the history of densities kept on the device: every step, every layer's
    budget, count and selection against the oracle, for three sequences with different scores."""
    L, bt, steps, k_cap, k_mean, n = 6, 3, 5, 16, 5.0, 200
    prior = math.log(n)
    rng = np.random.default_rng(77)
    sharp = rng.uniform(0.5, 12.0, size=(L, bt))            # how peaked each layer's scores are
    theta_sum = torch.zeros(bt, L, device=DEV); n_steps = torch.zeros(bt, device=DEV)
    budget = torch.zeros(bt, device=DEV); rest = torch.zeros(L, bt, device=DEV)
    theta_step = torch.zeros(L, bt, device=DEV)
    idx = torch.zeros(bt, k_cap, dtype=torch.int32, device=DEV)
    n_sel = torch.zeros(L, bt, dtype=torch.int32, device=DEV)
    b_out = torch.zeros(L, bt, device=DEV)
    nb_end = torch.full((bt,), n, dtype=torch.int32, device=DEV)
    hists = [orc.CutoffHistory(L, prior) for _ in range(bt)]
    for t in range(steps):
        B.cutoff_next_step(bt, L, k_mean, prior, theta_step if t > 0 else None, theta_sum, n_steps, budget, rest)
        torch.cuda.synchronize()
        want_rest = np.array([h.rest_sums() for h in hists]).T                      # [L][bt]
        assert np.allclose(rest.cpu().numpy(), want_rest, rtol=1e-5, atol=1e-6), f"rest sums, step {t}"
        assert np.allclose(budget.cpu().numpy(), L * k_mean)
        scores = rng.standard_normal((L, bt, n)).astype(np.float32) * 0.05
        scores[:, :, :8] += (sharp[:, :, None] * rng.uniform(0.5, 1.0, size=(L, bt, 8))).astype(np.float32) * 0.1
        sd = torch.from_numpy(scores).to(DEV)
        for l in range(L):
            B.select(bt, sd[l], n, n, 0, nb_end, k_cap, budget, rest[l], idx, n_sel[l], theta_step[l], b_out[l])
        torch.cuda.synchronize()
        for s in range(bt):
            thetas = [orc.information_density(f64(scores[l, s])) for l in range(L)]
            assert np.allclose(theta_step[:, s].cpu().numpy(), thetas, atol=TOL_THETA)
            b_want = orc.step_budgets(thetas, hists[s].rest_sums(), k_mean)
            assert np.allclose(b_out[:, s].cpu().numpy(), b_want, rtol=TOL_BUDGET, atol=TOL_BUDGET)
            for l in range(L):
                if abs(b_want[l] + 0.5 - round(b_want[l] + 0.5)) > 1e-3:            # not at a rounding edge
                    assert int(n_sel[l, s]) == orc.cutoff_count(b_want[l], k_cap, n), f"E, step {t} layer {l} seq {s}"
            hists[s].add_step(thetas)
    B.cutoff_next_step(bt, L, k_mean, prior, theta_step, theta_sum, n_steps, budget, rest)
    torch.cuda.synchronize()
    assert np.allclose(n_steps.cpu().numpy(), steps)
    assert np.allclose(theta_sum.cpu().numpy() / steps, np.array([h.means() for h in hists]), rtol=1e-5)


def test_planted_block_recall_per_variant_equals_the_oracles():
    """The recall statistic bench.py reports for the retrieval variants of the ablation (Sec. 5.3,
    Table 3), on a reduced workload with strongly planted blocks: computed from the library's
    selections and from the oracle's, variant by variant (probe-Query or mean pooling, fixed k or
    cut-off, one selection or one per KV head)."""
    import bench
    base = synth.scaled(synth.WORKLOADS["c3_128k"], n_ctx=16384, alpha=16.0, shift=2.0, n_planted=12)
    sh, m, kc = base.shape, base.window, base.k_cap
    _say("[case] recall per variant, 16K tokens, strong planted signal")
    sel_gpu = {}
    got = bench._recall_of(base, torch, B, H, synth, sel_gpu)
    # the order in which the bench takes its selections
    sel_gpu = dict(zip(("probe_query_fixed_k", "mean_pooling_fixed_k", "per_kv_head_fixed_k", "probe_query_cutoff"),
                       (sel_gpu[i] for i in range(4))))
    q, k, _ = synth.gen_layer(base, DEV)         # the bench draws its inputs on the device: the same ones here
    rep = f64(synth.pick_rep_keys(k, sh.block_size, sh.n_rep))
    planted = set(synth.planted_blocks(base))
    T = base.n_ctx // m
    nb_begin = sh.n_init // sh.block_size
    stats = orc.RunningStats(sh.d_model)
    tally = {n: [0, 0, 0] for n in sel_gpu}
    near_cut = 5e-4          # the GPU's probe is an fp32 one: blocks this close to the cut may change sides
    for t in range(T):
        flat = f64(q[t * m:(t + 1) * m]).reshape(m, -1)
        z, s2 = stats.update(flat)
        probe, _ = orc.probe_query(flat, orc.activation_bias(flat, z, s2))
        pooled, _ = orc.probe_query(flat, np.ones_like(flat))
        w0 = t * m
        end = H.eligible_range(sh, w0)[1]
        cut = synth.cutoff_state(base, max(end - nb_begin, 0), t, 0)
        sels = {"probe_query_fixed_k": [orc.retrieve(probe, rep, w0, sh.n_init, sh.n_local, 128, sh.group, kc)],
                "mean_pooling_fixed_k": [orc.retrieve(pooled, rep, w0, sh.n_init, sh.n_local, 128, sh.group, kc)],
                "probe_query_cutoff": [orc.retrieve(probe, rep, w0, sh.n_init, sh.n_local, 128, sh.group, kc, cut)],
                "per_kv_head_fixed_k": orc.retrieve_per_head(probe, rep, w0, sh.n_init, sh.n_local, 128, sh.group, kc)}
        p = {b for b in planted if nb_begin <= b < end}
        for name, rows in sels.items():
            for j, res in enumerate(rows):
                row = t * len(rows) + j
                gi, gn = sel_gpu[name][0][row], sel_gpu[name][1][row]
                assert gn == res["count"], (name, t, j)
                differ = set(gi[:gn]) ^ set(res["idx"])
                if differ:
                    score_of = dict(zip(res["eligible"], res["scores"]))
                    kth = sorted(res["scores"], reverse=True)[res["count"] - 1]
                    assert all(abs(score_of[b] - kth) < near_cut for b in differ), (name, t, j, differ)
                if p:
                    tally[name][0] += len(set(res["idx"]) & p)
                    tally[name][1] += len(res["idx"])
                    tally[name][2] += len(p)
    for name, (hit, sel, tot) in tally.items():
        want_recall, want_prec = hit / max(tot, 1), hit / max(sel, 1)
        _say(f"  {name}: recall {got[name]['recall']:.4f} (oracle {want_recall:.4f}), "
             f"precision {got[name]['precision']:.4f} (oracle {want_prec:.4f})")
        # blocks that all but tie at the cut may change sides: a few hits either way
        assert abs(got[name]["recall"] - want_recall) <= 0.01, name
        assert abs(got[name]["precision"] - want_prec) <= 0.01, name
    assert got["probe_query_fixed_k"]["recall"] > got["mean_pooling_fixed_k"]["recall"]


@pytest.mark.parametrize("topk", [False, True])
def test_algorithm_1_in_its_three_loops(topk):
    """Alg. 1 as it is printed: the density of every layer first (actqkv_select, density only),
    then every budget (actqkv_cutoff_budgets: the mean density of a layer still to come is that
    layer's own), then the selections with the counts given.  Against the oracle: densities,
    budgets (which also telescope to L k theta^l / sum theta, with nothing left of B_kv), counts
    and selected blocks, for sequences with different eligible ranges (one with a single block,
    one with none) and the density over all eligible blocks or over the k_cap best ones."""
    L, bt, k_cap, k_mean = 7, 5, 24, 6.0
    n_blocks = [300, 1200, 40, 1, 0]
    n_max = max(n_blocks) + 2
    nb_begin = 2
    rng = np.random.default_rng(404 + topk)
    sharp = rng.uniform(0.5, 30.0, size=(L, bt))
    scores = rng.standard_normal((L, bt, n_max)).astype(np.float32) * 0.05
    scores[:, :, nb_begin:nb_begin + 6] += (sharp[:, :, None] * rng.uniform(0.5, 1.0, size=(L, bt, 6))).astype(np.float32) * 0.1
    sd = torch.from_numpy(scores).to(DEV)
    nb_end = torch.tensor([nb_begin + n for n in n_blocks], dtype=torch.int32, device=DEV)
    theta = torch.full((L, bt), -1.0, device=DEV)
    budget = torch.zeros(L, bt, device=DEV)
    count = torch.zeros(L, bt, dtype=torch.int32, device=DEV)
    left = torch.full((bt,), 9.0, device=DEV)
    idx = torch.full((L, bt, k_cap), -7, dtype=torch.int32, device=DEV)
    b_rep = torch.zeros(L, bt, device=DEV)
    flag_t = B.SELECT_ENTROPY_TOPK if topk else 0
    for l in range(L):                                   # first loop: densities only
        B.select(bt, sd[l], n_max, n_max, nb_begin, nb_end, k_cap, None, None, idx[l], count[l], theta[l], None,
                 flags=B.SELECT_DENSITY_ONLY | flag_t)
    torch.cuda.synchronize()
    assert bool((idx == -7).all()) and bool((count == 0).all())          # nothing but theta was written
    B.cutoff_budgets(bt, L, k_mean, k_cap, theta, budget, count, left)   # second loop
    torch.cuda.synchronize()
    given = count.clone()
    for l in range(L):                                   # third loop: the selections
        B.select(bt, sd[l], n_max, n_max, nb_begin, nb_end, k_cap, None, None, idx[l], count[l], None, b_rep[l],
                 flags=B.SELECT_GIVEN_COUNT | flag_t)
    torch.cuda.synchronize()
    th, bu = theta.cpu().numpy(), budget.cpu().numpy()
    for s, n in enumerate(n_blocks):
        el = [f64(scores[l, s, nb_begin:nb_begin + n]) for l in range(L)]
        if n == 0:
            want_t = [0.0] * L
        else:
            want_t = [orc.information_density_topk(e, k_cap) if topk else orc.information_density(e) for e in el]
        assert np.allclose(th[:, s], want_t, atol=TOL_THETA), f"densities, sequence {s}"
        rest = [sum(want_t[l + 1:]) for l in range(L)]
        want_b = orc.step_budgets(want_t, rest, k_mean)
        assert np.allclose(bu[:, s], want_b, rtol=TOL_BUDGET, atol=TOL_BUDGET), f"budgets, sequence {s}"
        if sum(want_t) > 0:
            closed = [L * k_mean * t / sum(want_t) for t in want_t]       # the budgets telescope
            assert np.allclose(bu[:, s], closed, rtol=5e-4, atol=1e-3)
        assert abs(float(left[s])) < 1e-3 * L * k_mean                    # the whole budget is handed out
        for l in range(L):
            b = want_b[l]
            if abs(b + 0.5 - round(b + 0.5)) > 1e-3:
                assert int(given[l, s]) == min(k_cap, max(1, math.floor(b + 0.5))), (l, s)
            e = min(int(given[l, s]), n)
            assert int(count[l, s]) == e and float(b_rep[l, s]) == float(e)
            res = {"idx": orc.select_blocks(el[l], range(nb_begin, nb_begin + n), e), "scores": el[l],
                   "nb_begin": nb_begin}
            got = idx[l, s].cpu().tolist()
            assert got[e:] == [-1] * (k_cap - e)
            if got[:e] != res["idx"]:             # only blocks that all but tie may swap
                sc = {b_: float(scores[l, s, b_]) for b_ in set(got[:e]) | set(res["idx"])}
                assert sorted(sc[b_] for b_ in got[:e]) == pytest.approx(sorted(sc[b_] for b_ in res["idx"]), abs=2e-5)


def test_pipeline_with_ragged_last_window_and_short_context():
    """The three-stream schedule on a context that is not a multiple of the window (the last
    window goes out as a call of its own) and on one shorter than a chunk."""
    for n_ctx in (512 * 5 + 77, 700):
        w = synth.scaled(synth.WORKLOADS["c3_128k"], n_ctx=n_ctx, k_cap=8, name=f"pipe_{n_ctx}")
        sh = w.shape
        q, k, v = synth.gen_layer(w, "cpu", 0)
        rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
        cutoffs = []
        for t in range(w.n_windows):
            b, e = H.eligible_range(sh, t * w.window)
            cutoffs.append(synth.cutoff_state(w, e - b, t, 0))
        qd, kc, vc = q.to(DEV), H.blocked_k(k.to(DEV), sh, w.n_blocks), H.blocked_vt(v.to(DEV), sh, w.n_blocks)
        repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=DEV)
        repd[: rep.shape[0]] = rep.to(DEV)
        runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, DEV)
        plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, DEV)
        bud0 = plan.budget.clone()
        pipe = H.PrefillPipeline(runner, plan)
        outs = []
        # the last schedule asks for a second team of attention workgroups: with 4 windows per call
        # there is no queue (a workgroup per item), so the second call of each pair does nothing
        for overlap, batched, late in ((False, False, 0), (True, False, 0), (True, True, 0), (True, True, 32)):
            runner.reset()
            plan.budget.copy_(bud0)
            out = torch.zeros_like(qd)
            pipe.run(qd, kc, vc, repd, out, overlap=overlap, chunk=4, score_chunk=4, batched=batched,
                     late_cus=late, attention_cus=224 if overlap else 256)
            torch.cuda.synchronize()
            outs.append((out, pipe.idx.clone(), pipe.n_sel.clone()))
        for other in outs[1:]:
            assert torch.equal(outs[0][1], other[1]) and torch.equal(outs[0][2], other[2])
            diff = (outs[0][0].float() - other[0].float()).abs().max().item()
            assert diff <= TOL_OUT["bf16"] * outs[0][0].float().abs().max().item()
        outs[1] = outs[2]
        want = oracle_windows(q, k, v, rep, sh, w.window, w.k_cap, cutoffs, [w.n_windows - 1])
        res = want[w.n_windows - 1]
        err = out_error(outs[1][0][res["w0"]:res["w0"] + res["out"].shape[0]], res["out"])
        assert err < TOL_OUT["bf16"], f"last window of {n_ctx}: {err}"


def test_mean_pooling_probe_variant():
    """The ablation baseline: every token of the window weighs 1/m, the statistics are still kept."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")
    cs = B.c_shape(sh)
    m, d = 512, 32 * 128
    g = torch.Generator().manual_seed(321)
    q = (torch.randn(2, m, 32, 128, generator=g) * 1.5 + 0.3).to(torch.bfloat16)
    qd = q.to(DEV)
    runs = {}
    for name, flags in (("probe", B.STATS_UPDATE), ("mean", B.STATS_UPDATE | B.PROBE_MEAN_POOLING)):
        r = H.LayerRunner(sh, 2, m, 8, 4, DEV)
        w = torch.zeros(2, m, device=DEV)
        B.build_probe(cs, 2, m, qd, r.stats, flags, r.probe, r.probe_kv, r.probe_norm, w, r.workspace)
        torch.cuda.synchronize()
        runs[name] = (r.probe.cpu(), r.probe_kv.cpu(), r.probe_norm.cpu(), w.cpu(), r.stats.cpu())
    assert torch.equal(runs["probe"][4], runs["mean"][4])            # same statistics either way
    for s in range(2):
        want, wts = orc.probe_query(f64(q[s]).reshape(m, d), np.ones((m, d)))
        assert np.allclose(wts, 1.0 / m)
        assert rel_to_max(runs["mean"][0][s], want) < TOL_PROBE
        assert np.allclose(runs["mean"][3][s].numpy(), 1.0 / m, rtol=1e-6)
        assert abs(float(runs["mean"][2][s]) - np.linalg.norm(want)) < TOL_PROBE * np.linalg.norm(want)
        kv = want.reshape(8, 4, 128).sum(axis=1).reshape(-1)
        assert rel_to_max(runs["mean"][1][s], kv) < TOL_PROBE
        assert rel_to_max(runs["probe"][0][s], want) > 10 * TOL_PROBE   # the activation-aware probe differs


@pytest.mark.parametrize("dtype,hq,hkv,d,m,calls", [
    ("bf16", 32, 8, 128, 512, (3, 5)),      # the benchmarked shape; a second call continues the first
    ("fp32", 6, 2, 64, 96, (1, 4)),         # fp32 storage, group size 3; a call of one window
    ("bf16", 8, 8, 128, 1100, (19,)),       # more than one pass of rows, more windows than a merge batch
])
def test_probe_of_consecutive_windows_in_one_call(dtype, hq, hkv, d, m, calls):
    """ACTQKV_PROBE_WINDOW_CHAIN: n consecutive windows of one sequence in one build_probe call
    give, window by window, the probe, weights and norm of Eq. (7)-(9) with the statistics of
    Eq. (8) over every query up to and including that window, and leave those of the last."""
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 512, dtype)
    cs = B.c_shape(sh)
    dd = hq * d
    n_total = sum(calls)
    _say(f"[case] probe chain {dtype} H{hq}/Hk{hkv}/D{d} m={m} calls={calls}")
    g = torch.Generator().manual_seed(99 + m)
    # a drifting mean and scale, so that the statistics of later windows differ from the first
    drift = torch.linspace(-0.5, 0.8, n_total).view(n_total, 1, 1, 1)
    q = torch.randn(n_total, m, hq, d, generator=g) * (1.0 + drift.abs()) + drift
    q[:, :, :, 5] *= 4.0                                  # a few loud channels
    q = q.to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    qd = q.to(DEV)
    n_max = max(calls)
    stats = torch.zeros(B.stats_floats(cs), device=DEV)
    ws = torch.zeros(B.workspace_bytes(cs, n_max, m, 8, 4), dtype=torch.uint8, device=DEV)
    probe = torch.zeros(n_total, dd, device=DEV)
    probe_kv = torch.zeros(n_total, hkv * d, device=DEV)
    norm = torch.zeros(n_total, device=DEV)
    wts = torch.zeros(n_total, m, device=DEV)
    t0 = 0
    for n in calls:
        B.build_probe(cs, n, m, qd[t0:t0 + n], stats, B.STATS_UPDATE | B.PROBE_WINDOW_CHAIN, probe[t0:t0 + n],
                      probe_kv[t0:t0 + n], norm[t0:t0 + n], wts[t0:t0 + n], ws)
        t0 += n
    torch.cuda.synchronize()
    rs = orc.RunningStats(dd)
    for t in range(n_total):
        qw = f64(q[t]).reshape(m, dd)
        z_bar, sigma2 = rs.update(qw)
        want, w_want = orc.probe_query(qw, orc.activation_bias(qw, z_bar, sigma2))
        assert rel_to_max(probe[t], want) < TOL_PROBE, f"probe, window {t}"
        assert rel_to_max(wts[t], w_want) < TOL_WEIGHT, f"weights, window {t}"
        assert abs(float(norm[t]) - np.linalg.norm(want)) < TOL_PROBE * np.linalg.norm(want)
        kv = want.reshape(hkv, hq // hkv, d).sum(axis=1).reshape(-1)
        assert rel_to_max(probe_kv[t], kv) < TOL_PROBE, f"probe_kv, window {t}"
    st = f64(stats)
    assert st[0] == n_total * m
    assert rel_to_max(st[4:4 + dd], rs.mean) < 1e-5
    assert rel_to_max(st[4 + dd:4 + 2 * dd], rs.m2) < 1e-4
    # the flag needs the update bit and a window of more than one token
    with pytest.raises(B.ActQKVError):
        B.build_probe(cs, 2, m, qd[:2], stats, B.PROBE_WINDOW_CHAIN, probe[:2], probe_kv[:2], norm[:2], None, ws)


def test_gather_blocks_from_pinned_host_memory():
    """actqkv_gather_blocks: the selected blocks of a store in pinned host memory land in the
    slots of the working cache, bit for bit; entries beyond n_sel and indices outside the store
    are skipped and reported as -1."""
    sh = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")
    cs = B.c_shape(sh)
    g = torch.Generator().manual_seed(77)
    nb_store, nb_work, k_cap, slot0 = 40, 16, 8, 2
    ks = torch.randn(2, nb_store, 8, 128, 128, generator=g).to(torch.bfloat16).pin_memory()
    vs = torch.randn(2, nb_store, 8, 128, 128, generator=g).to(torch.bfloat16).pin_memory()
    kw = torch.full((2, nb_work, 8, 128, 128), 7.0, dtype=torch.bfloat16, device=DEV)
    vw = torch.full((2, nb_work, 8, 128, 128), 7.0, dtype=torch.bfloat16, device=DEV)
    idx = torch.tensor([[5, 39, 0, 17, -1, 3, 3, 3], [12, 40, 11, 1, 2, 3, 4, 5]], dtype=torch.int32, device=DEV)
    n_sel = torch.tensor([4, 3], dtype=torch.int32, device=DEV)
    slots = torch.zeros(2, k_cap, dtype=torch.int32, device=DEV)
    B.gather_blocks(cs, 2, ks, vs, ks.stride(0), nb_store, idx, n_sel, k_cap, kw, vw, kw.stride(0), nb_work, slot0,
                    slots)
    torch.cuda.synchronize()
    want_slots = [[2, 3, 4, 5, -1, -1, -1, -1], [2, -1, 4, -1, -1, -1, -1, -1]]     # 40 is outside the store
    assert slots.cpu().tolist() == want_slots
    kw_c, vw_c = kw.cpu(), vw.cpu()
    for s in range(2):
        touched = set()
        for j, slot in enumerate(want_slots[s]):
            if slot >= 0:
                b = int(idx[s, j])
                assert torch.equal(kw_c[s, slot], ks[s, b]) and torch.equal(vw_c[s, slot], vs[s, b])
                touched.add(slot)
        for blk in range(nb_work):
            if blk not in touched:
                assert bool((kw_c[s, blk] == 7.0).all()) and bool((vw_c[s, blk] == 7.0).all())


def test_prefill_with_the_cache_in_host_memory():
    """The cache of the whole context in pinned host memory, a working cache of a few dozen
    blocks in HBM (HostCachePrefill): selections and attention outputs must equal those of the
    HBM-resident run, bit for bit (the same tiles go through the same kernel in the same order),
    and sampled windows are checked against the oracle."""
    w = synth.scaled(synth.WORKLOADS["c3_128k"], n_ctx=512 * 11 + 200, k_cap=8, name="host_cache")
    sh = w.shape
    _say(f"[case] {w.name} N={w.n_ctx} m={w.window} k_cap={w.k_cap}")
    q, k, v = synth.gen_layer(w, "cpu", 0)
    rep = synth.pick_rep_keys(k, sh.block_size, sh.n_rep)
    cutoffs = []
    for t in range(w.n_windows):
        b, e = H.eligible_range(sh, t * w.window)
        cutoffs.append(synth.cutoff_state(w, e - b, t, 0))
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    kc, vc = H.blocked_k(kd, sh, w.n_blocks), H.blocked_vt(vd, sh, w.n_blocks)
    repd = torch.zeros(w.n_blocks, sh.n_rep, sh.n_kv_heads, sh.head_dim, dtype=rep.dtype, device=DEV)
    repd[: rep.shape[0]] = rep.to(DEV)
    runner = H.LayerRunner(sh, 1, w.window, w.n_blocks, w.k_cap, DEV)
    plan = H.make_prefill_plan(sh, w.n_ctx, w.window, cutoffs, DEV)
    bud0 = plan.budget.clone()
    out_hbm = torch.zeros_like(qd)
    rec_hbm = H.prefill_layer(runner, plan, qd, kc, vc, repd, out_hbm, record=range(w.n_windows))
    torch.cuda.synchronize()
    k_store, v_store = kc.cpu().pin_memory(), vc.cpu().pin_memory()
    runner.reset()
    plan.budget.copy_(bud0)
    host = H.HostCachePrefill(runner, plan)
    assert host.nb_work < w.n_blocks // 2
    out_host = torch.zeros_like(qd)
    rec = host.run(qd, kd, vd, k_store, v_store, repd, out_host, record=range(w.n_windows))
    torch.cuda.synchronize()
    n_retrieving = 0
    for t in range(w.n_windows):
        assert torch.equal(rec[t]["idx"], rec_hbm[t]["idx"]) and int(rec[t]["n_sel"]) == int(rec_hbm[t]["n_sel"])
        n_retrieving += int(rec[t]["n_sel"]) > 0
    assert n_retrieving >= w.n_windows - 3
    assert torch.equal(out_host, out_hbm)
    # the overlapped schedule (selection chain ahead, data movement and attention on streams of
    # their own), with the host store EMPTY at the start: every block a window selects has been
    # written back from a working cache by then.  Twice in a row, eagerly (capturing this
    # four-stream schedule in a HIP graph ended in a host-side crash inside the runtime's
    # end-of-capture call; the schedule is not captured anywhere).
    k_zero, v_zero = torch.zeros_like(k_store).pin_memory(), torch.zeros_like(v_store).pin_memory()
    out_ov = torch.zeros_like(qd)

    def overlapped():
        runner.reset()
        plan.budget.copy_(bud0)
        return host.run_overlapped(qd, kd, vd, k_zero, v_zero, repd, out_ov)
    rec_ov = overlapped()
    torch.cuda.synchronize()
    for t in range(w.n_windows):
        assert torch.equal(rec_ov[t]["idx"], rec_hbm[t]["idx"]) and int(rec_ov[t]["n_sel"]) == int(rec_hbm[t]["n_sel"])
    assert torch.equal(out_ov, out_hbm)
    full = w.n_ctx // sh.block_size
    assert torch.equal(k_zero[:full], k_store[:full]) and torch.equal(v_zero[:full], v_store[:full])   # the store was rebuilt
    k_zero.zero_(); v_zero.zero_()
    out_ov.zero_()
    overlapped()
    torch.cuda.synchronize()
    assert torch.equal(out_ov, out_hbm)
    attend = [2, 7, w.n_windows - 1]
    want = oracle_windows(q, k, v, rep, sh, w.window, w.k_cap, cutoffs, attend)
    for t in attend:
        res = want[t]
        gi, gn = rec[t]["idx"].cpu().tolist(), int(rec[t]["n_sel"])
        ref = res["out"]
        if not check_selection(gi, gn, res, w.k_cap):
            ref = orc.retrieval_attention_window(f64(q[res["w0"]:res["w0"] + w.window]), f64(k), f64(v), res["w0"],
                                                 gi[:gn], sh.n_init, sh.n_local, sh.block_size, sh.group)
        err = out_error(out_host[res["w0"]:res["w0"] + ref.shape[0]], ref)
        assert err < TOL_OUT["bf16"], f"attention output, window {t}: {err}"


@pytest.mark.parametrize("dtype,hq,hkv,d,m,n_ctx", [("bf16", 32, 8, 128, 512, 512 * 7 + 130),
                                                   ("fp32", 8, 2, 64, 256, 256 * 9 + 40),
                                                   ("bf16", 32, 8, 128, 1, 2200)])
def test_retrieval_per_kv_head(dtype, hq, hkv, d, m, n_ctx):
    """The per-KV-head variant: actqkv_score_blocks_per_head, actqkv_select on batch * Hk rows
    (with a cut-off state per row) and actqkv_retrieval_attention_per_head against the oracle's
    retrieve_per_head / retrieval_attention_per_head, for a prefill window (matrix-core and
    row kernels) and a decode step."""
    sh = LayerShape(hq, hkv, d, 128, 4, 128, 256, dtype)
    cs = B.c_shape(sh)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(3 * d + m)
    k_cap, G = 6, hq // hkv
    _say(f"[case] per-KV-head retrieval {dtype} H{hq}/Hk{hkv}/D{d} m={m} N={n_ctx}")
    q_all = (torch.randn(n_ctx, hq, d, generator=g) * 1.2).to(td)
    k = torch.randn(n_ctx, hkv, d, generator=g).to(td)
    v = torch.randn(n_ctx, hkv, d, generator=g).to(td)
    nb = (n_ctx + 127) // 128
    # a few blocks every head likes, and one block only head 1 likes
    u = torch.randn(hkv, d, generator=g)
    for b in (3, 9):
        k[b * 128:(b + 1) * 128] = (k[b * 128:(b + 1) * 128].float() + 0.8 * u).to(td)
    k[5 * 128:6 * 128, 1] = (k[5 * 128:6 * 128, 1].float() + 1.5 * u[1]).to(td)
    w0 = n_ctx - m
    q = q_all[w0:].clone()
    q = (q.float() + 2.0 * u.repeat_interleave(G, dim=0)).to(td)
    rep = synth.pick_rep_keys(k, 128, 4)
    repd = torch.zeros(nb, 4, hkv, d, dtype=td, device=DEV)
    repd[: rep.shape[0]] = rep.to(DEV)
    kc, vc = H.blocked_k(k.to(DEV), sh, nb), H.blocked_vt(v.to(DEV), sh, nb)
    qd = q.to(DEV)
    runner = H.LayerRunner(sh, 1, m, nb, k_cap, DEV)
    B.build_probe(cs, 1, m, qd, runner.stats, True, runner.probe, runner.probe_kv, runner.probe_norm, None,
                  runner.workspace)
    nb_begin, nb_e = H.eligible_range(sh, w0)
    stride = runner.score_stride
    scores = torch.zeros(1, hkv, stride, device=DEV)
    nb_end = torch.full((1, hkv), nb_e, dtype=torch.int32, device=DEV)
    B.score_blocks_per_head(cs, 1, runner.probe, repd, 0, nb_e, nb_begin, nb_end, scores, stride)
    cut = [(2.0 * k_cap + 0.37 * hk, 1.5 * math.log(max(nb_e - nb_begin, 2))) for hk in range(hkv)]
    bud = torch.tensor([c[0] for c in cut], dtype=torch.float32, device=DEV)
    rest = torch.tensor([c[1] for c in cut], dtype=torch.float32, device=DEV)
    idx = torch.zeros(hkv, k_cap, dtype=torch.int32, device=DEV)
    n_sel = torch.zeros(hkv, dtype=torch.int32, device=DEV)
    theta = torch.zeros(hkv, device=DEV)
    budget = torch.zeros(hkv, device=DEV)
    B.select(hkv, scores.view(hkv, stride), stride, nb_e, nb_begin, nb_end.view(hkv), k_cap, bud, rest, idx, n_sel,
             theta, budget)
    out = torch.zeros_like(qd)
    n_ctx_d = torch.tensor([n_ctx], dtype=torch.int32, device=DEV)
    B.retrieval_attention(cs, 1, m, qd, kc, vc, 0, nb, n_ctx_d, idx, n_sel, k_cap, out, None, runner.workspace,
                          per_head=True)
    torch.cuda.synchronize()
    probe64 = f64(runner.probe[0])                      # the GPU's probe (its own parity is tested elsewhere)
    want = orc.retrieve_per_head(probe64, f64(rep), w0, sh.n_init, sh.n_local, 128, G, k_cap, cut)
    sel = []
    for hk in range(hkv):
        res = want[hk]
        gs = f64(scores[0, hk])[res["eligible"]]
        assert np.abs(gs - res["scores"]).max() < TOL_SCORE, f"scores, head {hk}"
        assert abs(float(theta[hk]) - res["theta"]) < TOL_THETA
        gi, gn = idx[hk].cpu().tolist(), int(n_sel[hk])
        check_selection(gi, gn, res, k_cap)
        sel.append(gi[:gn])
    assert len({tuple(x) for x in sel}) > 1, "the heads should not all select the same blocks here"
    ref = orc.retrieval_attention_per_head(f64(q), f64(k), f64(v), w0, sel, sh.n_init, sh.n_local, 128, G)
    err = out_error(out, ref)
    assert err < TOL_OUT[dtype], f"attention output: {err}"
    # the same selection for every head through the per-head call = the shared call
    idx_same = idx[0:1].repeat(hkv, 1).contiguous()
    n_same = n_sel[0:1].repeat(hkv).contiguous()
    out_a, out_b = torch.zeros_like(qd), torch.zeros_like(qd)
    B.retrieval_attention(cs, 1, m, qd, kc, vc, 0, nb, n_ctx_d, idx_same, n_same, k_cap, out_a, None,
                          runner.workspace, per_head=True)
    B.retrieval_attention(cs, 1, m, qd, kc, vc, 0, nb, n_ctx_d, idx[0:1], n_sel[0:1], k_cap, out_b, None,
                          runner.workspace)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b)
