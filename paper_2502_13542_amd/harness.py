"""Host-side driver around the library: cache layout conversion, window
bookkeeping and the window-by-window / step-by-step loops of Sec. 3.1.  It only
allocates, converts layouts and calls the four entry points in order; every
arithmetic step of the path runs inside libactqkv.so.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B
from .synth import LayerShape


# ---------------------------------------------------------------- geometry
def local_start(shape: LayerShape, w0: int) -> int:
    """First token of the local span of a window that starts at w0 (same rule as the kernels)."""
    i0 = min(shape.n_init, w0)
    a = w0 - shape.n_local
    a = (a // shape.block_size) * shape.block_size if a > 0 else 0
    return max(i0, a)


def eligible_range(shape: LayerShape, w0: int) -> Tuple[int, int]:
    """[nb_begin, nb_end): blocks wholly between the initial tokens and the local span."""
    nb_begin = shape.n_init // shape.block_size
    return nb_begin, max(nb_begin, local_start(shape, w0) // shape.block_size)


# ---------------------------------------------------------------- layouts
def blocked_k(k: torch.Tensor, shape: LayerShape, nb_capacity: Optional[int] = None) -> torch.Tensor:
    """[N][Hk][D] -> k_cache [nb][Hk][Bs][D], zero-padded to whole blocks."""
    n, hk, d = k.shape
    bs = shape.block_size
    nb = (n + bs - 1) // bs if nb_capacity is None else nb_capacity
    out = torch.zeros(nb, hk, bs, d, dtype=k.dtype, device=k.device)
    full = n // bs
    out[:full] = k[: full * bs].reshape(full, bs, hk, d).permute(0, 2, 1, 3)
    if n > full * bs:
        out[full, :, : n - full * bs] = k[full * bs:].permute(1, 0, 2)
    return out


def blocked_vt(v: torch.Tensor, shape: LayerShape, nb_capacity: Optional[int] = None) -> torch.Tensor:
    """[N][Hk][D] -> v_cache [nb][Hk][D][Bs] (values transposed inside a block), zero-padded."""
    n, hk, d = v.shape
    bs = shape.block_size
    nb = (n + bs - 1) // bs if nb_capacity is None else nb_capacity
    out = torch.zeros(nb, hk, d, bs, dtype=v.dtype, device=v.device)
    full = n // bs
    out[:full] = v[: full * bs].reshape(full, bs, hk, d).permute(0, 2, 3, 1)
    if n > full * bs:
        out[full, :, :, : n - full * bs] = v[full * bs:].permute(1, 2, 0)
    return out


# ---------------------------------------------------------------- one layer of one (batch of) sequence(s)
class LayerRunner:
    """Device buffers of one layer and the call sequence of one window / step."""

    def __init__(self, shape: LayerShape, batch: int, m: int, nb_capacity: int, k_cap: int,
                 device="cuda"):
        self.shape, self.batch, self.m, self.nb_capacity, self.k_cap = shape, batch, m, nb_capacity, k_cap
        self.cs = B.c_shape(shape)
        self.device = device
        d, dk = shape.d_model, shape.n_kv_heads * shape.head_dim
        f32 = dict(dtype=torch.float32, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        self.stats = torch.zeros(batch, B.stats_floats(self.cs), **f32)
        self.probe = torch.empty(batch, d, **f32)
        self.probe_kv = torch.empty(batch, dk, **f32)
        self.probe_norm = torch.empty(batch, **f32)
        self.weights = torch.empty(batch, m, **f32)
        self.score_stride = (nb_capacity + 3) // 4 * 4
        self.scores = torch.zeros(batch, self.score_stride, **f32)
        self.idx = torch.full((batch, k_cap), -1, **i32)
        self.n_sel = torch.zeros(batch, **i32)
        self.theta = torch.zeros(batch, **f32)
        self.budget = torch.zeros(batch, **f32)
        ws = B.workspace_bytes(self.cs, batch, m, nb_capacity, k_cap)
        self.workspace = torch.zeros(ws, dtype=torch.uint8, device=device)

    def reset(self) -> None:
        self.stats.zero_()

    def step(self, q_win: torch.Tensor, k_cache, v_cache, rep_keys, n_ctx: torch.Tensor,
             nb_end: torch.Tensor, nb_end_max: int, out: torch.Tensor,
             budget_remaining: Optional[torch.Tensor] = None,
             theta_rest_sum: Optional[torch.Tensor] = None, update_stats: bool = True,
             m: Optional[int] = None, lse=None, stream=None) -> None:
        """probe -> scores -> selection -> attention for one window (or decode step).
        nb_end_max: host-side upper bound of nb_end, sizes the scoring launch.
        budget_remaining / theta_rest_sum: [batch] fp32 cut-off state, or None."""
        sh, cs, bt = self.shape, self.cs, self.batch
        m = self.m if m is None else m
        nb_begin = sh.n_init // sh.block_size
        cache_stride = k_cache.stride(0) if k_cache.dim() == 5 else 0
        rep_stride = rep_keys.stride(0) if rep_keys.dim() == 5 else 0
        B.build_probe(cs, bt, m, q_win, self.stats, update_stats, self.probe, self.probe_kv,
                      self.probe_norm, self.weights, self.workspace, stream)
        nb_cap = min(max(nb_end_max, nb_begin), self.nb_capacity)
        B.score_blocks(cs, bt, self.probe_kv, self.probe_norm, rep_keys, rep_stride, nb_cap, nb_begin,
                       nb_end, self.scores, self.score_stride, stream)
        B.select(bt, self.scores, self.score_stride, nb_cap, nb_begin, nb_end, self.k_cap, budget_remaining,
                 theta_rest_sum, self.idx, self.n_sel, self.theta, self.budget, stream)
        B.retrieval_attention(cs, bt, m, q_win, k_cache, v_cache, cache_stride, self.nb_capacity, n_ctx,
                              self.idx, self.n_sel, self.k_cap, out, lse, self.workspace, stream)

    def decode_step(self, q_tok: torch.Tensor, k_cache, v_cache, rep_keys, n_ctx: torch.Tensor,
                    nb_end: torch.Tensor, nb_end_max: int, out: torch.Tensor,
                    budget_remaining: Optional[torch.Tensor] = None,
                    theta_rest_sum: Optional[torch.Tensor] = None, k_new=None, v_new=None, pos0=None,
                    lse=None, stream=None) -> None:
        """A decode step in two calls (three launches): (cache update,) probe, scores and selection
        (actqkv_decode_retrieve), then the attention.  k_new, v_new, pos0: the new
        token's key, value and position per sequence, or None if the cache already holds it."""
        sh, cs, bt = self.shape, self.cs, self.batch
        nb_begin = sh.n_init // sh.block_size
        cache_stride = k_cache.stride(0) if k_cache.dim() == 5 else 0
        rep_stride = rep_keys.stride(0) if rep_keys.dim() == 5 else 0
        nb_cap = min(max(nb_end_max, nb_begin, 1), self.nb_capacity)
        B.decode_retrieve(cs, bt, q_tok, k_new, v_new, pos0, k_cache, v_cache, cache_stride, rep_keys,
                          rep_stride, nb_cap if k_new is None else self.nb_capacity, nb_begin, nb_end,
                          self.probe, self.probe_kv, self.probe_norm, self.scores, self.score_stride,
                          self.k_cap, budget_remaining, theta_rest_sum, self.idx, self.n_sel, self.theta,
                          self.budget, stream)
        B.retrieval_attention(cs, bt, 1, q_tok, k_cache, v_cache, cache_stride, self.nb_capacity, n_ctx,
                              self.idx, self.n_sel, self.k_cap, out, lse, self.workspace, stream)

    def decode_step_two_launches(self, q_tok: torch.Tensor, k_cache, v_cache, rep_keys, n_ctx: torch.Tensor,
                                 nb_end: torch.Tensor, out: torch.Tensor,
                                 budget_in: Optional[torch.Tensor] = None,
                                 theta_rest_sum: Optional[torch.Tensor] = None,
                                 budget_after: Optional[torch.Tensor] = None, k_new=None, v_new=None,
                                 pos0=None, lse=None, stream=None) -> None:
        """A decode step in two launches: (cache update,) probe and scores in the first
        (actqkv_decode_retrieve, scores only), selection and attention in the second
        (actqkv_decode_select_attention).  bf16, head_dim 128 only."""
        sh, cs, bt = self.shape, self.cs, self.batch
        nb_begin = sh.n_init // sh.block_size
        cache_stride = k_cache.stride(0) if k_cache.dim() == 5 else 0
        rep_stride = rep_keys.stride(0) if rep_keys.dim() == 5 else 0
        B.decode_retrieve(cs, bt, q_tok, k_new, v_new, pos0, k_cache, v_cache, cache_stride, rep_keys,
                          rep_stride, self.nb_capacity, nb_begin, nb_end, self.probe, self.probe_kv,
                          self.probe_norm, self.scores, self.score_stride, self.k_cap, None, None, None,
                          None, None, None, stream, flags=B.DECODE_SCORES_ONLY)
        B.decode_select_attention(cs, bt, q_tok, k_cache, v_cache, cache_stride, self.nb_capacity, n_ctx,
                                  self.scores, self.score_stride, nb_begin, nb_end, self.k_cap, budget_in,
                                  theta_rest_sum, budget_after, self.idx, self.n_sel, self.theta,
                                  self.budget, out, lse, self.workspace, stream)


    def decode_step_one_launch(self, q_tok: torch.Tensor, k_cache, v_cache, rep_keys, n_ctx: torch.Tensor,
                               nb_end: torch.Tensor, out: torch.Tensor,
                               budget_in: Optional[torch.Tensor] = None,
                               theta_rest_sum: Optional[torch.Tensor] = None,
                               budget_after: Optional[torch.Tensor] = None, k_new=None, v_new=None,
                               lse=None, stream=None, flags: int = 0) -> None:
        """A decode step in one launch (actqkv_decode_layer): the token is written at position
        n_ctx - 1.  bf16, head_dim 128 only."""
        sh, cs, bt = self.shape, self.cs, self.batch
        nb_begin = sh.n_init // sh.block_size
        cache_stride = k_cache.stride(0) if k_cache.dim() == 5 else 0
        rep_stride = rep_keys.stride(0) if rep_keys.dim() == 5 else 0
        B.decode_layer(cs, bt, q_tok, k_new, v_new, k_cache, v_cache, cache_stride, rep_keys, rep_stride,
                       self.nb_capacity, n_ctx, nb_begin, nb_end, self.scores, self.score_stride, self.k_cap,
                       budget_in, theta_rest_sum, budget_after, self.idx, self.n_sel, self.theta, self.budget,
                       out, lse, self.workspace, stream, flags)


@dataclass
class PrefillPlan:
    """Per-window device scalars of a single-sequence prefill, uploaded once."""
    n_windows: int
    w0: List[int]
    rows: List[int]
    nb_end_host: List[int]
    n_ctx: torch.Tensor      # int32 [T]
    nb_end: torch.Tensor     # int32 [T]
    budget: Optional[torch.Tensor]   # float32 [T]: B_kv handed to each window, or None
    rest: Optional[torch.Tensor]     # float32 [T]: R of each window, or None


def make_prefill_plan(shape: LayerShape, n_ctx: int, m: int,
                      cutoffs: Optional[Sequence[Tuple[float, float]]], device="cuda") -> PrefillPlan:
    w0s = list(range(0, n_ctx, m))
    rows = [min(m, n_ctx - w) for w in w0s]
    nb_end = [eligible_range(shape, w)[1] for w in w0s]
    nctx = [w + r for w, r in zip(w0s, rows)]
    budget = rest = None
    if cutoffs is not None:
        budget = torch.tensor([c[0] for c in cutoffs], dtype=torch.float32, device=device)
        rest = torch.tensor([c[1] for c in cutoffs], dtype=torch.float32, device=device)
    return PrefillPlan(len(w0s), w0s, rows, nb_end,
                       torch.tensor(nctx, dtype=torch.int32, device=device),
                       torch.tensor(nb_end, dtype=torch.int32, device=device), budget, rest)


def prefill_layer(runner: LayerRunner, plan: PrefillPlan, q: torch.Tensor, k_cache, v_cache, rep_keys,
                  out: torch.Tensor, record: Optional[Sequence[int]] = None,
                  windows: Optional[Sequence[int]] = None) -> Dict[int, Dict[str, torch.Tensor]]:
    """Runs the windows of one sequence in order.  q, out [N][H][D].  `record` lists the
    windows whose intermediate results are copied out (for parity checks)."""
    rec: Dict[int, Dict[str, torch.Tensor]] = {}
    m = runner.m
    for t in (range(plan.n_windows) if windows is None else windows):
        w0, rows = plan.w0[t], plan.rows[t]
        bud = None if plan.budget is None else plan.budget[t:t + 1]
        rest = None if plan.rest is None else plan.rest[t:t + 1]
        runner.step(q[w0:w0 + rows], k_cache, v_cache, rep_keys, plan.n_ctx[t:t + 1],
                    plan.nb_end[t:t + 1], plan.nb_end_host[t], out[w0:w0 + rows], bud, rest, True, rows)
        if record is not None and t in record:
            rec[t] = dict(probe=runner.probe[0].clone(), probe_kv=runner.probe_kv[0].clone(),
                          probe_norm=runner.probe_norm[0].clone(),
                          weights=runner.weights[0, :rows].clone(), scores=runner.scores[0].clone(),
                          idx=runner.idx[0].clone(), n_sel=runner.n_sel[0].clone(),
                          theta=runner.theta[0].clone(), budget=runner.budget[0].clone(),
                          budget_after=None if bud is None else bud[0].clone())
    return rec


class PrefillPipeline:
    """The windows of one layer as two dependency chains.  The probe / score / select chain
    of a window depends on the windows before it (running statistics of Eq. (8), the budget of
    Eq. (12)); the attention of a window depends only on that window's own selection.  With
    overlap=True the attention calls go to a second stream, so the chain of later windows runs
    beside the attention of earlier ones; every window keeps its own selection, and the two
    streams use separate workspaces.  The results are those of window order."""

    MAX_CHUNK = 32

    def __init__(self, runner: LayerRunner, plan: PrefillPlan):
        self.runner, self.plan = runner, plan
        dev = runner.device
        self.idx = torch.full((plan.n_windows, runner.k_cap), -1, dtype=torch.int32, device=dev)
        self.n_sel = torch.zeros(plan.n_windows, dtype=torch.int32, device=dev)
        # one workspace for the attention stream: calls of up to MAX_CHUNK windows, and of a single
        # (ragged) window, whose key tiles are cut into pieces and need room for the partials
        ws = max(B.workspace_bytes(runner.cs, n, runner.m, runner.nb_capacity, runner.k_cap)
                 for n in (1, 2, self.MAX_CHUNK))
        self.ws_attn = torch.zeros(ws, dtype=torch.uint8, device=dev)
        self.ws_attn_b = torch.zeros(ws, dtype=torch.uint8, device=dev)   # two teams: chunks alternate workspaces
        self.side = torch.cuda.Stream(device=dev)
        # the probe of every window, for the schedule that scores behind the probe chain
        dk = runner.shape.n_kv_heads * runner.shape.head_dim
        self.probe_kv = torch.empty(plan.n_windows, dk, dtype=torch.float32, device=dev)
        self.probe_norm = torch.empty(plan.n_windows, dtype=torch.float32, device=dev)
        self.side_score = torch.cuda.Stream(device=dev)
        # the chunk-at-a-time schedule: probes and scores of up to MAX_CHUNK windows per call
        self.probe_chunk = torch.empty(self.MAX_CHUNK, runner.shape.n_q_heads * runner.shape.head_dim,
                                       dtype=torch.float32, device=dev)
        self.scores_chunk = torch.zeros(self.MAX_CHUNK, runner.score_stride, dtype=torch.float32, device=dev)
        self.ws_probe = torch.zeros(B.workspace_bytes(runner.cs, self.MAX_CHUNK, runner.m, runner.nb_capacity,
                                                      runner.k_cap), dtype=torch.uint8, device=dev)

    def _attention(self, call, stream, late_cus: int = 0, stream_late=None) -> None:
        """call: the arguments of actqkv_retrieval_attention up to the workspace."""
        if self.attention_cus >= 256 and late_cus == 0:
            B.retrieval_attention(*call, stream)
        else:
            B.retrieval_attention_teams(*call, self.attention_cus, late_cus, stream, stream_late)

    def run(self, q: torch.Tensor, k_cache, v_cache, rep_keys, out: torch.Tensor, overlap: bool = True,
            events=None, chunk: int = 32, score_chunk: int = 16, batched: bool = False,
            late_cus: int = 0, attention_cus: int = 256, prelude_events=None) -> None:
        """q, out [N][H][D].  events: optional per-window (start, end) event pairs recorded around
        the attention call of a window; with overlap, the pair of a chunk's first window brackets
        the chunk's one call, on the stream it runs on.  chunk: with overlap, the second stream picks up
        the attention of `chunk` windows at a time, once the last of them has its selection:
        one dependency between the streams per chunk, and ONE attention call for the chunk (the
        windows are batch entries that share the cache; with that many query tiles in a launch
        the key tiles need not be cut into pieces, so nothing has to be merged).  score_chunk > 0
        (with overlap) also moves scoring and selection to a stream of their own, that many
        windows behind the probes (see _run_three_streams); 0 keeps them on the current stream.
        attention_cus: compute units the attention calls on the second stream may fill (the rest
        serves the other chain); late_cus > 0 (batched only): see _run_batched.
        prelude_events (batched only): per-window (start, end) event pairs; the pair of a chunk's
        first window brackets the chunk's probe, score and select calls on the current stream."""
        r, plan = self.runner, self.plan
        sh, cs = r.shape, r.cs
        nb_begin = sh.n_init // sh.block_size
        cur = torch.cuda.current_stream()
        chunk = max(1, min(chunk, self.MAX_CHUNK))
        self.attention_cus = attention_cus if overlap else 256
        if overlap and batched:
            return self._run_batched(q, k_cache, v_cache, rep_keys, out, events, chunk, late_cus, prelude_events)
        if overlap and score_chunk > 0:
            return self._run_three_streams(q, k_cache, v_cache, rep_keys, out, events, chunk, score_chunk)

        def attend(t, stream):
            w0, rows = plan.w0[t], plan.rows[t]
            self._attention((cs, 1, rows, q[w0:w0 + rows], k_cache, v_cache, 0, r.nb_capacity,
                             plan.n_ctx[t:t + 1], self.idx[t], self.n_sel[t:t + 1], r.k_cap,
                             out[w0:w0 + rows], None, self.ws_attn), stream)

        if overlap:
            self.side.wait_stream(cur)
        pending = []
        self.chunk_starts = []          # first window of every attention call of this run
        for t in range(plan.n_windows):
            w0, rows = plan.w0[t], plan.rows[t]
            qw = q[w0:w0 + rows]
            bud = None if plan.budget is None else plan.budget[t:t + 1]
            rest = None if plan.rest is None else plan.rest[t:t + 1]
            nb_cap = min(max(plan.nb_end_host[t], nb_begin), r.nb_capacity)
            B.build_probe(cs, 1, rows, qw, r.stats, True, r.probe, r.probe_kv, r.probe_norm, None,
                          r.workspace)
            B.score_blocks(cs, 1, r.probe_kv, r.probe_norm, rep_keys, 0, nb_cap, nb_begin,
                           plan.nb_end[t:t + 1], r.scores, r.score_stride)
            B.select(1, r.scores, r.score_stride, nb_cap, nb_begin, plan.nb_end[t:t + 1], r.k_cap, bud,
                     rest, self.idx[t], self.n_sel[t:t + 1], None, None)
            if not overlap:
                self.chunk_starts.append(t)
                if events is not None:
                    events[t][0].record()
                attend(t, None)
                if events is not None:
                    events[t][1].record()
                continue
            pending.append(t)
            if len(pending) == chunk or t == plan.n_windows - 1:
                done = torch.cuda.Event()
                done.record(cur)
                self.side.wait_event(done)
                t0, n_p = pending[0], len(pending)
                self.chunk_starts.append(t0)
                if events is not None:
                    events[t0][0].record(self.side)
                if n_p > 1 and all(plan.rows[u] == r.m for u in pending):
                    w0 = plan.w0[t0]
                    self._attention((cs, n_p, r.m, q[w0:w0 + n_p * r.m], k_cache, v_cache, 0,
                                     r.nb_capacity, plan.n_ctx[t0:t0 + n_p], self.idx[t0:t0 + n_p],
                                     self.n_sel[t0:t0 + n_p], r.k_cap, out[w0:w0 + n_p * r.m], None,
                                     self.ws_attn), self.side)
                else:
                    for u in pending:
                        attend(u, self.side)
                if events is not None:
                    events[t0][1].record(self.side)
                pending = []
        if overlap:
            cur.wait_stream(self.side)

    def _run_batched(self, q, k_cache, v_cache, rep_keys, out, events, chunk, late_cus=0,
                     prelude_events=None) -> None:
        """A chunk of windows per call, for every step of the path.  The running statistics of
        Eq. (8) are the only thing a window hands to the next one within a layer, and merging a
        window into them needs nothing but that window's own moments; scores, density, budget
        and selection of a window depend on its probe alone.  So `chunk` consecutive full
        windows go through one build_probe call (ACTQKV_PROBE_WINDOW_CHAIN), one score_blocks
        and one select call on the current stream, and one attention call on the second stream,
        which works on chunk c while the current stream prepares chunk c + 1.  A ragged last
        window goes through calls of its own.

        late_cus > 0: the attention leaves compute units to the current stream (attention_cus of
        256 are its own), but the current stream needs them only while it prepares the next
        chunk; so the attention call of a chunk (actqkv_retrieval_attention_teams) is made once
        the NEXT chunk's preparation has been enqueued: its first team goes to the second
        stream, which has been waiting for nothing but this chunk's selection, and its second
        team of late_cus workgroups to the current stream, behind that preparation, where it
        takes its share of what is left in the chunk's queue.
        Chunks alternate between two workspaces, so a chunk's queue is never touched by the
        next chunk's launches."""
        r, plan = self.runner, self.plan
        sh, cs = r.shape, r.cs
        nb_begin = sh.n_init // sh.block_size
        cur, last = torch.cuda.current_stream(), self.side
        last.wait_stream(cur)
        self.chunk_starts = []

        def single(u):
            w0, rows = plan.w0[u], plan.rows[u]
            bud = None if plan.budget is None else plan.budget[u:u + 1]
            rest = None if plan.rest is None else plan.rest[u:u + 1]
            nb_cap = min(max(plan.nb_end_host[u], nb_begin), r.nb_capacity)
            B.build_probe(cs, 1, rows, q[w0:w0 + rows], r.stats, True, r.probe, self.probe_kv[u],
                          self.probe_norm[u:u + 1], None, r.workspace)
            B.score_blocks(cs, 1, self.probe_kv[u], self.probe_norm[u:u + 1], rep_keys, 0, nb_cap,
                           nb_begin, plan.nb_end[u:u + 1], r.scores, r.score_stride)
            B.select(1, r.scores, r.score_stride, nb_cap, nb_begin, plan.nb_end[u:u + 1], r.k_cap, bud,
                     rest, self.idx[u], self.n_sel[u:u + 1], None, None)

        def attend(pending):
            t_first, call = pending
            if events is not None:
                events[t_first][0].record(last)
            self._attention(call, last, late_cus, cur)
            if events is not None:
                events[t_first][1].record(last)

        t0, n_chunks, pending = 0, 0, None
        while t0 < plan.n_windows:
            n_p = 0
            while t0 + n_p < plan.n_windows and n_p < chunk and plan.rows[t0 + n_p] == r.m:
                n_p += 1
            if prelude_events is not None:
                prelude_events[t0][0].record(cur)
            if n_p >= 2:
                w0, t1 = plan.w0[t0], t0 + n_p
                B.build_probe(cs, n_p, r.m, q[w0:w0 + n_p * r.m], r.stats,
                              B.STATS_UPDATE | B.PROBE_WINDOW_CHAIN, self.probe_chunk, self.probe_kv[t0:t1],
                              self.probe_norm[t0:t1], None, self.ws_probe)
                nb_cap = min(max(plan.nb_end_host[t1 - 1], nb_begin), r.nb_capacity)
                B.score_blocks(cs, n_p, self.probe_kv[t0:t1], self.probe_norm[t0:t1], rep_keys, 0, nb_cap,
                               nb_begin, plan.nb_end[t0:t1], self.scores_chunk, r.score_stride)
                B.select(n_p, self.scores_chunk, r.score_stride, nb_cap, nb_begin, plan.nb_end[t0:t1],
                         r.k_cap, None if plan.budget is None else plan.budget[t0:t1],
                         None if plan.rest is None else plan.rest[t0:t1], self.idx[t0:t1],
                         self.n_sel[t0:t1], None, None)
            else:
                n_p = 1
                single(t0)
            if prelude_events is not None:
                prelude_events[t0][1].record(cur)
            selected = torch.cuda.Event()
            selected.record(cur)
            if pending is not None:
                attend(pending)          # the chunk before this one; its second team follows this preparation
            last.wait_event(selected)
            self.chunk_starts.append(t0)
            w0, rows = plan.w0[t0], plan.rows[t0]
            call = (cs, n_p, rows, q[w0:w0 + n_p * rows], k_cache, v_cache, 0, r.nb_capacity,
                    plan.n_ctx[t0:t0 + n_p], self.idx[t0:t0 + n_p], self.n_sel[t0:t0 + n_p],
                    r.k_cap, out[w0:w0 + n_p * rows], None)
            call += (self.ws_attn if n_chunks % 2 == 0 else self.ws_attn_b,)
            pending = (t0, call)
            n_chunks += 1
            t0 += n_p
        if pending is not None:
            attend(pending)
        cur.wait_stream(last)

    def _run_three_streams(self, q, k_cache, v_cache, rep_keys, out, events, chunk, score_chunk) -> None:
        """The selection chain cut in two as well.  The probe of a window (statistics, bias,
        weights) depends only on the statistics of the window before; scoring and selection
        depend on the window's probe and on the budget the window before left.  So the probes run
        ahead on the current stream, scoring and selection follow on a second stream
        `score_chunk` windows at a time, and the attention on a third, `chunk` windows at a time."""
        r, plan = self.runner, self.plan
        sh, cs = r.shape, r.cs
        nb_begin = sh.n_init // sh.block_size
        cur, mid, last = torch.cuda.current_stream(), self.side_score, self.side
        mid.wait_stream(cur)
        last.wait_stream(cur)
        self.chunk_starts = []
        to_score, to_attend = [], []
        for t in range(plan.n_windows):
            w0, rows = plan.w0[t], plan.rows[t]
            B.build_probe(cs, 1, rows, q[w0:w0 + rows], r.stats, True, r.probe, self.probe_kv[t],
                          self.probe_norm[t:t + 1], None, r.workspace)
            to_score.append(t)
            final = t == plan.n_windows - 1
            if len(to_score) < score_chunk and not final:
                continue
            probed = torch.cuda.Event()
            probed.record(cur)
            mid.wait_event(probed)
            for u in to_score:
                bud = None if plan.budget is None else plan.budget[u:u + 1]
                rest = None if plan.rest is None else plan.rest[u:u + 1]
                nb_cap = min(max(plan.nb_end_host[u], nb_begin), r.nb_capacity)
                B.score_blocks(cs, 1, self.probe_kv[u], self.probe_norm[u:u + 1], rep_keys, 0, nb_cap,
                               nb_begin, plan.nb_end[u:u + 1], r.scores, r.score_stride, mid)
                B.select(1, r.scores, r.score_stride, nb_cap, nb_begin, plan.nb_end[u:u + 1], r.k_cap, bud,
                         rest, self.idx[u], self.n_sel[u:u + 1], None, None, mid)
            to_attend += to_score
            to_score = []
            if len(to_attend) < chunk and not final:
                continue
            selected = torch.cuda.Event()
            selected.record(mid)
            last.wait_event(selected)
            for a0 in range(0, len(to_attend), chunk):
                piece = to_attend[a0:a0 + chunk]
                t0, n_p = piece[0], len(piece)
                self.chunk_starts.append(t0)
                if events is not None:
                    events[t0][0].record(last)
                if n_p > 1 and all(plan.rows[u] == r.m for u in piece):
                    w0 = plan.w0[t0]
                    self._attention((cs, n_p, r.m, q[w0:w0 + n_p * r.m], k_cache, v_cache, 0,
                                     r.nb_capacity, plan.n_ctx[t0:t0 + n_p], self.idx[t0:t0 + n_p],
                                     self.n_sel[t0:t0 + n_p], r.k_cap, out[w0:w0 + n_p * r.m], None,
                                     self.ws_attn), last)
                else:
                    for u in piece:
                        w0, rows = plan.w0[u], plan.rows[u]
                        self._attention((cs, 1, rows, q[w0:w0 + rows], k_cache, v_cache, 0,
                                         r.nb_capacity, plan.n_ctx[u:u + 1], self.idx[u],
                                         self.n_sel[u:u + 1], r.k_cap, out[w0:w0 + rows], None,
                                         self.ws_attn), last)
                if events is not None:
                    events[t0][1].record(last)
            to_attend = []
        cur.wait_stream(mid)
        cur.wait_stream(last)


class HostCachePrefill:
    """Single-sequence prefill of one layer with the key-value cache in pinned host memory
    (Sec. 3.1: the cache may be kept in CPU memory).  HBM holds the representative keys of all
    blocks (scoring never touches the cache) and a working cache of n_init/Bs + k_cap +
    (n_local + m)/Bs + 1 blocks: the initial tokens, k_cap slots that `actqkv_gather_blocks`
    fills from the host store with the blocks a window selects, then the local span and the
    window itself.  The attention runs on the working cache as on any cache: the local span and
    the window sit at positions shifted by a multiple of the block size (only the order of the
    positions matters to the kernel), the selection it is given are the slot numbers.

    Per window: the window's keys and values (token-major, as a model hands them over) are
    appended behind the local span (`actqkv_append_kv`); the local span moves with the window,
    so two working caches alternate and the span's blocks are carried over with
    `actqkv_copy_bytes`.  While the context is still shorter than n_init + n_local the working
    cache simply holds it whole at its true positions.  Needs m, n_init, n_local multiples of
    the block size (only the last window may be ragged)."""

    GROUP = 4                 # windows per hand-over between the streams of the overlapped schedule
    N_WORK = 2 * GROUP + 1    # working caches: a group being attended to, a group being filled, one source

    def __init__(self, runner: LayerRunner, plan: PrefillPlan):
        sh = runner.shape
        bs = sh.block_size
        assert runner.batch == 1 and runner.m % bs == 0 and sh.n_init % bs == 0 and sh.n_local % bs == 0
        self.runner, self.plan = runner, plan
        dev = runner.device
        self.slot0 = sh.n_init // bs
        self.tail0 = self.slot0 + runner.k_cap
        self.nb_work = self.tail0 + (sh.n_local + runner.m) // bs + 1
        st = torch.float32 if sh.dtype == "fp32" else torch.bfloat16
        shape_k = (self.nb_work, sh.n_kv_heads, bs, sh.head_dim)
        shape_v = (self.nb_work, sh.n_kv_heads, sh.head_dim, bs)
        self.k_work = [torch.zeros(shape_k, dtype=st, device=dev) for _ in range(self.N_WORK)]
        self.v_work = [torch.zeros(shape_v, dtype=st, device=dev) for _ in range(self.N_WORK)]
        self.idx_slots = torch.full((1, runner.k_cap), -1, dtype=torch.int32, device=dev)
        self.n_ctx_work = torch.zeros(1, dtype=torch.int32, device=dev)
        self.pos0_work = torch.zeros(1, dtype=torch.int32, device=dev)
        self.workspace = torch.zeros(B.workspace_bytes(runner.cs, 1, runner.m, self.nb_work, runner.k_cap),
                                     dtype=torch.uint8, device=dev)
        self.gathered_blocks = 0
        self.block_bytes = sh.n_kv_heads * bs * sh.head_dim * self.k_work[0].element_size()   # K or V of a block
        # the overlapped schedule: every window keeps its own selection and scalars, and the data
        # movement and the attention have streams of their own
        T = plan.n_windows
        self.idx_all = torch.full((T, runner.k_cap), -1, dtype=torch.int32, device=dev)
        self.n_sel_all = torch.zeros(T, dtype=torch.int32, device=dev)
        self.idx_slots_all = torch.full((T, runner.k_cap), -1, dtype=torch.int32, device=dev)
        # (four streams with the current one: a process has four hardware queues here, and streams that
        # share one run their kernels one after the other)
        self.mover, self.attender, self.writer = (torch.cuda.Stream(device=dev) for _ in range(3))
        self.geo = self.window_geometry()
        self.n_ctx_w = torch.tensor([g["pos0"] + plan.rows[t] for t, g in enumerate(self.geo)], dtype=torch.int32,
                                    device=dev)
        self.pos0_w = torch.tensor([g["pos0"] for g in self.geo], dtype=torch.int32, device=dev)
        # per-window views and events, made once (slicing and creating them costs the host as much as
        # a launch, and the overlapped schedule is bound by what the host can enqueue)
        one = lambda x: None if x is None else [x[t:t + 1] for t in range(T)]
        self.v_idx, self.v_nsel, self.v_slots = one(self.idx_all), one(self.n_sel_all), one(self.idx_slots_all)
        self.v_nctx, self.v_pos0, self.v_nb_end = one(self.n_ctx_w), one(self.pos0_w), one(plan.nb_end)
        self.v_bud, self.v_rest = one(plan.budget), one(plan.rest)
        self.ev_appended = [torch.cuda.Event() for _ in range(T)]
        self.ev_written = [torch.cuda.Event() for _ in range(T)]

    def _copy_blocks(self, src, dst, src_block: int, dst_block: int, n: int, stream=None) -> None:
        if n > 0:
            bb = self.block_bytes
            B.copy_bytes_at(dst, dst_block * bb, src, src_block * bb, n * bb, stream)

    def run(self, q: torch.Tensor, k_tok: torch.Tensor, v_tok: torch.Tensor, k_store: torch.Tensor,
            v_store: torch.Tensor, rep_keys: torch.Tensor, out: torch.Tensor,
            record: Optional[Sequence[int]] = None, gather_events=None) -> Dict[int, Dict[str, torch.Tensor]]:
        """q, out [N][H][D]; k_tok, v_tok [N][Hk][D] on the device (the windows' new keys and
        values); k_store, v_store: the blocked cache of the whole context in pinned host memory
        (already holding every block a window can select, i.e. everything older than its local
        span); rep_keys [nb][r][Hk][D] on the device.  gather_events: optional per-window
        (start, end) event pairs recorded around the window's actqkv_gather_blocks call."""
        r, plan = self.runner, self.plan
        sh, cs, bs = r.shape, r.cs, r.shape.block_size
        nb_begin = sh.n_init // bs
        nb_store = k_store.shape[0]
        rec: Dict[int, Dict[str, torch.Tensor]] = {}
        cur, delta, has_init = 0, 0, [True, False]     # cache in use, real block - working block of its tail
        self.gathered_blocks = 0
        for t in range(plan.n_windows):
            w0, rows = plan.w0[t], plan.rows[t]
            l0 = local_start(sh, w0)
            if l0 <= sh.n_init:
                # the whole context fits: true positions, nothing is eligible for retrieval
                new, pos0, new_delta = 0, w0, 0
                assert cur == 0 and w0 + rows <= self.nb_work * bs
            else:
                new = 1 - cur
                n_loc = (w0 - l0) // bs
                if not has_init[new]:
                    self._copy_blocks(self.k_work[cur], self.k_work[new], 0, 0, self.slot0)
                    self._copy_blocks(self.v_work[cur], self.v_work[new], 0, 0, self.slot0)
                    has_init[new] = True
                self._copy_blocks(self.k_work[cur], self.k_work[new], l0 // bs - delta, self.tail0, n_loc)
                self._copy_blocks(self.v_work[cur], self.v_work[new], l0 // bs - delta, self.tail0, n_loc)
                pos0 = (self.tail0 + n_loc) * bs
                new_delta = l0 // bs - self.tail0
            self.pos0_work.fill_(pos0)
            self.n_ctx_work.fill_(pos0 + rows)
            B.append_kv(cs, 1, rows, k_tok[w0:w0 + rows], v_tok[w0:w0 + rows], self.pos0_work, self.k_work[new],
                        self.v_work[new], 0, None, 0, self.nb_work)
            bud = None if plan.budget is None else plan.budget[t:t + 1]
            rest = None if plan.rest is None else plan.rest[t:t + 1]
            nb_cap = min(max(plan.nb_end_host[t], nb_begin), r.nb_capacity)
            qw = q[w0:w0 + rows]
            B.build_probe(cs, 1, rows, qw, r.stats, True, r.probe, r.probe_kv, r.probe_norm, None, r.workspace)
            B.score_blocks(cs, 1, r.probe_kv, r.probe_norm, rep_keys, 0, nb_cap, nb_begin, plan.nb_end[t:t + 1],
                           r.scores, r.score_stride)
            B.select(1, r.scores, r.score_stride, nb_cap, nb_begin, plan.nb_end[t:t + 1], r.k_cap, bud, rest,
                     r.idx, r.n_sel, r.theta, r.budget)
            if gather_events is not None:
                gather_events[t][0].record()
            B.gather_blocks(cs, 1, k_store, v_store, 0, nb_store, r.idx, r.n_sel, r.k_cap, self.k_work[new],
                            self.v_work[new], 0, self.nb_work, self.slot0, self.idx_slots)
            if gather_events is not None:
                gather_events[t][1].record()
            B.retrieval_attention(cs, 1, rows, qw, self.k_work[new], self.v_work[new], 0, self.nb_work,
                                  self.n_ctx_work, self.idx_slots, r.n_sel, r.k_cap, out[w0:w0 + rows], None,
                                  self.workspace)
            if record is not None and t in record:
                rec[t] = dict(idx=r.idx[0].clone(), n_sel=r.n_sel[0].clone(), idx_slots=self.idx_slots[0].clone())
            cur, delta = new, new_delta
        return rec

    def window_geometry(self):
        """Per window: (working cache, the cache the local span comes from, real block - working block
        of the tail, first working block of the local span in the source cache, blocks of local
        span, position of the window's first token in the working cache, needs the initial blocks
        copied).  Host-side bookkeeping only."""
        r, plan = self.runner, self.plan
        sh, bs = r.shape, r.shape.block_size
        geo = []
        cur, delta, has_init = 0, 0, [True] + [False] * (self.N_WORK - 1)
        for t in range(plan.n_windows):
            w0, rows = plan.w0[t], plan.rows[t]
            l0 = local_start(sh, w0)
            if l0 <= sh.n_init:
                assert cur == 0 and w0 + rows <= self.nb_work * bs
                geo.append(dict(new=0, src=0, src_block=0, n_loc=0, pos0=w0, copy_init=False, retrieving=False))
                new, new_delta = 0, 0
            else:
                new = (cur + 1) % self.N_WORK
                n_loc = (w0 - l0) // bs
                geo.append(dict(new=new, src=cur, src_block=l0 // bs - delta, n_loc=n_loc,
                                pos0=(self.tail0 + n_loc) * bs, copy_init=not has_init[new], retrieving=True))
                has_init[new] = True
                new_delta = l0 // bs - self.tail0
            cur, delta = new, new_delta
        return geo

    def run_overlapped(self, q: torch.Tensor, k_tok: torch.Tensor, v_tok: torch.Tensor, k_store: torch.Tensor,
                       v_store: torch.Tensor, rep_keys: torch.Tensor, out: torch.Tensor,
                       write_back: bool = True) -> Dict[int, Dict[str, torch.Tensor]]:
        """The same pass with the host link kept busy.  Four chains, handed over GROUP windows at a
        time (a hand-over between streams costs the host more than a launch): on the current stream
        the selection chain (it needs the queries and the representative keys only) and what is
        always resident - the local span into the window's working cache, the window's keys and
        values behind it; with write_back a second stream copies the window's new blocks from the
        working cache to the host store (the link carries both directions at once), so the store
        may start empty; a third does nothing but gather the selected blocks from the host store
        into the slots, back to back; a fourth attends.  A window can select
        blocks of the window two before it, so its gather waits for that window's write-back.
        Results are those of run()."""
        r, plan = self.runner, self.plan
        sh, cs, bs = r.shape, r.cs, r.shape.block_size
        nb_begin = sh.n_init // bs
        nb_store = k_store.shape[0]
        T, G = plan.n_windows, self.GROUP
        geo, n_ctx_w, pos0_w = self.geo, self.n_ctx_w, self.pos0_w
        cur = torch.cuda.current_stream()
        for st in (self.mover, self.attender, self.writer):
            st.wait_stream(cur)
        attended, written = {}, {}      # events: group g attended to; window t written back
        mover, attender, writer, prep = self.mover, self.attender, self.writer, cur
        for g0 in range(0, T, G):
            g, group = g0 // G, range(g0, min(g0 + G, T))
            # ---- selection chain (current stream)
            for t in group:
                w0, rows = plan.w0[t], plan.rows[t]
                bud = None if self.v_bud is None else self.v_bud[t]
                rest = None if self.v_rest is None else self.v_rest[t]
                nb_cap = min(max(plan.nb_end_host[t], nb_begin), r.nb_capacity)
                B.build_probe(cs, 1, rows, q[w0:w0 + rows], r.stats, True, r.probe, r.probe_kv, r.probe_norm, None,
                              r.workspace)
                B.score_blocks(cs, 1, r.probe_kv, r.probe_norm, rep_keys, 0, nb_cap, nb_begin, self.v_nb_end[t],
                               r.scores, r.score_stride)
                B.select(1, r.scores, r.score_stride, nb_cap, nb_begin, self.v_nb_end[t], r.k_cap, bud, rest,
                         self.v_idx[t], self.v_nsel[t], None, None)
            selected = torch.cuda.Event()
            selected.record(cur)
            # ---- The working caches go round: the ones this group fills were last used two groups ago
            # (attention, write-back, source of a local span).
            for st in (prep, mover):
                if g - 2 in attended:
                    st.wait_event(attended[g - 2])
                    last = min((g - 1) * G, T) - 1
                    if last in written:
                        st.wait_event(written[last])
            # ---- what is always resident (still the current stream): the local span into the window's
            # working cache, the window's keys and values behind it; the new blocks back to the store
            # (second stream)
            for t in group:
                w0, rows = plan.w0[t], plan.rows[t]
                ge = geo[t]
                kw, vw = self.k_work[ge["new"]], self.v_work[ge["new"]]
                if ge["retrieving"]:
                    ks, vs = self.k_work[ge["src"]], self.v_work[ge["src"]]
                    if ge["copy_init"]:
                        self._copy_blocks(ks, kw, 0, 0, self.slot0, prep)
                        self._copy_blocks(vs, vw, 0, 0, self.slot0, prep)
                    self._copy_blocks(ks, kw, ge["src_block"], self.tail0, ge["n_loc"], prep)
                    self._copy_blocks(vs, vw, ge["src_block"], self.tail0, ge["n_loc"], prep)
                B.append_kv(cs, 1, rows, k_tok[w0:w0 + rows], v_tok[w0:w0 + rows], self.v_pos0[t], kw, vw, 0,
                            None, 0, self.nb_work, prep)
                if write_back and rows // bs > 0:
                    self.ev_appended[t].record(prep)
                    writer.wait_event(self.ev_appended[t])
                    wb0, n_wb = ge["pos0"] // bs, rows // bs
                    self._copy_blocks(kw, k_store, wb0, w0 // bs, n_wb, writer)
                    self._copy_blocks(vw, v_store, wb0, w0 // bs, n_wb, writer)
                    written[t] = self.ev_written[t]
                    written[t].record(writer)
            prepped = torch.cuda.Event()
            prepped.record(prep)
            # ---- the selected blocks over the host link into the slots (third stream: nothing but
            # gathers, back to back, so that the link never waits for anything else)
            mover.wait_event(selected)
            for t in group:
                ge = geo[t]
                if t - 2 in written:
                    mover.wait_event(written[t - 2])         # the newest blocks this window can select
                B.gather_blocks(cs, 1, k_store, v_store, 0, nb_store, self.v_idx[t], self.v_nsel[t], r.k_cap,
                                self.k_work[ge["new"]], self.v_work[ge["new"]], 0, self.nb_work, self.slot0,
                                self.v_slots[t], mover)
            moved = torch.cuda.Event()
            moved.record(mover)
            # ---- attention (fourth stream)
            attender.wait_event(moved)
            attender.wait_event(prepped)
            for t in group:
                w0, rows = plan.w0[t], plan.rows[t]
                ge = geo[t]
                B.retrieval_attention(cs, 1, rows, q[w0:w0 + rows], self.k_work[ge["new"]], self.v_work[ge["new"]],
                                      0, self.nb_work, self.v_nctx[t], self.v_slots[t], self.v_nsel[t], r.k_cap,
                                      out[w0:w0 + rows], None, self.workspace, attender)
            attended[g] = torch.cuda.Event()
            attended[g].record(attender)
        for st in (self.mover, self.attender, self.writer):
            cur.wait_stream(st)
        return {t: dict(idx=self.idx_all[t], n_sel=self.n_sel_all[t], idx_slots=self.idx_slots_all[t])
                for t in range(T)}
