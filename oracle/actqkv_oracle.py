"""CPU oracle for the ActQKV per-layer retrieval-attention path (numpy, fp64).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares no code with the
HIP library and imports nothing from the package.

It is written for reading, not for speed: every function is one definition or
one algorithm step of the paper, in the paper's order and notation, with the
citation beside it.  Nothing is blocked, fused or reordered.  All arithmetic is
float64; inputs are the stored bits (fp32 or bf16) widened exactly.

Readings taken where the paper is silent or ambiguous (each one is also listed
in the design notes of the repository):
  * Sec. 4.1, Eq. (7): the square and the division act per channel; the mean
    and the variance are vectors over the d = H*D channels of a query.
  * Eq. (8): statistics run over all queries of windows 1..t, the current
    window included, with the unbiased denominator m*t - 1.
  * Eq. (9): the norm of the bias matrix is the entrywise L1 norm, so the
    weights of the window's tokens sum to one.
  * Heads: the paper works with one d-dimensional query per token, so the
    probe-Query, the block scores and the selection are shared by all heads.
    With grouped-query attention a key is repeated to the H query heads
    (query head h reads KV head h // G) before the cosine of Eq. (10).
  * Blocks: the retrieval unit is a block of consecutive tokens (Sec. 5.1
    works with chunks).  A block's score is the mean of Eq. (10) over its r
    representative keys, which are an input.
  * Eq. (11): plain softmax (no temperature), natural logarithm, over the
    eligible blocks.
  * Eq. (12) / Alg. 1: the budget is counted in blocks; the sum of the mean
    densities of the layers still to come is an input R; the number of blocks
    taken is E = round-half-up(B^l), at least 1, at most k_cap and the number
    of eligible blocks; B_kv is decremented by the real-valued B^l.
  * Sorting by the softmax of the scores is sorting by the scores; equal
    scores keep the lower block index first.
  * Cache update (Eq. (4)): concatenation.  Which tokens represent a block is
    not stated in the paper (it builds on earlier block-retrieval work); the
    rule taken: the r tokens whose key over all KV heads together has the
    largest L2 norm, ties to the lower position, kept in position order.
  * Attention (Eq. (2), (3)): scale 1/sqrt(D); the first n_init tokens and the
    n_local tokens before the window (start rounded down to a block boundary)
    are always visible; the window itself is causal; queries and keys are
    taken as given (already position-encoded).

parity unpinned: which of these readings the authors' own code takes.  The
paper prints no numeric example, so no value can pin them; every function below
is pinned by closed forms, invariants, special cases and brute force instead.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

VAR_EPS = 1e-12


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------
# Sec. 4.1: Activation Bias and probe-Query
# --------------------------------------------------------------------------
def running_stats_literal(q_all) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (8), written out.  q_all [m*t][d]: every query of windows 1..t.
    Returns (z_bar [d], sigma2 [d]).  With a single query the variance has a
    zero denominator; it is returned as 0 and floored by the caller."""
    q_all = _f64(q_all)
    n = q_all.shape[0]
    z_bar = q_all.sum(axis=0) / n
    dev2 = ((q_all - z_bar) ** 2).sum(axis=0)
    sigma2 = dev2 / (n - 1) if n > 1 else np.zeros_like(dev2)
    return z_bar, sigma2


class RunningStats:
    """The same two vectors as running_stats_literal, kept window by window so
    that a long context need not be stored: count, mean and the sum of squared
    deviations are merged with each new window (the textbook pairwise update,
    exact up to rounding order)."""

    def __init__(self, d: int):
        self.n = 0
        self.mean = np.zeros(d)
        self.m2 = np.zeros(d)

    def update(self, q_win) -> Tuple[np.ndarray, np.ndarray]:
        q_win = _f64(q_win)
        nb = q_win.shape[0]
        mean_b = q_win.mean(axis=0)
        m2_b = ((q_win - mean_b) ** 2).sum(axis=0)
        na = self.n
        n = na + nb
        delta = mean_b - self.mean
        self.mean = self.mean + delta * (nb / n)
        self.m2 = self.m2 + m2_b + delta ** 2 * (na * nb / n)
        self.n = n
        return self.z_bar, self.sigma2

    @property
    def z_bar(self) -> np.ndarray:
        return self.mean

    @property
    def sigma2(self) -> np.ndarray:
        return self.m2 / (self.n - 1) if self.n > 1 else np.zeros_like(self.m2)


def activation_bias(q_win, z_bar, sigma2, eps: float = VAR_EPS) -> np.ndarray:
    """Eq. (7): Phi [m][d], phi_j = (q_j - z_bar)^2 / sigma^2 per channel.
    A zero variance is floored at eps."""
    q_win = _f64(q_win)
    return (q_win - _f64(z_bar)) ** 2 / np.maximum(_f64(sigma2), eps)


def probe_query(q_win, phi) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (9): Q_probe = sum_j (||phi_j||_1 / ||Phi||_1) q_j.
    Returns (Q_probe [d], weights [m]).  If every bias is zero the weights are
    uniform (mean pooling)."""
    q_win = _f64(q_win)
    a = np.abs(_f64(phi)).sum(axis=1)          # ||phi_j||_1
    total = a.sum()                            # ||Phi||_1, entrywise
    m = q_win.shape[0]
    w = a / total if total > 0.0 else np.full(m, 1.0 / m)
    return w @ q_win, w


# --------------------------------------------------------------------------
# Sec. 3.2 / Sec. 4.2: scores, density, budget, selection
# --------------------------------------------------------------------------
def cosine(a, b) -> float:
    """Eq. (10).  Zero if either vector is zero."""
    a = _f64(a).ravel()
    b = _f64(b).ravel()
    na = math.sqrt(float(a @ a))
    nb = math.sqrt(float(b @ b))
    if na == 0.0 or nb == 0.0:
        return 0.0
    return float(a @ b) / (na * nb)


def block_scores(q_probe, rep_keys, group: int) -> np.ndarray:
    """Score of every block in rep_keys [NB][r][Hk][D] against Q_probe [H*D]:
    the mean over the block's r representative keys of Eq. (10), each key
    repeated to the H = Hk*group query heads."""
    rep_keys = _f64(rep_keys)
    nb, r = rep_keys.shape[:2]
    s = np.zeros(nb)
    for b in range(nb):
        acc = 0.0
        for j in range(r):
            k_hat = np.repeat(rep_keys[b, j], group, axis=0)     # [H][D], head h <- h // G
            acc += cosine(q_probe, k_hat)
        s[b] = acc / r
    return s


def block_scores_per_head(q_probe, rep_keys, group: int) -> np.ndarray:
    """The variant of the head-merged reading in which every KV head retrieves for itself:
    scores [Hk][NB], row hk being block_scores of the model cut down to KV head hk and its
    `group` query heads (the probe restricted to those heads, the keys of that head)."""
    rep_keys = _f64(rep_keys)
    hk_n, d = rep_keys.shape[2], rep_keys.shape[3]
    probe = _f64(q_probe).reshape(hk_n, group * d)
    return np.stack([block_scores(probe[hk], rep_keys[:, :, hk:hk + 1], group) for hk in range(hk_n)])


def information_density(scores) -> float:
    """Eq. (11): entropy (natural log) of softmax(scores)."""
    s = _f64(scores)
    e = np.exp(s - s.max())
    p = e / e.sum()
    return float(-(p * np.log(p)).sum())


def information_density_topk(scores, k: int) -> float:
    """The other reading of Eq. (11) (its domain is stated as the whole cache, while the
    perplexities Fig. 3 shows are close to the number of retrieved chunks): the same entropy
    over the k highest scores only."""
    s = np.sort(_f64(scores))[::-1][:k]
    return information_density(s)


def layer_budget(theta: float, rest: float, b_kv: float) -> float:
    """Eq. (12): B^l = Theta^l / (Theta^l + R) * B_kv, R = the summed mean
    densities of the layers still to come.  0/0 (one eligible block, nothing
    to come) hands over the whole remaining budget."""
    den = theta + rest
    return b_kv if den <= 0.0 else theta / den * b_kv


def cutoff_count(b_l: float, k_cap: int, n_eligible: int) -> int:
    """Alg. 1's E^l from the real-valued budget: round half up, at least one
    block, at most the capacity and the number of eligible blocks."""
    return int(min(k_cap, n_eligible, max(1, math.floor(b_l + 0.5))))


def select_blocks(scores, block_ids, count: int) -> List[int]:
    """Alg. 1, third loop / Eq. (5): block ids sorted by score, descending,
    equal scores by ascending id; the first `count` of them."""
    s = _f64(scores)
    ids = np.asarray(block_ids, dtype=np.int64)
    order = np.lexsort((ids, -s))               # primary -s ascending, then id
    return [int(ids[i]) for i in order[:count]]


# --------------------------------------------------------------------------
# key-set geometry (Sec. 5.1: attention sinks + local span + retrieved blocks)
# --------------------------------------------------------------------------
def local_start(w0: int, n_init: int, n_local: int, block: int) -> int:
    """First token of the local span of a window that starts at w0."""
    i0 = min(n_init, w0)
    a = w0 - n_local
    a = (a // block) * block if a > 0 else 0
    return max(i0, a)


def eligible_blocks(w0: int, n_init: int, n_local: int, block: int) -> List[int]:
    """Blocks that lie wholly after the initial tokens and wholly before the
    local span: the candidates of Eq. (5)."""
    l0 = local_start(w0, n_init, n_local, block)
    return [b for b in range(0, l0 // block + 1)
            if b * block >= n_init and (b + 1) * block <= l0]


def key_positions(w0: int, p: int, selected: Sequence[int], n_init: int, n_local: int,
                  block: int) -> List[int]:
    """Positions visible to the query at position p (w0 <= p) of the window
    starting at w0: initial tokens, the selected blocks, the local span and the
    window's own tokens up to p."""
    i0 = min(n_init, w0)
    l0 = local_start(w0, n_init, n_local, block)
    pos = list(range(0, i0))
    for b in selected:
        pos.extend(range(b * block, (b + 1) * block))
    pos.extend(range(l0, p + 1))
    return pos


def attention_rows(q_rows, k_all, v_all, positions: Sequence[int], group: int,
                   scale: Optional[float] = None) -> np.ndarray:
    """softmax(q K^T * scale) V for query rows q_rows [n][H][D] that all see
    exactly the keys at `positions` of k_all/v_all [N][Hk][D] (Eq. (1))."""
    q_rows = _f64(q_rows)
    n, h_n, d = q_rows.shape
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    pos = np.asarray(positions, dtype=np.int64)
    out = np.zeros((n, h_n, d))
    for h in range(h_n):
        g = h // group
        k = _f64(k_all[pos, g])
        v = _f64(v_all[pos, g])
        s = (q_rows[:, h] @ k.T) * scale
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h] = p @ v
    return out


def retrieval_attention(q_win, k_all, v_all, w0: int, selected: Sequence[int], n_init: int,
                        n_local: int, block: int, group: int,
                        rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Eq. (2) (prefill window) and Eq. (3) (decode, a window of one token):
    attention of the window's queries over [K^t, K*].  q_win [m][H][D];
    k_all, v_all hold every token up to the end of the window.  The causal mask
    inside the window is applied by giving each row its own key set.
    `rows` restricts the computation to some rows of the window (sampling)."""
    q_win = np.asarray(q_win)
    m = q_win.shape[0]
    rows = list(range(m)) if rows is None else list(rows)
    out = np.zeros((len(rows),) + q_win.shape[1:])
    for i, j in enumerate(rows):
        pos = key_positions(w0, w0 + j, selected, n_init, n_local, block)
        out[i] = attention_rows(q_win[j:j + 1], k_all, v_all, pos, group)[0]
    return out


def retrieval_attention_window(q_win, k_all, v_all, w0: int, selected: Sequence[int],
                               n_init: int, n_local: int, block: int, group: int) -> np.ndarray:
    """The same result as retrieval_attention for a whole window, computed with
    one masked score matrix per head instead of one key list per row (used
    where the row-by-row form would take hours; tests check the two agree)."""
    q_win = _f64(q_win)
    m, h_n, d = q_win.shape
    scale = 1.0 / math.sqrt(d)
    pos = np.asarray(key_positions(w0, w0 + m - 1, selected, n_init, n_local, block),
                     dtype=np.int64)
    visible = pos[None, :] <= (w0 + np.arange(m))[:, None]          # causal inside the window
    out = np.zeros((m, h_n, d))
    for h in range(h_n):
        g = h // group
        k = _f64(k_all[pos, g])
        v = _f64(v_all[pos, g])
        s = (q_win[:, h] @ k.T) * scale
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h] = p @ v
    return out


def retrieval_attention_per_head(q_win, k_all, v_all, w0: int, selected_per_head: Sequence[Sequence[int]],
                                 n_init: int, n_local: int, block: int, group: int) -> np.ndarray:
    """Eq. (2) with a selection of its own for every KV head: the query heads of group hk attend
    over the blocks selected_per_head[hk]."""
    q_win = np.asarray(q_win)
    out = np.zeros(q_win.shape)
    for hk, sel in enumerate(selected_per_head):
        hs = slice(hk * group, (hk + 1) * group)
        out[:, hs] = retrieval_attention_window(q_win[:, hs], np.asarray(k_all)[:, hk:hk + 1],
                                                np.asarray(v_all)[:, hk:hk + 1], w0, sel, n_init, n_local,
                                                block, group)
    return out


# --------------------------------------------------------------------------
# one retrieval step and the window loop
# --------------------------------------------------------------------------
def retrieve(q_probe, rep_keys, w0: int, n_init: int, n_local: int, block: int, group: int,
             k_cap: int, cutoff: Optional[Tuple[float, float]] = None) -> Dict:
    """Scores, density, budget and selection for one probe-Query (Alg. 1 for
    one layer).  cutoff = (B_kv, R) enables the dynamic cut-off; None takes the
    k_cap best blocks.  Returns a dict with the eligible ids, their scores,
    theta, budget (B^l), count (E), idx (selected ids, best first) and the
    remaining budget."""
    elig = eligible_blocks(w0, n_init, n_local, block)
    res = {"eligible": elig, "scores": np.zeros(0), "theta": 0.0, "budget": 0.0,
           "count": 0, "idx": [], "b_kv_after": None if cutoff is None else cutoff[0]}
    if not elig:
        return res
    s = block_scores(q_probe, np.asarray(rep_keys)[elig], group)
    theta = information_density(s)
    if cutoff is None:
        count = min(k_cap, len(elig))
        b_l = float(count)
    else:
        b_kv, rest = cutoff
        b_l = layer_budget(theta, rest, b_kv)
        count = cutoff_count(b_l, k_cap, len(elig))
        res["b_kv_after"] = b_kv - b_l
    res.update(scores=s, theta=theta, budget=b_l, count=count,
               idx=select_blocks(s, elig, count))
    return res


def retrieve_per_head(q_probe, rep_keys, w0: int, n_init: int, n_local: int, block: int, group: int,
                      k_cap: int, cutoffs: Optional[Sequence[Tuple[float, float]]] = None) -> List[Dict]:
    """`retrieve` run for every KV head on its own (scores, density, budget, count and
    selection per head); cutoffs[hk] = (B_kv, R) of that head, or None."""
    rep_keys = _f64(rep_keys)
    hk_n, d = rep_keys.shape[2], rep_keys.shape[3]
    probe = _f64(q_probe).reshape(hk_n, group * d)
    return [retrieve(probe[hk], rep_keys[:, :, hk:hk + 1], w0, n_init, n_local, block, group, k_cap,
                     None if cutoffs is None else cutoffs[hk]) for hk in range(hk_n)]


def prefill_layer(q, k, v, rep_keys, m: int, n_init: int, n_local: int, block: int,
                  k_cap: int, cutoffs: Optional[Sequence[Tuple[float, float]]] = None,
                  attend: Optional[Sequence[int]] = None, fast_attention: bool = True,
                  eps: float = VAR_EPS) -> List[Dict]:
    """Window-by-window prefill of one layer of one sequence (Sec. 3.1 with the
    selection of Sec. 4).  q [N][H][D]; k, v [N][Hk][D]; rep_keys
    [NB][r][Hk][D].  cutoffs[t] = (B_kv, R) per window or None.  `attend`
    lists the windows whose attention output is wanted (all if None); the
    probe and the selection are computed for every window either way."""
    q = np.asarray(q)
    n, h_n, d = q.shape
    group = h_n // k.shape[1]
    stats = RunningStats(h_n * d)
    out = []
    t = 0
    for w0 in range(0, n, m):
        q_win = q[w0:w0 + m]
        flat = _f64(q_win).reshape(q_win.shape[0], h_n * d)
        z_bar, sigma2 = stats.update(flat)
        phi = activation_bias(flat, z_bar, sigma2, eps)
        q_probe, w = probe_query(flat, phi)
        cut = None if cutoffs is None else cutoffs[t]
        res = retrieve(q_probe, rep_keys, w0, n_init, n_local, block, group, k_cap, cut)
        res.update(w0=w0, probe=q_probe, weights=w)
        if attend is None or t in attend:
            fn = retrieval_attention_window if fast_attention else retrieval_attention
            res["out"] = fn(q_win, k, v, w0, res["idx"], n_init, n_local, block, group)
        out.append(res)
        t += 1
    return out


def decode_step(q_tok, k, v, rep_keys, n_ctx: int, n_init: int, n_local: int, block: int,
                k_cap: int, cutoff: Optional[Tuple[float, float]] = None) -> Dict:
    """One decode step of one layer of one sequence (Eq. (3); Sec. 4.2: the
    probe-Query of a decode step is the query itself).  q_tok [H][D]; k, v hold
    n_ctx tokens, the new token's key and value last."""
    q_tok = np.asarray(q_tok)
    h_n, d = q_tok.shape
    group = h_n // k.shape[1]
    w0 = n_ctx - 1
    res = retrieve(_f64(q_tok).reshape(-1), rep_keys, w0, n_init, n_local, block, group,
                   k_cap, cutoff)
    res["out"] = retrieval_attention(q_tok[None], k[:n_ctx], v[:n_ctx], w0, res["idx"],
                                     n_init, n_local, block, group)[0]
    return res


# --------------------------------------------------------------------------
# Sec. 3.1, Eq. (4): cache update; representatives of a finished block
# --------------------------------------------------------------------------
def append_cache(k_cache, v_cache, k_new, v_new) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (4): the cache after a step is the cache before it with the step's keys and
    values appended.  All arrays [tokens][Hk][D]."""
    return (np.concatenate([np.asarray(k_cache), np.asarray(k_new)], axis=0),
            np.concatenate([np.asarray(v_cache), np.asarray(v_new)], axis=0))


def representative_tokens(k_block, r: int) -> List[int]:
    """Positions (inside the block, ascending) of the r tokens of k_block [Bs][Hk][D] whose
    key, all KV heads taken together, has the largest L2 norm; equal norms: lower position."""
    kb = _f64(k_block)
    norms = [math.sqrt(float((kb[j] * kb[j]).sum())) for j in range(kb.shape[0])]
    order = sorted(range(len(norms)), key=lambda j: (-norms[j], j))
    return sorted(order[:r])


def representative_keys(k_all, block: int, r: int) -> np.ndarray:
    """[NB][r][Hk][D] for the complete blocks of k_all [N][Hk][D] (same bits as stored)."""
    k_all = np.asarray(k_all)
    nb = k_all.shape[0] // block
    out = np.zeros((nb, r) + k_all.shape[1:], dtype=k_all.dtype)
    for b in range(nb):
        kb = k_all[b * block:(b + 1) * block]
        for slot, j in enumerate(representative_tokens(kb, r)):
            out[b, slot] = kb[j]
    return out


# --------------------------------------------------------------------------
# Sec. 4.2, Eq. (12) / Alg. 1 across the layers of a step and across steps
# --------------------------------------------------------------------------
class CutoffHistory:
    """The means of the layers' information densities over the steps so far, which stand in
    for the layers a step has not reached yet (Eq. (12): the sum over j > l of the mean
    density of layer j)."""

    def __init__(self, n_layers: int, theta_prior: float):
        self.sums = [0.0] * n_layers
        self.steps = 0
        self.prior = float(theta_prior)

    def means(self) -> List[float]:
        return [x / self.steps if self.steps > 0 else self.prior for x in self.sums]

    def rest_sums(self) -> List[float]:
        """R^l = sum of the mean densities of the layers after l, for every l."""
        mean = self.means()
        return [math.fsum(mean[l + 1:]) for l in range(len(mean))]

    def add_step(self, thetas: Sequence[float]) -> None:
        for l, th in enumerate(thetas):
            self.sums[l] += float(th)
        self.steps += 1


def step_budgets(thetas: Sequence[float], rest_sums: Sequence[float], k_mean: float) -> List[float]:
    """Second loop of Alg. 1 for one step: B_kv starts at L * k; layer l takes
    B^l = Theta^l / (Theta^l + R^l) * B_kv and leaves the rest."""
    b_kv = len(thetas) * float(k_mean)
    out = []
    for th, rest in zip(thetas, rest_sums):
        b_l = layer_budget(float(th), float(rest), b_kv)
        out.append(b_l)
        b_kv -= b_l
    return out
