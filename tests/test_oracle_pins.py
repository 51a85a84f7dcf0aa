"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numeric example for its Eq. (7)-(12), so every pin
is a closed form, an invariant, a special case that reduces to a textbook or
library routine, or brute force on tiny inputs.  They are chosen so that a
plausible slip in the oracle (a dropped term, n instead of n-1, a transposed
operand, a wrong head mapping, an off-by-one in the key set) fails one of them.
"""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
from scipy.spatial.distance import cosine as scipy_cosine_distance

from oracle import actqkv_oracle as orc

RNG = np.random.default_rng(7)


# ---------------------------------------------------------------- Sec. 4.1
def test_hand_example_eq7_to_eq9():
    # One channel, three queries 0, 1, 2: mean 1, unbiased variance 1,
    # biases 1, 0, 1, weights 1/2, 0, 1/2, probe = 1.
    q = np.array([[0.0], [1.0], [2.0]])
    z, s2 = orc.running_stats_literal(q)
    assert z[0] == 1.0 and s2[0] == 1.0
    phi = orc.activation_bias(q, z, s2)
    assert phi[:, 0].tolist() == [1.0, 0.0, 1.0]
    probe, w = orc.probe_query(q, phi)
    assert w.tolist() == [0.5, 0.0, 0.5] and probe[0] == 1.0
    # Two channels with different spread: the division is per channel.
    q = np.array([[0.0, 0.0], [2.0, 20.0], [4.0, 10.0]])
    z, s2 = orc.running_stats_literal(q)
    assert z.tolist() == [2.0, 10.0] and s2.tolist() == [4.0, 100.0]
    phi = orc.activation_bias(q, z, s2)
    assert np.allclose(phi, [[1.0, 1.0], [0.0, 1.0], [1.0, 0.0]])
    probe, w = orc.probe_query(q, phi)
    assert np.allclose(w, [0.5, 0.25, 0.25])
    assert np.allclose(probe, [0.5 * 0 + 0.25 * 2 + 0.25 * 4, 0.25 * 20 + 0.25 * 10])


def test_p1_weights_sum_to_one():
    q = RNG.normal(size=(37, 24))
    z, s2 = orc.running_stats_literal(q)
    _, w = orc.probe_query(q, orc.activation_bias(q, z, s2))
    assert (w >= 0).all() and abs(w.sum() - 1.0) < 1e-14


def test_p2_first_window_bias_mass():
    # At t = 1 every channel's biases sum to m - 1 (unbiased variance), so the
    # entrywise L1 norm of Phi is (m - 1) * d.  n instead of n - 1 gives m * d.
    m, d = 29, 12
    q = RNG.normal(size=(m, d)) * RNG.uniform(0.1, 9.0, size=d) + RNG.normal(size=d)
    z, s2 = orc.running_stats_literal(q)
    phi = orc.activation_bias(q, z, s2)
    assert np.allclose(phi.sum(axis=0), m - 1, rtol=1e-12)
    assert math.isclose(np.abs(phi).sum(), (m - 1) * d, rel_tol=1e-12)


def test_p3_equal_bias_is_mean_pooling():
    q = RNG.normal(size=(2, 16))
    z, s2 = orc.running_stats_literal(q)
    probe, w = orc.probe_query(q, orc.activation_bias(q, z, s2))
    assert np.allclose(w, 0.5) and np.allclose(probe, q.mean(axis=0))
    # all-zero bias (identical queries): uniform weights
    q = np.tile(RNG.normal(size=(1, 8)), (5, 1))
    z, s2 = orc.running_stats_literal(q)
    probe, w = orc.probe_query(q, orc.activation_bias(q, z, s2))
    assert np.allclose(w, 0.2) and np.allclose(probe, q[0])


def test_p4_affine_invariance_of_weights():
    q = RNG.normal(size=(21, 10))
    alpha = RNG.uniform(0.5, 4.0, size=10) * RNG.choice([-1.0, 1.0], size=10)
    beta = RNG.normal(size=10) * 3
    w = []
    for x in (q, q * alpha + beta):
        z, s2 = orc.running_stats_literal(x)
        w.append(orc.probe_query(x, orc.activation_bias(x, z, s2))[1])
    assert np.allclose(w[0], w[1], rtol=1e-10)


def test_outlier_token_dominates_probe():
    # A token far from the mean gets the largest weight (Eq. (6)'s intent).
    q = RNG.normal(size=(64, 8))
    q[17] += 25.0
    z, s2 = orc.running_stats_literal(q)
    _, w = orc.probe_query(q, orc.activation_bias(q, z, s2))
    assert int(np.argmax(w)) == 17 and w[17] > 0.4


def test_p5_streaming_stats_match_two_pass():
    d = 9
    wins = [RNG.normal(size=(n, d)) * 3 + 5 for n in (16, 16, 16, 7)]
    st = orc.RunningStats(d)
    for i, w in enumerate(wins):
        z, s2 = st.update(w)
        cat = np.concatenate(wins[: i + 1], axis=0)
        z_l, s2_l = orc.running_stats_literal(cat)
        assert np.allclose(z, z_l, rtol=1e-12) and np.allclose(s2, s2_l, rtol=1e-12)
        assert np.allclose(z_l, np.mean(cat, axis=0))
        assert np.allclose(s2_l, np.var(cat, axis=0, ddof=1))


# ---------------------------------------------------------------- Eq. (10)
def test_p6_cosine():
    a, b = RNG.normal(size=40), RNG.normal(size=40)
    c = orc.cosine(a, b)
    assert math.isclose(c, 1.0 - scipy_cosine_distance(a, b), rel_tol=1e-12)
    assert -1.0 <= c <= 1.0
    assert math.isclose(orc.cosine(3.5 * a, 0.2 * b), c, rel_tol=1e-12)
    assert math.isclose(orc.cosine(a, -b), -c, rel_tol=1e-12)
    assert orc.cosine(a, np.zeros(40)) == 0.0
    assert orc.cosine([1, 0, 0], [0, 2, 0]) == 0.0


def test_p6_block_scores_group_mapping():
    hk, g, d, nb, r = 3, 4, 8, 5, 2
    rep = RNG.normal(size=(nb, r, hk, d))
    probe = RNG.normal(size=(hk * g, d))
    s = orc.block_scores(probe.reshape(-1), rep, g)
    # independent expansion: query head h reads KV head h // g
    for b in range(nb):
        acc = 0.0
        for j in range(r):
            k_hat = np.stack([rep[b, j, h // g] for h in range(hk * g)])
            acc += 1.0 - scipy_cosine_distance(probe.reshape(-1), k_hat.reshape(-1))
        assert math.isclose(s[b], acc / r, rel_tol=1e-12)
    assert (np.abs(s) <= 1.0).all()
    # probe equal across the heads of a group and keys proportional to it: score 1
    base = RNG.normal(size=(hk, d))
    probe1 = np.repeat(base, g, axis=0).reshape(-1)
    rep1 = np.stack([np.stack([base * c for c in (0.5, 7.0)])])
    assert math.isclose(orc.block_scores(probe1, rep1, g)[0], 1.0, rel_tol=1e-12)
    # G = 1 is the plain cosine
    s1 = orc.block_scores(probe[:hk].reshape(-1), rep, 1)
    assert math.isclose(s1[2], np.mean([1.0 - scipy_cosine_distance(probe[:hk].ravel(),
                                                                   rep[2, j].ravel())
                                        for j in range(r)]), rel_tol=1e-12)


# ---------------------------------------------------------------- Eq. (11), (12)
def test_p7_information_density():
    n = 46
    assert math.isclose(orc.information_density(np.full(n, 0.3)), math.log(n), rel_tol=1e-13)
    s = RNG.uniform(-1, 1, size=n)
    th = orc.information_density(s)
    assert math.isclose(th, scipy.stats.entropy(scipy.special.softmax(s)), rel_tol=1e-12)
    assert th < math.log(n) and math.exp(th) <= n
    # spreading the scores out around their mean lowers the density
    wide = s.mean() + 3.0 * (s - s.mean())
    assert orc.information_density(wide) < th
    # shift invariance
    assert math.isclose(orc.information_density(s + 0.25), th, rel_tol=1e-12)


def test_p8_budgets_telescope():
    L, k_bar = 32, 46
    theta = RNG.uniform(2.0, 4.0, size=L)
    b_kv = float(L * k_bar)
    budgets = []
    for l in range(L):
        rest = float(theta[l + 1:].sum())          # exact driver: mean density = the layer's own
        b = orc.layer_budget(float(theta[l]), rest, b_kv)
        budgets.append(b)
        b_kv -= b
    budgets = np.array(budgets)
    assert np.allclose(budgets, L * k_bar * theta / theta.sum(), rtol=1e-10)
    assert math.isclose(budgets.sum(), L * k_bar, rel_tol=1e-12) and abs(b_kv) < 1e-9
    # equal densities: every layer gets k_bar
    b_kv = float(L * k_bar)
    for l in range(L):
        b = orc.layer_budget(3.0, 3.0 * (L - 1 - l), b_kv)
        assert math.isclose(b, k_bar, rel_tol=1e-10)
        b_kv -= b


def test_p7b_information_density_over_the_best_blocks():
    """The variant reading of Eq. (11): entropy over the k highest scores.  Closed forms: k equal
    scores on top give ln k whatever lies below; with k >= n it is the plain density; it never
    exceeds ln k; two scores a and a - d on top give the binary entropy of 1 / (1 + e^-d)."""
    rng = np.random.default_rng(5)
    low = rng.uniform(-3.0, -1.0, size=40)
    s = np.concatenate([low, np.full(7, 0.5)])
    rng.shuffle(s)
    assert math.isclose(orc.information_density_topk(s, 7), math.log(7), rel_tol=1e-13)
    assert orc.information_density_topk(s, 8) < math.log(8)
    assert math.isclose(orc.information_density_topk(s, 100), orc.information_density(s), rel_tol=1e-13)
    assert math.isclose(orc.information_density_topk(s, len(s)), orc.information_density(s), rel_tol=1e-13)
    d = 0.75
    two = np.concatenate([low, [1.0, 1.0 - d]])
    p = 1.0 / (1.0 + math.exp(-d))
    assert math.isclose(orc.information_density_topk(two, 2), -(p * math.log(p) + (1 - p) * math.log(1 - p)),
                        rel_tol=1e-12)
    assert orc.information_density_topk(np.array([0.3]), 4) == 0.0
    # brute force on a tiny case: every subset of size k has at most the entropy bound, and the
    # function picks the subset of the k largest
    t = rng.normal(size=6)
    best = sorted(t)[-3:]
    e = np.exp(np.array(best) - max(best)); q = e / e.sum()
    assert math.isclose(orc.information_density_topk(t, 3), float(-(q * np.log(q)).sum()), rel_tol=1e-12)


def test_p8b_scores_and_attention_per_kv_head():
    """Per-KV-head retrieval (the alternative to the head-merged reading).  Closed forms: a
    block whose key of head hk is parallel to that head's share of the probe scores exactly 1 in
    row hk and what the other heads' keys give elsewhere; with one KV head the rows are the
    merged scores; exchanging two KV heads exchanges the rows; giving every head the same
    selection reproduces the merged attention; a head's output depends on its own selection only."""
    rng = np.random.default_rng(21)
    hk_n, g, d, nb, r = 3, 2, 8, 6, 2
    probe = rng.normal(size=(hk_n * g, d))
    rep = rng.normal(size=(nb, r, hk_n, d))
    share = probe.reshape(hk_n, g, d)
    # head 1 of block 4: every representative key parallel to the SUM of the group's probe rows
    # is not enough for cosine 1 (the key is repeated to both heads); make the group's rows equal
    probe[2] = probe[3]
    rep[4, :, 1] = 2.5 * probe[2]
    s = orc.block_scores_per_head(probe.reshape(-1), rep, g)
    assert s.shape == (hk_n, nb) and math.isclose(s[1, 4], 1.0, rel_tol=1e-12)
    assert abs(s[0, 4]) < 1.0 and abs(s[2, 4]) < 1.0
    one = orc.block_scores_per_head(probe[:g].reshape(-1), rep[:, :, :1], g)
    assert np.allclose(one[0], orc.block_scores(probe[:g].reshape(-1), rep[:, :, :1], g), rtol=1e-13)
    perm = [2, 1, 0]
    probe_p = probe.reshape(hk_n, g, d)[perm].reshape(hk_n * g, d)
    s_p = orc.block_scores_per_head(probe_p.reshape(-1), rep[:, :, perm], g)
    assert np.allclose(s_p, s[perm], rtol=1e-13)
    # the merged score is NOT the mean of the rows (the norms differ per head): a real variant
    assert not np.allclose(orc.block_scores(probe.reshape(-1), rep, g), s.mean(axis=0))
    # attention
    n, m, block = 6 * 4 + 3, 4, 4
    q = rng.normal(size=(m, hk_n * g, d))
    k = rng.normal(size=(n, hk_n, d))
    v = rng.normal(size=(n, hk_n, d))
    w0 = n - m
    same = orc.retrieval_attention_per_head(q, k, v, w0, [[1, 3]] * hk_n, 4, 4, block, g)
    assert np.allclose(same, orc.retrieval_attention(q, k, v, w0, [1, 3], 4, 4, block, g), rtol=1e-12, atol=1e-14)
    a = orc.retrieval_attention_per_head(q, k, v, w0, [[1], [2, 3], []], 4, 4, block, g)
    b = orc.retrieval_attention_per_head(q, k, v, w0, [[1], [3], [2]], 4, 4, block, g)
    assert np.allclose(a[:, :g], b[:, :g], rtol=1e-13) and not np.allclose(a[:, g:2 * g], b[:, g:2 * g])
    # the per-head retrieval is `retrieve` on the cut-down model
    res = orc.retrieve_per_head(probe.reshape(-1), rep, 5 * block, block, block, block, g, 2, None)
    elig = orc.eligible_blocks(5 * block, block, block, block)
    for hk in range(hk_n):
        assert res[hk]["idx"] == orc.select_blocks(s[hk][elig], elig, 2)


def test_p9_budget_monotone_in_density():
    thetas = np.linspace(0.01, 7.0, 200)
    b = [orc.layer_budget(float(t), 90.0, 640.0) for t in thetas]
    assert all(x < y for x, y in zip(b, b[1:]))
    e = [orc.cutoff_count(x, 32, 1000) for x in b]
    assert all(x <= y for x, y in zip(e, e[1:]))
    assert orc.cutoff_count(0.2, 32, 1000) == 1          # never fewer than one block
    assert orc.cutoff_count(99.0, 32, 1000) == 32        # capacity
    assert orc.cutoff_count(99.0, 32, 5) == 5            # not more than there are
    assert orc.cutoff_count(6.5, 32, 1000) == 7 and orc.cutoff_count(6.49, 32, 1000) == 6


def test_p10_selection_is_a_stable_sort_prefix():
    for trial in range(50):
        n = int(RNG.integers(1, 12))
        s = RNG.integers(0, 4, size=n) / 4.0               # many ties
        ids = sorted(RNG.choice(100, size=n, replace=False).tolist())
        # brute force: repeatedly take the best remaining, lowest id on ties
        remaining = list(zip(s.tolist(), ids))
        expect = []
        while remaining:
            best = max(x[0] for x in remaining)
            pick = min(i for (v, i) in remaining if v == best)
            expect.append(pick)
            remaining = [x for x in remaining if x[1] != pick]
        for count in range(0, n + 1):
            assert orc.select_blocks(s, ids, count) == expect[:count]
    assert sorted(orc.select_blocks(RNG.normal(size=6), list(range(3, 9)), 6)) == list(range(3, 9))


# ---------------------------------------------------------------- geometry
@pytest.mark.parametrize("n_init,n_local,block", [(128, 256, 128), (128, 512, 128), (64, 96, 32),
                                                  (0, 64, 32), (64, 0, 32)])
def test_key_set_partition(n_init, n_local, block):
    # With every eligible block selected, the visible positions of the query at
    # p are exactly 0..p, each once.
    for w0 in list(range(0, 9 * block, block)) + [5, block + 3, 7 * block + 17, 2000]:
        elig = orc.eligible_blocks(w0, n_init, n_local, block)
        l0 = orc.local_start(w0, n_init, n_local, block)
        assert min(n_init, w0) <= l0 <= w0
        assert w0 - l0 < n_local + block or l0 == min(n_init, w0)
        if w0 - n_local >= n_init:
            assert w0 - l0 >= n_local
        for p in (w0, w0 + 1, w0 + block + 1):
            pos = orc.key_positions(w0, p, elig, n_init, n_local, block)
            assert sorted(pos) == list(range(p + 1))


# ---------------------------------------------------------------- attention
def _dense_causal_attention(q, k, v):
    """Textbook causal attention, one query at a time: q [N][H][D], k, v [N][Hk][D]."""
    n, h_n, d = q.shape
    g = h_n // k.shape[1]
    out = np.zeros((n, h_n, d))
    for p in range(n):
        for h in range(h_n):
            logits = np.array([np.dot(q[p, h], k[i, h // g]) for i in range(p + 1)]) / math.sqrt(d)
            pr = scipy.special.softmax(logits)
            out[p, h] = sum(pr[i] * v[i, h // g] for i in range(p + 1))
    return out


@pytest.mark.parametrize("fast", [False, True])
def test_p11_select_all_is_dense_causal_attention(fast):
    n, h_n, hk, d, m, block, n_init, n_local, r = 96, 4, 2, 8, 16, 8, 8, 16, 2
    q = RNG.normal(size=(n, h_n, d))
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    rep = k[: (n // block) * block].reshape(n // block, block, hk, d)[:, :r]
    res = orc.prefill_layer(q, k, v, rep, m, n_init, n_local, block, k_cap=10 ** 6,
                            fast_attention=fast)
    got = np.concatenate([w["out"] for w in res], axis=0)
    want = _dense_causal_attention(q, k, v)
    assert np.abs(got - want).max() < 1e-13
    # the last windows do have eligible blocks, and all of them were taken
    assert res[-1]["idx"] and sorted(res[-1]["idx"]) == res[-1]["eligible"]


def test_p11_decode_select_all_is_last_row_of_dense():
    n, h_n, hk, d, block, n_init, n_local, r = 75, 4, 2, 8, 8, 8, 16, 2
    q = RNG.normal(size=(n, h_n, d))
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    rep = k[: (n // block) * block].reshape(n // block, block, hk, d)[:, :r]
    res = orc.decode_step(q[-1], k, v, rep, n, n_init, n_local, block, k_cap=10 ** 6)
    want = _dense_causal_attention(q, k, v)[-1]
    assert np.abs(res["out"] - want).max() < 1e-13


def test_p12_attention_rows():
    n, hk, d = 40, 2, 8
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    q = RNG.normal(size=(3, 4, d))
    # one visible key: the output is its value
    o = orc.attention_rows(q, k, v, [11], group=2)
    assert np.allclose(o[:, 0], v[11, 0]) and np.allclose(o[:, 3], v[11, 1])
    # constant values: probabilities sum to one
    vc = np.tile(RNG.normal(size=(1, hk, d)), (n, 1, 1))
    o = orc.attention_rows(q, k, vc, list(range(n)), group=2)
    assert np.allclose(o[:, 1], vc[0, 0]) and np.allclose(o[:, 2], vc[0, 1])
    # the order of the gathered keys does not matter
    a = orc.attention_rows(q, k, v, [3, 4, 5, 20, 21], group=2)
    b = orc.attention_rows(q, k, v, [21, 3, 20, 5, 4], group=2)
    assert np.allclose(a, b, rtol=1e-12)
    # a key with a much larger logit takes all the mass
    k2 = k.copy()
    k2[7, 0] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    o = orc.attention_rows(q[:1], k2, v, list(range(n)), group=2)
    assert np.allclose(o[0, 0], v[7, 0], atol=1e-9)


def test_window_attention_forms_agree_with_selection():
    n, h_n, hk, d, m, block, n_init, n_local = 160, 4, 2, 8, 16, 8, 8, 16
    q = RNG.normal(size=(n, h_n, d))
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    w0 = 128
    sel = [9, 3, 5]
    a = orc.retrieval_attention(q[w0:w0 + m], k, v, w0, sel, n_init, n_local, block, 2)
    b = orc.retrieval_attention_window(q[w0:w0 + m], k, v, w0, sel, n_init, n_local, block, 2)
    assert np.abs(a - b).max() < 1e-13
    # hidden blocks really are hidden: changing an unselected, non-local block changes nothing
    k2, v2 = k.copy(), v.copy()
    k2[4 * block:5 * block] += 3.0
    v2[4 * block:5 * block] -= 2.0
    c = orc.retrieval_attention(q[w0:w0 + m], k2, v2, w0, sel, n_init, n_local, block, 2)
    assert np.abs(a - c).max() == 0.0


# ---------------------------------------------------------------- end to end
def test_p13_planted_blocks_are_retrieved():
    n, h_n, hk, d, m, block, n_init, n_local, r = 2048, 4, 2, 16, 64, 32, 32, 64, 4
    g = h_n // hk
    u = RNG.normal(size=(hk, d))
    u /= np.linalg.norm(u)
    q = RNG.normal(size=(n, h_n, d))
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    outl = RNG.uniform(size=n) < 0.05
    q[outl] += 12.0 * np.repeat(u, g, axis=0)
    planted = [3, 11, 17, 30]
    for b in planted:
        k[b * block:(b + 1) * block] += 4.0 * u
    rep = k.reshape(n // block, block, hk, d)[:, :r]
    res = orc.prefill_layer(q, k, v, rep, m, n_init, n_local, block, k_cap=4, attend=[])
    last = res[-1]
    assert sorted(last["idx"]) == planted
    assert last["theta"] < math.log(len(last["eligible"]))


def test_cutoff_path_and_budget_bookkeeping():
    n, h_n, hk, d, m, block, n_init, n_local, r = 1024, 4, 2, 16, 64, 32, 32, 64, 2
    q = RNG.normal(size=(n, h_n, d))
    k = RNG.normal(size=(n, hk, d))
    v = RNG.normal(size=(n, hk, d))
    rep = k.reshape(n // block, block, hk, d)[:, :r]
    cut = [(40.0, 30.0)] * (n // m)
    res = orc.prefill_layer(q, k, v, rep, m, n_init, n_local, block, k_cap=8, cutoffs=cut,
                            attend=[])
    for w in res:
        ne = len(w["eligible"])
        if ne == 0:
            assert w["count"] == 0 and w["idx"] == []
            continue
        b = w["theta"] / (w["theta"] + 30.0) * 40.0
        assert math.isclose(w["budget"], b, rel_tol=1e-12)
        assert math.isclose(w["b_kv_after"], 40.0 - b, rel_tol=1e-12)
        assert w["count"] == min(8, ne, max(1, math.floor(b + 0.5))) == len(w["idx"])
        top = np.sort(w["scores"])[::-1][: w["count"]]
        got = [w["scores"][w["eligible"].index(i)] for i in w["idx"]]
        assert np.allclose(got, top)


# ---------------------------------------------------------------- Eq. (4) and the representatives
def test_append_is_concatenation_and_blocks_are_stable():
    rng = np.random.default_rng(7)
    k = rng.standard_normal((300, 2, 8)); v = rng.standard_normal((300, 2, 8))
    kc, vc = k[:0], v[:0]
    for a, b in [(0, 130), (130, 131), (131, 300)]:       # a window, one token, a ragged rest
        kc, vc = orc.append_cache(kc, vc, k[a:b], v[a:b])
    assert np.array_equal(kc, k) and np.array_equal(vc, v)
    # representatives of a finished block do not change when later tokens arrive
    r1 = orc.representative_keys(k[:140], 128, 4)
    r2 = orc.representative_keys(k, 128, 4)
    assert r1.shape == (1, 4, 2, 8) and r2.shape == (2, 4, 2, 8) and np.array_equal(r1[0], r2[0])


def test_representative_tokens_hand_example_with_tie():
    # norms over both heads: token0 5, token1 5 (tie with token0), token2 1, token3 13, token4 0
    kb = np.zeros((5, 2, 2))
    kb[0, 0] = [3, 0]; kb[0, 1] = [0, 4]
    kb[1, 0] = [0, 5]
    kb[2, 1] = [1, 0]
    kb[3, 0] = [5, 0]; kb[3, 1] = [12, 0]
    assert orc.representative_tokens(kb, 1) == [3]
    assert orc.representative_tokens(kb, 2) == [0, 3]          # the tie goes to the lower position
    assert orc.representative_tokens(kb, 3) == [0, 1, 3]
    assert orc.representative_tokens(kb, 5) == [0, 1, 2, 3, 4]


def test_representative_tokens_against_brute_force_and_torch_recipe():
    import itertools
    import torch
    rng = np.random.default_rng(11)
    kb = rng.standard_normal((9, 2, 4))
    norms = np.sqrt((kb ** 2).sum(axis=(1, 2)))
    for r in (1, 3, 4):
        # the chosen set maximises the sum of norms over all r-subsets (distinct norms: unique)
        best = max(itertools.combinations(range(9), r), key=lambda c: norms[list(c)].sum())
        assert orc.representative_tokens(kb, r) == sorted(best)
    # an independent recipe (torch: norms, stable descending sort, positions back in order) on a few
    # blocks; the ragged tail of 17 tokens has no representatives
    k = torch.randn(3 * 128 + 17, 4, 16, generator=torch.Generator().manual_seed(3))
    kb3 = k[: 3 * 128].reshape(3, 128, 4, 16)
    norm2 = kb3.double().pow(2).sum(dim=(2, 3))                                   # [block][token]
    top = torch.sort(norm2, dim=1, descending=True, stable=True).indices[:, :4]
    pos = torch.sort(top, dim=1).values                                           # position order
    want = torch.stack([kb3[b, pos[b]] for b in range(3)]).numpy()
    got = orc.representative_keys(k.numpy(), 128, 4)
    assert got.shape == want.shape and np.array_equal(got, want)


def test_small_branches_of_the_statistics_and_the_budget():
    # Eq. (12) with nothing to divide by (one eligible block: density ln 1 = 0, and no layer to come):
    # the layer takes the whole remaining budget
    assert orc.layer_budget(0.0, 0.0, 7.25) == 7.25
    assert orc.layer_budget(0.0, 3.0, 7.25) == 0.0            # a zero density beside layers to come: nothing
    # Eq. (8) after a single query: no spread to estimate, the variance is 0 in every channel
    st = orc.RunningStats(3)
    z, s2 = st.update(np.array([[1.0, -2.0, 0.5]]))
    assert np.array_equal(z, [1.0, -2.0, 0.5]) and np.array_equal(s2, [0.0, 0.0, 0.0])
    # Eq. (7): eps is a floor under the variance, max(var, eps), not an added term.  With a
    # variance of eps/4 the divisor is eps; with 4 eps it is 4 eps (var + eps would give 1.25 eps
    # and 5 eps)
    eps = 1e-6
    q, z = np.array([[2.0, 2.0]]), np.zeros(2)
    phi = orc.activation_bias(q, z, np.array([eps / 4, 4 * eps]), eps)
    assert phi[0] == pytest.approx([4.0 / eps, 4.0 / (4 * eps)], rel=1e-12)


# ---------------------------------------------------------------- Eq. (12) across layers and steps
def test_cutoff_history_means_rest_sums_and_budgets():
    rng = np.random.default_rng(5)
    L, T, k = 6, 9, 4.0
    th = rng.uniform(1.0, 6.0, size=(T, L))
    hist = orc.CutoffHistory(L, theta_prior=2.5)
    assert hist.rest_sums() == pytest.approx([2.5 * (L - 1 - l) for l in range(L)])   # no history: the prior
    for t in range(T):
        rest = hist.rest_sums()
        if t > 0:
            mean = th[:t].mean(axis=0)
            want = np.concatenate([np.cumsum(mean[::-1])[::-1][1:], [0.0]])           # suffix sums by numpy
            assert rest == pytest.approx(want, rel=1e-12)
        b = orc.step_budgets(th[t], rest, k)
        assert sum(b) == pytest.approx(L * k, rel=1e-12)      # the last layer takes what is left
        assert all(x > 0 for x in b)
        hist.add_step(th[t])
    assert hist.means() == pytest.approx(th.mean(axis=0), rel=1e-12)


def test_cutoff_constant_density_gives_every_layer_k():
    # equal densities in all layers and steps: B^l = B_kv_left / (L - l) = k for every layer
    L, k = 8, 5.0
    hist = orc.CutoffHistory(L, theta_prior=3.0)
    for _ in range(3):
        b = orc.step_budgets([3.0] * L, hist.rest_sums(), k)
        assert b == pytest.approx([k] * L, rel=1e-12)
        hist.add_step([3.0] * L)


# ---------------------------------------------------------------- tests/golden: hand-worked cases
def _fixture(name):
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        rows = [[float(x) for x in row.split()] for row in val.split(";")]
        out[key.strip()] = np.array(rows if len(rows) > 1 else rows[0])
    return out


def test_golden_fixtures():
    f = _fixture("eq7_9_probe.txt")
    z, s2 = orc.running_stats_literal(f["q"])
    assert np.array_equal(z, f["mean"]) and np.array_equal(s2, f["var"])
    phi = orc.activation_bias(f["q"], z, s2)
    assert np.allclose(phi, f["phi"], rtol=0, atol=1e-15)
    probe, w = orc.probe_query(f["q"], phi)
    assert np.allclose(w, f["weights"], rtol=0, atol=1e-15) and np.allclose(probe, f["probe"], rtol=0, atol=1e-14)
    st = orc.RunningStats(2)                                  # the streaming form gives the same
    z2, s22 = st.update(f["q"])
    assert np.allclose(z2, f["mean"]) and np.allclose(s22, f["var"])

    g = _fixture("eq11_12_cutoff.txt")
    theta = orc.information_density(np.log(g["scores_ln"]))
    assert theta == pytest.approx(float(g["theta_over_ln2"][0]) * math.log(2.0), rel=1e-14)
    budgets = orc.step_budgets(g["densities"], g["rest"], float(g["k"][0]))
    assert budgets == pytest.approx(g["budgets"].tolist(), rel=1e-14)
    b_kv = len(budgets) * float(g["k"][0])
    for th, rest, want in zip(g["densities"], g["rest"], g["budgets"]):
        assert orc.layer_budget(float(th), float(rest), b_kv) == pytest.approx(want, rel=1e-14)
        b_kv -= want
    counts = [orc.cutoff_count(b, int(g["k_cap"][0]), 40) for b in budgets]
    assert counts == [int(c) for c in g["counts"]]
