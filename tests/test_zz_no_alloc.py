"""The attention entry point that allocates nothing (actqkv_retrieval_attention_static: the
library's own scratch array instead of a caller's workspace) against
actqkv_retrieval_attention on the same inputs, through the C ABI.  The two run the same
kernels in the same launch shape, so their outputs must be identical bit for bit (which is
within every tolerance of the parity tests); the existing entry point itself is checked
against the oracle on sampled rows.  Every case is a pair of calls in a row on the shared
array, the second with a smaller input, and uses scratch memory: a single prefill window is cut
into pieces with partial results, a decode sequence is split over several workgroups."""
import numpy as np
import pytest
import torch

from oracle import actqkv_oracle as orc
from paper_2502_13542_amd import binding as B
from paper_2502_13542_amd import harness as H
from paper_2502_13542_amd.synth import LayerShape

from parity_utils import TOL_OUT, f64, out_error

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(sh, bt, m, nb, k_cap, seed, lse=False):
    td = torch.bfloat16 if sh.dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(seed)
    rng = np.random.default_rng(seed)
    ks = [torch.randn(nb * 128, sh.n_kv_heads, sh.head_dim, generator=g).to(td) for _ in range(bt)]
    vs = [torch.randn(nb * 128, sh.n_kv_heads, sh.head_dim, generator=g).to(td) for _ in range(bt)]
    kc = torch.stack([H.blocked_k(x.to(DEV), sh, nb) for x in ks])
    vc = torch.stack([H.blocked_vt(x.to(DEV), sh, nb) for x in vs])
    q = torch.randn(bt, m, sh.n_q_heads, sh.head_dim, generator=g).to(td)
    n_ctx = [int(rng.integers(max(m, nb * 64), nb * 128 + 1)) for _ in range(bt)]
    idx = torch.full((bt, k_cap), -1, dtype=torch.int32)
    n_sel = torch.zeros(bt, dtype=torch.int32)
    chosen = []
    for s in range(bt):
        b, e = H.eligible_range(sh, n_ctx[s] - m)
        cnt = int(rng.integers(1, min(k_cap, max(e - b, 1)) + 1)) if e > b else 0
        pick = (rng.permutation(max(e - b, 0))[:cnt] + b).tolist()
        idx[s, :cnt] = torch.tensor(pick, dtype=torch.int32)
        n_sel[s] = cnt
        chosen.append(pick)
    return dict(sh=sh, cs=B.c_shape(sh), bt=bt, m=m, nb=nb, k_cap=k_cap, ks=ks, vs=vs, kc=kc, vc=vc, q=q,
                qd=q.to(DEV), n_ctx=n_ctx, n_ctx_d=torch.tensor(n_ctx, dtype=torch.int32, device=DEV),
                idx=idx.to(DEV), n_sel=n_sel.to(DEV), chosen=chosen, lse=lse)


def _run_both(c):
    sh, cs, bt, m, nb, k_cap = c["sh"], c["cs"], c["bt"], c["m"], c["nb"], c["k_cap"]
    shape_out = (bt, m, sh.n_q_heads, sh.head_dim)
    ref = torch.zeros(shape_out, dtype=c["qd"].dtype, device=DEV)
    got = torch.full(shape_out, 7.0, dtype=c["qd"].dtype, device=DEV)
    lse_ref = torch.zeros(bt, sh.n_q_heads, m, device=DEV) if c["lse"] else None
    lse_got = torch.ones(bt, sh.n_q_heads, m, device=DEV) if c["lse"] else None
    ws = torch.zeros(B.workspace_bytes(cs, bt, m, nb, k_cap), dtype=torch.uint8, device=DEV)
    assert ws.numel() > 8192, "the case must use scratch memory beyond the counters"
    B.retrieval_attention(cs, bt, m, c["qd"], c["kc"], c["vc"], c["kc"].stride(0), nb, c["n_ctx_d"], c["idx"],
                          c["n_sel"], k_cap, ref, lse_ref, ws)
    B.retrieval_attention_static(cs, bt, m, c["qd"], c["kc"], c["vc"], c["kc"].stride(0), nb, c["n_ctx_d"],
                                 c["idx"], c["n_sel"], k_cap, got, lse_got)
    torch.cuda.synchronize()
    assert torch.equal(got, ref), "the static-scratch call differs from the workspace call"
    if c["lse"]:
        assert torch.equal(lse_got, lse_ref)
    # and the reference call itself against the oracle, on sampled rows
    group = sh.n_q_heads // sh.n_kv_heads
    for s in range(bt):
        w0 = c["n_ctx"][s] - m
        for r in sorted({0, m // 2, m - 1}):
            pos = orc.key_positions(w0, w0 + r, c["chosen"][s], sh.n_init, sh.n_local, 128)
            want = orc.attention_rows(f64(c["q"][s, r])[None], f64(c["ks"][s]), f64(c["vs"][s]), pos, group)[0]
            err = out_error(got[s, r], want)
            assert err < TOL_OUT[sh.dtype], (s, r, err)


def test_static_scratch_attention_equals_the_workspace_call():
    llama = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")
    small = LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16")
    print("prefill window, 512 then 200 tokens", flush=True)
    _run_both(_case(llama, 1, 512, 40, 8, 101))          # 4 pieces per query tile: partial results
    _run_both(_case(llama, 1, 200, 24, 4, 102, lse=True))
    print("decode batch, 6 then 2 sequences", flush=True)
    _run_both(_case(llama, 6, 1, 48, 16, 103, lse=True))  # several workgroups per (sequence, KV head)
    _run_both(_case(small, 2, 1, 20, 4, 104))
    print("batch of windows (queue counters), 12 then 3", flush=True)
    _run_both(_case(small, 12, 256, 30, 6, 105))
    _run_both(_case(small, 3, 128, 12, 2, 106))
    print("fp32 rows (no scratch used by the kernel), after the others", flush=True)
    c = _case(LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32"), 2, 96, 10, 4, 107)
    sh, cs = c["sh"], c["cs"]
    ref = torch.zeros(2, 96, 8, 64, device=DEV)
    got = torch.zeros_like(ref)
    ws = torch.zeros(B.workspace_bytes(cs, 2, 96, 10, 4), dtype=torch.uint8, device=DEV)
    B.retrieval_attention(cs, 2, 96, c["qd"], c["kc"], c["vc"], c["kc"].stride(0), 10, c["n_ctx_d"], c["idx"],
                          c["n_sel"], 4, ref, None, ws)
    B.retrieval_attention_static(cs, 2, 96, c["qd"], c["kc"], c["vc"], c["kc"].stride(0), 10, c["n_ctx_d"],
                                 c["idx"], c["n_sel"], 4, got, None)
    torch.cuda.synchronize()
    assert torch.equal(got, ref)


def test_static_scratch_attention_refuses_what_does_not_fit():
    # 128 query heads, 1024 sequences: the partial results of the decode step exceed the array
    big = LayerShape(128, 16, 128, 128, 4, 128, 512, "bf16")
    cs = B.c_shape(big)
    q = torch.zeros(1024, 1, 128, 128, dtype=torch.bfloat16, device=DEV)
    kc = torch.zeros(1, 2, 16, 128, 128, dtype=torch.bfloat16, device=DEV)
    n = torch.full((1024,), 200, dtype=torch.int32, device=DEV)
    idx = torch.full((1024, 4), -1, dtype=torch.int32, device=DEV)
    out = torch.zeros_like(q)
    with pytest.raises(B.ActQKVError) as e:
        B.retrieval_attention_static(cs, 1024, 1, q, kc, kc, 0, 2, n, idx, n, 4, out, None)
    assert e.value.code == -4 and "scratch" in str(e.value)
