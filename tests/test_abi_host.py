"""Host-side checks of the C ABI that need no GPU: the library builds and loads, exports
every symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2502_13542_amd import binding as B
from paper_2502_13542_amd.synth import LayerShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LLAMA = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")


@pytest.fixture(scope="module")
def lib():
    return B.load_library()


def test_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "actqkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(actqkv_[a-z_]+)\s*\(", text))
    assert {"actqkv_build_probe", "actqkv_score_blocks", "actqkv_select",
            "actqkv_retrieval_attention"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in actqkv.h but not exported"
    assert declared == set(B.SIGNATURES), "binding and header disagree"
    assert lib.actqkv_version() == int(re.search(r"#define ACTQKV_VERSION (\d+)", text).group(1))


def test_header_is_plain_c(tmp_path):
    """include/actqkv.h compiles as C99 with warnings on (no C++ or HIP types in the signatures)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "actqkv.h"\nint use(void) { return actqkv_version() > 0 ? ACTQKV_OK : ACTQKV_EINVAL; }\n')
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                          "-c", str(src), "-o", str(tmp_path / "use_header.o")], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.CShape) == 40
    assert B.CShape.softmax_scale.offset == 32 and B.CShape.var_eps.offset == 36


def test_sizes(lib):
    cs = B.c_shape(LLAMA)
    assert B.stats_floats(cs) == 4 + 2 * 4096
    ws = B.workspace_bytes(cs, 1, 512, 1024, 32)
    assert ws >= 4096 and ws % 256 == 0
    assert B.workspace_bytes(cs, 16, 1, 520, 32) >= 4096


A16 = 0x10000  # fake, aligned, never dereferenced: every check below fails before a launch


def _probe(lib, cs, **kw):
    a = dict(batch=1, m=512, q=A16, stats=A16, upd=1, probe=A16, pkv=A16, pn=A16, w=None, ws=A16,
             wsb=1 << 30)
    a.update(kw)
    return lib.actqkv_build_probe(ctypes.byref(cs), a["batch"], a["m"], a["q"], a["stats"], a["upd"],
                                  a["probe"], a["pkv"], a["pn"], a["w"], a["ws"], a["wsb"], None)


def test_workspace_serves_smaller_calls(lib):
    """A workspace sized for (batch, m) is at least what any call with fewer entries or shorter
    windows asks for: few short windows need partial results, many long ones none, and a
    window too long for the matrix-core kernel needs no attention scratch at all."""
    for sh in (LLAMA, LayerShape(8, 2, 128, 128, 4, 128, 256, "bf16"), LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32")):
        cs = B.c_shape(sh)
        for batch, m in ((32, 512), (1, 4096), (4, 2048), (16, 1)):
            big = B.workspace_bytes(cs, batch, m, 1024, 32)
            for b2 in sorted(b for b in {1, 2, batch // 2 or 1, batch} if b <= batch):
                for m2 in sorted(x for x in {1, 77, 128, m // 2 or 1, m} if x <= m):
                    assert B.workspace_bytes(cs, b2, m2, 1024, 32) <= big, (sh, batch, m, b2, m2)


def test_build_probe_rejects(lib):
    cs = B.c_shape(LLAMA)
    assert _probe(lib, cs, batch=0) == -1
    assert _probe(lib, cs, m=0) == -1
    assert _probe(lib, cs, q=None) == -1 and b"q_win" in lib.actqkv_last_error()
    assert _probe(lib, cs, q=A16 + 4) == -3
    assert _probe(lib, cs, ws=None) == -4
    assert _probe(lib, cs, wsb=100) == -4 and b"needs" in lib.actqkv_last_error()
    assert lib.actqkv_build_probe(None, 1, 1, A16, A16, 0, A16, A16, A16, None, A16, 1 << 20, None) == -1
    # consecutive windows of one sequence: need the update bit and m >= 2; unknown bits
    assert _probe(lib, cs, batch=4, upd=B.PROBE_WINDOW_CHAIN) == -1 and b"ACTQKV_STATS_UPDATE" in lib.actqkv_last_error()
    assert _probe(lib, cs, batch=4, m=1, upd=B.PROBE_WINDOW_CHAIN | B.STATS_UPDATE) == -1
    assert _probe(lib, cs, upd=8) == -1 and b"unknown bits" in lib.actqkv_last_error()


@pytest.mark.parametrize("field,value,code", [("head_dim", 96, -2), ("n_kv_heads", 5, -2),
                                              ("block_size", 64, -2), ("n_rep", 17, -2),
                                              ("n_init", 100, -2), ("dtype", 7, -1),
                                              ("n_q_heads", 0, -1), ("softmax_scale", -1.0, -1)])
def test_shape_rejects(lib, field, value, code):
    cs = B.c_shape(LLAMA)
    setattr(cs, field, value)
    assert _probe(lib, cs) == code
    assert B.stats_floats(cs) == 0


def test_score_select_attention_reject(lib):
    cs = B.c_shape(LLAMA)
    sb = lambda **k: lib.actqkv_score_blocks(ctypes.byref(cs), k.get("batch", 1), A16, A16,
                                             k.get("rep", A16), k.get("stride", 0), k.get("cap", 64), 1,
                                             A16, A16, k.get("ss", 64), None)
    assert sb(rep=None) == -1 and sb(rep=A16 + 8) == -3 and sb(ss=10) == -1 and sb(cap=-1) == -1
    assert sb(batch=2, stride=8) == -1 and sb(stride=4) == -3 and sb(cap=9000, ss=9000) == -2
    se = lambda **k: lib.actqkv_select(1, A16, 64, 64, 1, A16, k.get("k_cap", 32), k.get("flags", 0),
                                       k.get("bud"), k.get("rest"), k.get("idx", A16), A16, None, None, None)
    assert se(k_cap=0) == -2 and se(k_cap=65) == -2 and se(idx=None) == -1 and se(flags=2) == -1
    assert se(bud=A16 + 2, rest=A16) == -3 and se(bud=A16) == -1 and se(rest=A16) == -1
    at = lambda **k: lib.actqkv_retrieval_attention(ctypes.byref(cs), 1, k.get("m", 512), A16,
                                                    k.get("kc", A16), A16, 0, k.get("cap", 64), A16, A16,
                                                    A16, 32, k.get("out", A16), None, k.get("ws", A16),
                                                    k.get("wsb", 1 << 30), None)
    assert at(kc=None) == -1 and at(out=A16 + 2) == -3 and at(ws=None) == -4 and at(wsb=8) == -4
    assert at(m=0) == -1 and at(cap=2) == -1 and at(cap=0) == -1
    sp = lambda **k: lib.actqkv_score_blocks_per_head(ctypes.byref(cs), 1, k.get("probe", A16), k.get("rep", A16), 0,
                                                      k.get("cap", 64), 1, A16, A16, k.get("ss", 64), None)
    assert sp(probe=None) == -1 and sp(rep=A16 + 8) == -3 and sp(ss=10) == -1 and sp(cap=9000, ss=9000) == -2
    assert lib.actqkv_retrieval_attention_per_head(ctypes.byref(cs), 1, 512, A16, None, A16, 0, 64, A16, A16, A16, 32,
                                                   A16, None, A16, 1 << 30, None) == -1
    ap = lambda **k: lib.actqkv_append_kv_probe(ctypes.byref(cs), 1, k.get("q", A16), A16, A16, A16, A16, A16, 0, None,
                                                0, k.get("cap", 64), k.get("probe", A16), A16, A16, None)
    assert ap(q=None) == -1 and b"q_tok" in lib.actqkv_last_error() and ap(probe=None) == -1
    assert ap(cap=0) == -1 and ap(q=A16 + 2) == -3
    ga = lambda **k: lib.actqkv_gather_blocks(ctypes.byref(cs), 1, k.get("ks", A16), A16, 0, k.get("nbs", 64), A16,
                                              A16, k.get("k_cap", 32), k.get("kc", A16), A16, 0, k.get("cap", 64),
                                              k.get("slot0", 1), None, None)
    assert ga(ks=None) == -1 and ga(kc=A16 + 4) == -3 and ga(k_cap=65) == -2 and ga(nbs=0) == -1
    assert ga(slot0=40) == -1 and b"outside the cache" in lib.actqkv_last_error() and ga(slot0=-1) == -1
    with pytest.raises(B.ActQKVError):
        B._check(at(wsb=8))


def test_workspace_serves_every_launch_shape(lib):
    """The launch shape is an argument of the attention call, not process-wide state: a workspace
    of actqkv_workspace_bytes is accepted with every first_cus (the host checks run up to the
    launch, which fails without a GPU: any code but EWORKSPACE and the argument errors)."""
    cs = B.c_shape(LLAMA)
    for batch, m in ((1, 512), (2, 512), (32, 512), (1, 96)):
        full = B.workspace_bytes(cs, batch, m, 1024, 32)
        for cus in (1, 8, 64, 192, 224, 256):
            rc = lib.actqkv_retrieval_attention_teams(
                ctypes.byref(cs), batch, m, A16, A16, A16, 0, 1024, A16, A16, A16, 32, A16, None, A16, full,
                cus, 0, None, None)
            assert rc in (0, -5), (batch, m, cus, B.last_error())


def test_attention_cache_larger_than_a_selection(lib):
    """The attention selects nothing, so the 8192-block limit of one selection does not apply to
    its cache; the calls that select keep it."""
    cs = B.c_shape(LLAMA)
    att = lambda nb: lib.actqkv_retrieval_attention(
        ctypes.byref(cs), 1, 512, A16, A16, A16, 0, nb, A16, A16, A16, 32, A16, None, A16, 1 << 30, None)
    assert att(8193) in (0, -5) and att(1 << 20) in (0, -5)
    assert att((1 << 23) + 1) == -2 and b"2^30" in lib.actqkv_last_error()
    sel = lambda nb: lib.actqkv_select(1, A16, nb, nb, 0, A16, 32, 0, None, None, A16, A16, None, None, None)
    assert sel(8193) == -2 and b"8192" in lib.actqkv_last_error()


def test_copy_bytes_rejects(lib):
    assert lib.actqkv_copy_bytes(None, A16, 1024, None) == -1
    assert lib.actqkv_copy_bytes(A16, None, 1024, None) == -1
    assert lib.actqkv_copy_bytes(A16, A16 + 4096, 1000, None) == -1      # not a multiple of 16
    assert lib.actqkv_copy_bytes(A16 + 4, A16 + 4096, 1024, None) == -3  # alignment
    assert lib.actqkv_copy_bytes(A16, A16 + 4096, 0, None) == 0          # nothing to do, nothing launched


def test_append_kv_rejects(lib):
    cs = B.c_shape(LLAMA)
    call = lambda **kw: lib.actqkv_append_kv(ctypes.byref(cs), kw.get("batch", 1), kw.get("m", 512),
                                             kw.get("k", A16), kw.get("v", A16), kw.get("pos0", A16),
                                             kw.get("kc", A16), kw.get("vc", A16), kw.get("cs", 0),
                                             kw.get("rep", A16), kw.get("rs", 0), kw.get("nb", 8), None)
    assert call(m=0) == -1 and call(batch=0) == -1 and call(nb=0) == -1
    assert call(k=None) == -1 and call(pos0=None) == -1 and call(vc=None) == -1
    assert call(k=A16 + 2) == -3 and call(cs=12) == -3
    assert call(batch=2, cs=8) == -1                       # stride smaller than one sequence's cache


def test_decode_retrieve_rejects(lib):
    cs = B.c_shape(LLAMA)
    call = lambda **k: lib.actqkv_decode_retrieve(
        ctypes.byref(cs), k.get("batch", 1), k.get("q", A16), k.get("kn", A16), k.get("vn", A16),
        k.get("pos0", A16), k.get("kc", A16), A16, k.get("cs", 0), k.get("rep", A16), k.get("rs", 0),
        k.get("cap", 64), 1, k.get("nb_end", A16), None, None, None, k.get("scores", A16), k.get("ss", 64),
        k.get("k_cap", 32), k.get("flags", 0), k.get("bud"), k.get("rest"), k.get("idx", A16), A16, None, None, None)
    assert call(q=None) == -1 and b"q_tok" in lib.actqkv_last_error() and call(q=A16 + 2) == -3
    assert call(kn=None) == -1 and call(pos0=None) == -1 and call(kc=None) == -1     # a partial cache update
    assert call(rep=None) == -1 and call(nb_end=None) == -1 and call(scores=None) == -1 and call(idx=None) == -1
    assert call(cap=0) == -1 and call(cap=9000, ss=9000) == -2 and call(ss=10) == -1
    assert call(k_cap=0) == -2 and call(k_cap=65) == -2 and call(flags=4) == -1
    assert call(bud=A16) == -1 and call(bud=A16 + 2, rest=A16) == -3
    assert call(batch=2, cs=8) == -1 and call(batch=2, cs=1 << 40, rs=8) == -1 and call(cs=12) == -3


def test_decode_select_attention_rejects(lib):
    cs = B.c_shape(LLAMA)
    call = lambda **k: lib.actqkv_decode_select_attention(
        ctypes.byref(k.get("shape", cs)), k.get("batch", 1), k.get("q", A16), k.get("kc", A16), A16, k.get("stride", 0),
        k.get("cap", 64), k.get("n_ctx", A16), k.get("scores", A16), k.get("ss", 64), 1, k.get("nb_end", A16),
        k.get("k_cap", 32), k.get("flags", 0), k.get("bud"), k.get("rest"), k.get("after"), k.get("idx", A16),
        k.get("n_sel", A16), None, None, k.get("out", A16), None, k.get("ws", A16), k.get("wsb", 1 << 30), None)
    assert call(q=None) == -1 and call(kc=A16 + 2) == -3 and call(scores=None) == -1 and call(out=None) == -1
    assert call(idx=None) == -1 and call(n_sel=None) == -1 and call(n_ctx=None) == -1 and call(nb_end=None) == -1
    assert call(cap=0) == -1 and call(ss=10) == -1 and call(k_cap=65) == -2 and call(flags=2) == -1
    assert call(bud=A16) == -1 and call(bud=A16, rest=A16, after=A16) == -1     # in place is not allowed
    assert b"budget_after" in lib.actqkv_last_error()
    assert call(batch=2, stride=8) == -1 and call(stride=4) == -3
    assert call(ws=None) == -4 and call(wsb=8) == -4
    fp32 = B.c_shape(LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32"))
    assert call(shape=fp32) == -2                                               # a bf16, head_dim 128 kernel


def test_decode_layer_rejects(lib):
    """The whole decode layer in one launch: everything is refused on the host before a kernel runs."""
    cs = B.c_shape(LLAMA)
    call = lambda **k: lib.actqkv_decode_layer(
        ctypes.byref(k.get("shape", cs)), k.get("batch", 1), k.get("q", A16), k.get("kn", A16), k.get("vn", A16),
        k.get("kc", A16), A16, k.get("cs", 0), k.get("rep", A16), k.get("rs", 0), k.get("cap", 64),
        k.get("n_ctx", A16), 1, k.get("nb_end", A16), k.get("scores", A16), k.get("ss", 64), k.get("k_cap", 32),
        k.get("flags", 0), k.get("bud"), k.get("rest"), k.get("after"), k.get("idx", A16), k.get("n_sel", A16),
        None, None, k.get("out", A16), None, k.get("ws", A16), k.get("wsb", 1 << 30), None)
    assert call(q=None) == -1 and call(kn=None) == -1 and b"together" in lib.actqkv_last_error()
    assert call(kc=None) == -1 and call(rep=None) == -1 and call(kc=A16 + 2) == -3
    assert call(n_ctx=None) == -1 and call(nb_end=None) == -1 and call(scores=None) == -1
    assert call(idx=None) == -1 and call(n_sel=None) == -1 and call(out=None) == -1
    assert call(cap=0) == -1 and call(cap=9000, ss=9000) == -2 and call(ss=10) == -1
    assert call(k_cap=0) == -2 and call(k_cap=65) == -2
    assert call(flags=2) == -1 and call(flags=8) == -1 and b"unknown flag" in lib.actqkv_last_error()
    assert call(bud=A16) == -1 and call(bud=A16, rest=A16, after=A16) == -1
    assert b"budget_after" in lib.actqkv_last_error()
    assert call(batch=385) == -2 and b"batch" in lib.actqkv_last_error()
    assert call(batch=2, cs=8) == -1 and call(batch=2, cs=1 << 40, rs=8) == -1 and call(cs=12) == -3
    assert call(ws=None) == -4 and call(wsb=8) == -4
    fp32 = B.c_shape(LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32"))
    assert call(shape=fp32) == -2


def test_blocked_representatives_equal_the_token_major_rule():
    """The harness rule for the representative keys of a synthetic cache, on a blocked cache and on
    token-major keys: the same keys (it is an input recipe; the oracle's rule is pinned on its own)."""
    import torch
    from paper_2502_13542_amd import synth
    g = torch.Generator().manual_seed(5)
    k = torch.randn(3 * 128, 2, 16, generator=g)
    k[130] = k[131]                                       # a tie: the earlier position wins
    blocked = k.reshape(3, 128, 2, 16).permute(0, 2, 1, 3)[None].contiguous()
    assert torch.equal(synth.pick_rep_keys(k, 128, 4), synth.pick_rep_keys_blocked(blocked, 4)[0])


def test_retrieval_attention_teams_rejects(lib):
    cs = B.c_shape(LLAMA)
    call = lambda **k: lib.actqkv_retrieval_attention_teams(
        ctypes.byref(cs), 32, 512, k.get("q", A16), A16, A16, 0, 1024, A16, A16, A16, 32, k.get("out", A16), None,
        k.get("ws", A16), k.get("wsb", 1 << 30), k.get("first_cus", 224), k.get("late_cus", 32), None, None)
    assert call(late_cus=4) == -1 and call(late_cus=300) == -1 and call(late_cus=-1) == -1
    assert b"late_cus" in lib.actqkv_last_error()
    assert call(first_cus=0) == -1 and call(first_cus=257) == -1 and b"first_cus" in lib.actqkv_last_error()
    assert call(q=None) == -1 and call(out=A16 + 2) == -3 and call(ws=None) == -4 and call(wsb=8) == -4


def test_retrieval_attention_static_rejects(lib):
    """The entry point that allocates nothing: argument errors as in actqkv_retrieval_attention, and
    a call whose scratch need exceeds the library's own array is refused before anything runs."""
    cs = B.c_shape(LLAMA)
    call = lambda shape=cs, batch=1, m=512, **k: lib.actqkv_retrieval_attention_static(
        ctypes.byref(shape), batch, m, k.get("q", A16), A16, A16, 0, k.get("nb", 1024), A16, A16, A16,
        k.get("k_cap", 32), k.get("out", A16), None, None)
    assert call(q=None) == -1 and call(out=A16 + 2) == -3 and call(k_cap=65) == -2 and call(m=0) == -1
    big = B.c_shape(LayerShape(128, 16, 128, 128, 4, 128, 512, "bf16"))
    assert call(shape=big, batch=1024, m=1, nb=2) == -4
    msg = lib.actqkv_last_error().decode()
    assert "scratch" in msg and str(32 << 20) in msg


def test_cutoff_budgets_and_select_modes_reject(lib):
    f = ctypes.c_float
    call = lambda batch=2, L=32, k=8.0, cap=32, th=A16, b=A16, c=A16, left=None: \
        lib.actqkv_cutoff_budgets(batch, L, f(k), cap, th, b, c, left, None)
    assert call(batch=0) == -1 and call(k=0.0) == -1 and call(L=0) == -2 and call(L=2000) == -2
    assert call(cap=0) == -2 and call(cap=65) == -2
    assert call(th=None) == -1 and call(b=None) == -1 and call(c=A16 + 2) == -3 and call(left=A16 + 1) == -3
    sel = lambda flags, theta=A16, bud=None, rest=None: lib.actqkv_select(
        1, A16, 64, 64, 0, A16, 8, flags, bud, rest, A16, A16, theta, None, None)
    assert sel(B.SELECT_DENSITY_ONLY | B.SELECT_GIVEN_COUNT) == -1 and b"exclude" in lib.actqkv_last_error()
    assert sel(B.SELECT_DENSITY_ONLY, theta=None) == -1 and b"theta" in lib.actqkv_last_error()
    assert sel(B.SELECT_GIVEN_COUNT, bud=A16, rest=A16) == -1 and b"cut-off state" in lib.actqkv_last_error()
    assert sel(32) == -1 and b"unknown flag" in lib.actqkv_last_error()


def test_cutoff_next_step_rejects(lib):
    f = ctypes.c_float
    call = lambda batch=2, L=32, k=8.0, prior=6.0, prev=A16, ts=A16, ns=A16, b=A16, r=A16: \
        lib.actqkv_cutoff_next_step(batch, L, f(k), f(prior), prev, ts, ns, b, r, None)
    assert call(batch=0) == -1 and call(k=0.0) == -1 and call(prior=-1.0) == -1
    assert call(L=0) == -2 and call(L=2000) == -2
    assert call(ts=None) == -1 and call(b=None) == -1 and call(r=A16 + 2) == -3
