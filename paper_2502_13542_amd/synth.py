"""Seeded synthetic inputs for the retrieval-attention hot path.

This module only *draws inputs* (queries, keys, values, representative keys,
cut-off state).  It contains none of the method's arithmetic: no Activation
Bias, no probe-Query, no scoring, no selection, no attention.  Both the HIP
path and the CPU oracle are fed from here, so that they see identical bits.

The tensors stand in for the query/key/value activations of one LLaMA3-8B
attention layer on the paper's long-context workloads (Sec. 5.1: LongBench,
95 % of sequences within 32K tokens; InfiniteBench, about 122K tokens on
average, up to about 200K).  Only the lengths and the layer shape are taken
from there; the values are random.

Natural layouts produced here (token-major, what the oracle consumes):
    Q  [N][H][D]      K, V  [N][Hk][D]      rep_keys  [NB][r][Hk][D]

Generation is chunked (CHUNK tokens at a time, one generator per chunk), so a
chunk's bits depend only on (seed, tensor, layer, seq, chunk index, device
kind) and memory use stays bounded.  CPU and GPU generators give different
streams: a parity test draws once and hands the *same* tensor to both sides.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import torch

MASTER_SEED = 20250213
CHUNK = 4096

_TENSOR_ID = {"q": 1, "k": 2, "v": 3, "mask_q": 4, "mask_kv": 5, "u": 6,
              "planted": 7, "channels": 8, "cutoff": 9, "decode_q": 10,
              "decode_kv": 11}


@dataclass(frozen=True)
class LayerShape:
    """Shape of one attention layer and of its blocked KV cache."""
    n_q_heads: int          # H
    n_kv_heads: int         # Hk
    head_dim: int           # D
    block_size: int = 128   # Bs, tokens per KV block
    n_rep: int = 4          # r, representative keys per block
    n_init: int = 128       # initial tokens always attended
    n_local: int = 512      # local span before the window, always attended
    dtype: str = "bf16"     # "fp32" | "bf16" (storage; accumulation is fp32)

    @property
    def group(self) -> int:          # G = H / Hk
        return self.n_q_heads // self.n_kv_heads

    @property
    def d_model(self) -> int:        # d = H * D, the paper's hidden size of a query
        return self.n_q_heads * self.head_dim

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


@dataclass(frozen=True)
class Workload:
    name: str
    shape: LayerShape
    n_ctx: int                   # N, context length in tokens
    window: int                  # m
    k_cap: int                   # capacity of the selection ("top-k")
    cutoff: bool                 # dynamic cut-off enabled
    seed: int
    outlier_rate: float = 0.01
    outlier_kind: str = "student_t"   # "boost" (C1) | "student_t" (C2..C5)
    alpha: float = 4.0           # outlier queries get + alpha * u_hat
    shift: float = 0.5           # planted keys get + shift * u
    n_planted: int = 16
    n_layers: int = 1
    batch: int = 1
    decode_steps: int = 0
    e_frac: Tuple[float, float] = (0.05, 0.60)   # cut-off: E / k_cap range

    @property
    def n_windows(self) -> int:
        return (self.n_ctx + self.window - 1) // self.window

    @property
    def n_blocks(self) -> int:
        return (self.n_ctx + self.shape.block_size - 1) // self.shape.block_size


_LLAMA = LayerShape(32, 8, 128, 128, 4, 128, 512, "bf16")

WORKLOADS: Dict[str, Workload] = {
    # configs[0]: small fp32 case, full parity on every window.
    "c1_8k_fp32": Workload("c1_8k_fp32", LayerShape(8, 2, 64, 128, 4, 128, 256, "fp32"),
                           8192, 256, 8, False, MASTER_SEED + 0, outlier_rate=0.02,
                           outlier_kind="boost", n_planted=8),
    # configs[1]: LLaMA3-8B layer, 32K prefill.
    "c2_32k": Workload("c2_32k", _LLAMA, 32768, 512, 16, False, MASTER_SEED + 1),
    # configs[2]: 128K prefill with the dynamic cut-off (the headline metric).
    "c3_128k": Workload("c3_128k", _LLAMA, 131072, 512, 32, True, MASTER_SEED + 2,
                        n_planted=32),
    # configs[3]: decode, 16 sequences x 32 layers x 64K cached tokens.
    "c4_decode": Workload("c4_decode", _LLAMA, 65536, 1, 32, True, MASTER_SEED + 3,
                          n_planted=32, n_layers=32, batch=16, decode_steps=256),
    # configs[4]: 200K-token stream, 32 layers.
    "c5_200k": Workload("c5_200k", _LLAMA, 204800, 512, 32, True, MASTER_SEED + 4,
                        n_planted=32, n_layers=32, outlier_rate=0.0175),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (reduced test sizes)."""
    return dataclasses.replace(w, **kw)


# --------------------------------------------------------------------------
# seeding
# --------------------------------------------------------------------------
def _mix(*vals: int) -> int:
    """64-bit mix of integers into one generator seed (splitmix-style)."""
    x = 0x9E3779B97F4A7C15
    for v in vals:
        x ^= (int(v) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2))
        x &= 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def _gen(device, *vals: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_mix(*vals))
    return g


def direction(w: Workload, layer: int = 0, seq: int = 0, device="cpu") -> torch.Tensor:
    """Seeded unit vector u in R^{Hk*D}, fp32, shape [Hk][D] (always drawn on the CPU)."""
    s = w.shape
    g = _gen("cpu", w.seed, _TENSOR_ID["u"], layer, seq)
    u = torch.randn(s.n_kv_heads, s.head_dim, generator=g, dtype=torch.float32)
    u = u / u.norm()
    return u.to(device)


def planted_blocks(w: Workload, layer: int = 0, seq: int = 0) -> List[int]:
    """Seeded block indices whose keys are shifted toward u.  They lie past the
    initial tokens and early enough to leave the local span during the run."""
    s = w.shape
    lo = s.n_init // s.block_size
    hi = w.n_blocks - (s.n_local + max(w.window, 1)) // s.block_size - 1
    hi = max(hi, lo + 1)
    g = _gen("cpu", w.seed, _TENSOR_ID["planted"], layer, seq)
    n = min(w.n_planted, hi - lo)
    perm = torch.randperm(hi - lo, generator=g)[:n] + lo
    return sorted(int(b) for b in perm)


def boosted_channels(w: Workload, layer: int = 0) -> torch.Tensor:
    """Four fixed channel indices (within a head) that carry activation outliers."""
    g = _gen("cpu", w.seed, _TENSOR_ID["channels"], layer)
    return torch.randperm(w.shape.head_dim, generator=g)[:4].sort().values


def layer_outlier_rate(w: Workload, layer: int) -> float:
    """Per-layer outlier rate; the multi-layer stream spreads 0.5 % .. 3 % over layers."""
    if w.n_layers > 1 and w.name.startswith("c5"):
        return 0.005 + (0.03 - 0.005) * layer / max(w.n_layers - 1, 1)
    return w.outlier_rate


# --------------------------------------------------------------------------
# token tensors
# --------------------------------------------------------------------------
def _student_t3(shape, g, device) -> torch.Tensor:
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    c = torch.randn((3,) + tuple(shape), generator=g, device=device, dtype=torch.float32)
    chi2 = (c * c).sum(0)
    return z / torch.sqrt(chi2 / 3.0)


def gen_q(w: Workload, start: int, count: int, device="cpu", layer: int = 0,
          seq: int = 0) -> torch.Tensor:
    """Queries of tokens [start, start+count): [count][H][D] in the storage dtype.
    start must be a multiple of CHUNK."""
    assert start % CHUNK == 0
    s = w.shape
    u_hat = direction(w, layer, seq, device).repeat_interleave(s.group, dim=0)  # [H][D]
    chans = boosted_channels(w, layer).to(device)
    rate = layer_outlier_rate(w, layer)
    out = []
    for c0 in range(start, start + count, CHUNK):
        n = min(CHUNK, start + count - c0)
        ci = c0 // CHUNK
        g = _gen(device, w.seed, _TENSOR_ID["q"], layer, seq, ci)
        q = torch.randn(CHUNK, s.n_q_heads, s.head_dim, generator=g, device=device,
                        dtype=torch.float32)
        gm = _gen(device, w.seed, _TENSOR_ID["mask_q"], layer, seq, ci)
        mask = torch.rand(CHUNK, generator=gm, device=device) < rate
        if w.outlier_kind == "student_t":
            rows = mask.nonzero().flatten()
            q[rows] = _student_t3((rows.numel(), s.n_q_heads, s.head_dim), gm, device)
        boost = torch.ones(s.head_dim, device=device)
        boost[chans] = 8.0
        if w.outlier_kind == "boost" or w.name.startswith("c5"):
            q = torch.where(mask[:, None, None], q * boost[None, None, :], q)
        q = q + mask[:, None, None].float() * (w.alpha * u_hat)[None]
        out.append(q[:n].to(s.torch_dtype))
    return torch.cat(out, 0) if len(out) > 1 else out[0]


def gen_kv(w: Workload, which: str, start: int, count: int, device="cpu", layer: int = 0,
           seq: int = 0) -> torch.Tensor:
    """Keys ("k") or values ("v") of tokens [start, start+count): [count][Hk][D]."""
    assert which in ("k", "v") and start % CHUNK == 0
    s = w.shape
    u = direction(w, layer, seq, device)
    planted = planted_blocks(w, layer, seq)
    rate = layer_outlier_rate(w, layer) if w.outlier_kind == "student_t" else 0.0
    out = []
    for c0 in range(start, start + count, CHUNK):
        n = min(CHUNK, start + count - c0)
        ci = c0 // CHUNK
        g = _gen(device, w.seed, _TENSOR_ID[which], layer, seq, ci)
        x = torch.randn(CHUNK, s.n_kv_heads, s.head_dim, generator=g, device=device,
                        dtype=torch.float32)
        if rate > 0.0:
            gm = _gen(device, w.seed, _TENSOR_ID["mask_kv"], layer, seq, ci,
                      _TENSOR_ID[which])
            mask = torch.rand(CHUNK, generator=gm, device=device) < rate
            rows = mask.nonzero().flatten()
            x[rows] = _student_t3((rows.numel(), s.n_kv_heads, s.head_dim), gm, device)
        if which == "k":
            for b in planted:
                lo, hi = b * s.block_size - c0, (b + 1) * s.block_size - c0
                lo, hi = max(lo, 0), min(hi, CHUNK)
                if lo < hi:
                    x[lo:hi] += w.shift * u[None]
        out.append(x[:n].to(s.torch_dtype))
    return torch.cat(out, 0) if len(out) > 1 else out[0]


def gen_layer(w: Workload, device="cpu", layer: int = 0, seq: int = 0, n_ctx: Optional[int] = None):
    """(Q, K, V) of one layer of one sequence in the natural layouts."""
    n = w.n_ctx if n_ctx is None else n_ctx
    return (gen_q(w, 0, n, device, layer, seq), gen_kv(w, "k", 0, n, device, layer, seq),
            gen_kv(w, "v", 0, n, device, layer, seq))


# --------------------------------------------------------------------------
# representative keys: the harness rule for synthetic caches
# --------------------------------------------------------------------------
def pick_rep_keys(k: torch.Tensor, block_size: int, n_rep: int) -> torch.Tensor:
    """Representative keys of every *complete* block: [NB][r][Hk][D].

    The paper does not say how a block's representatives are chosen (it takes
    them over from prior block-retrieval work); they are an input of the hot
    path.  The rule used for synthetic caches: the r tokens of the block whose
    key, taken over all KV heads together, has the largest L2 norm (ties: lower
    position), kept in position order.
    """
    n, hk, d = k.shape
    nb = n // block_size
    kb = k[: nb * block_size].reshape(nb, block_size, hk * d)
    norms = kb.float().pow(2).sum(-1)                                  # [NB][Bs]
    order = torch.sort(norms, dim=1, descending=True, stable=True).indices[:, :n_rep]
    order = torch.sort(order, dim=1).values                            # position order
    rep = torch.gather(kb, 1, order[:, :, None].expand(nb, n_rep, hk * d))
    return rep.reshape(nb, n_rep, hk, d).contiguous()


def pick_rep_keys_blocked(kc: torch.Tensor, n_rep: int) -> torch.Tensor:
    """The same rule on a cache in the blocked layout: kc [batch][nb][Hk][Bs][D] ->
    [batch][nb][r][Hk][D] (every block is taken as complete)."""
    bt, nb, hk, bs, d = kc.shape
    norms = kc.float().pow(2).sum(dim=(2, 4))                              # [batch][nb][Bs]
    top = torch.sort(norms, dim=2, descending=True, stable=True).indices[:, :, :n_rep]
    top = torch.sort(top, dim=2).values                                    # position order
    src = kc.permute(0, 1, 3, 2, 4)                                        # [batch][nb][Bs][Hk][D] view
    return torch.gather(src, 2, top[:, :, :, None, None].expand(bt, nb, n_rep, hk, d))


# --------------------------------------------------------------------------
# dynamic cut-off state
# --------------------------------------------------------------------------
def cutoff_state(w: Workload, n_eligible: int, step: int, layer: int = 0, seq: int = 0,
                 n_layers_total: int = 32) -> Tuple[float, float]:
    """Seeded (budget_remaining B_kv, R = sum of the mean densities of the layers
    still to come) for one (step, layer, sequence).

    The values are drawn so that the block count E the cut-off will allow lands
    between e_frac[0]*k_cap and e_frac[1]*k_cap for near-uniform scores, whose
    density is close to ln(n_eligible).  This plays the role of the per-layer
    density profile a full model would supply.
    """
    g = _gen("cpu", w.seed, _TENSOR_ID["cutoff"], step, layer, seq)
    r = torch.rand(3, generator=g, dtype=torch.float64)
    f = w.e_frac[0] + (w.e_frac[1] - w.e_frac[0]) * float(r[0])
    target_e = max(1.0, f * w.k_cap)
    th = math.log(max(n_eligible, 2))
    remaining = max(n_layers_total - 1 - layer, 0)
    rest = remaining * th * (0.8 + 0.4 * float(r[1]))
    budget = target_e * (th + rest) / th + (float(r[2]) - 0.5) * 0.25
    return float(budget), float(rest)


def decode_cutoff_profile(w: Workload, n_eligible: int, step: int = 0) -> Tuple[float, List[float]]:
    """Seeded cut-off inputs of one decode step over all layers: the initial budget B_kv
    and, per layer, R = the summed mean densities of the layers still to come.

    Per-layer target block counts b_l are drawn in e_frac * k_cap; R_l is set so that a
    layer whose density is close to ln(n_eligible) (near-uniform scores) is granted about
    b_l blocks out of what is left: R_l = ln(n_e) * sum_{j>l} b_j / b_l.  This stands in for
    the density profile a full model would have accumulated over earlier steps."""
    g = _gen("cpu", w.seed, _TENSOR_ID["cutoff"], 1 << 20, step)
    r = torch.rand(w.n_layers, generator=g, dtype=torch.float64)
    b = [(w.e_frac[0] + (w.e_frac[1] - w.e_frac[0]) * float(x)) * w.k_cap for x in r]
    th = math.log(max(n_eligible, 2))
    rest = []
    for l in range(w.n_layers):
        tail = sum(b[l + 1:])
        rest.append(th * tail / b[l])
    return float(sum(b)), rest
