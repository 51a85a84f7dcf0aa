"""Thin ctypes binding of libactqkv.so: same names as the C ABI, argument
marshalling only.  Tensors are torch tensors on the GPU (torch is used for
device memory and streams, nothing else); every step runs in the library's
kernels.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .synth import LayerShape

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libactqkv.so")

ACTQKV_F32, ACTQKV_BF16 = 0, 1
STATS_UPDATE, PROBE_MEAN_POOLING, PROBE_WINDOW_CHAIN = 1, 2, 4   # bits of build_probe's update_stats
SELECT_ENTROPY_TOPK = 1                                          # bit of select's flags
DECODE_SCORES_ONLY = 2                                           # bit of decode_retrieve's flags
DECODE_NO_WAIT = 4                                               # bit of decode_layer's flags
SELECT_DENSITY_ONLY, SELECT_GIVEN_COUNT = 8, 16                  # bits of select's flags
ERROR_NAMES = {0: "OK", -1: "EINVAL", -2: "ESHAPE", -3: "EALIGN", -4: "EWORKSPACE", -5: "EHIP"}


class ActQKVError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"actqkv error {ERROR_NAMES.get(code, code)}: {message}")
        self.code = code


class CShape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("n_rep", ctypes.c_int32), ("n_init", ctypes.c_int32),
                ("n_local", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("var_eps", ctypes.c_float)]


def c_shape(s: LayerShape, softmax_scale: float = 0.0, var_eps: float = 0.0) -> CShape:
    return CShape(s.n_q_heads, s.n_kv_heads, s.head_dim, s.block_size, s.n_rep, s.n_init,
                  s.n_local, ACTQKV_F32 if s.dtype == "fp32" else ACTQKV_BF16,
                  softmax_scale, var_eps)


_lib = None

_vp, _i, _i64, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
_shp = ctypes.POINTER(CShape)
SIGNATURES = {
    "actqkv_stats_floats": (_sz, [_shp]),
    "actqkv_workspace_bytes": (_sz, [_shp, _i, _i, _i, _i]),
    "actqkv_build_probe": (_i, [_shp, _i, _i, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "actqkv_score_blocks": (_i, [_shp, _i, _vp, _vp, _vp, _i64, _i, _i, _vp, _vp, _i64, _vp]),
    "actqkv_select": (_i, [_i, _vp, _i64, _i, _i, _vp, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "actqkv_retrieval_attention": (_i, [_shp, _i, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _i,
                                        _vp, _vp, _vp, _sz, _vp]),
    "actqkv_retrieval_attention_static": (_i, [_shp, _i, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _i,
                                               _vp, _vp, _vp]),
    "actqkv_retrieval_attention_per_head": (_i, [_shp, _i, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _i,
                                                 _vp, _vp, _vp, _sz, _vp]),
    "actqkv_score_blocks_per_head": (_i, [_shp, _i, _vp, _vp, _i64, _i, _i, _vp, _vp, _i64, _vp]),
    "actqkv_append_kv": (_i, [_shp, _i, _i, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i, _vp]),
    "actqkv_cutoff_budgets": (_i, [_i, _i, ctypes.c_float, _i, _vp, _vp, _vp, _vp, _vp]),
    "actqkv_cutoff_next_step": (_i, [_i, _i, ctypes.c_float, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp]),
    "actqkv_append_kv_probe": (_i, [_shp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i, _vp, _vp, _vp, _vp]),
    "actqkv_decode_retrieve": (_i, [_shp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i, _i, _vp, _vp, _vp,
                                    _vp, _vp, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "actqkv_decode_select_attention": (_i, [_shp, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _i64, _i, _vp, _i, _i,
                                            _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "actqkv_decode_layer": (_i, [_shp, _i, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i, _vp, _i, _vp, _vp, _i64, _i,
                                 _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "actqkv_retrieval_attention_teams": (_i, [_shp, _i, _i, _vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _i,
                                              _vp, _vp, _vp, _sz, _i, _i, _vp, _vp]),
    "actqkv_copy_bytes": (_i, [_vp, _vp, _sz, _vp]),
    "actqkv_gather_blocks": (_i, [_shp, _i, _vp, _vp, _i64, _i, _vp, _vp, _i, _vp, _vp, _i64, _i, _i, _vp, _vp]),
    "actqkv_last_error": (ctypes.c_char_p, []),
    "actqkv_version": (_i, []),
}


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads libactqkv.so (building it first if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("ACTQKV_LIB") or LIB_PATH    # another build of the library, for comparisons
    if path == LIB_PATH and not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from .build import build
        build()
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise ActQKVError(rc, load_library().actqkv_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ActQKVError(-1, "tensor is not on the GPU")
    if not t.is_contiguous():
        raise ActQKVError(-1, "tensor is not contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ActQKVError(-1, f"tensor dtype {t.dtype}, expected {dtype}")
    return t.data_ptr()


_PINNED_STORAGES = {}     # storage address -> is it pinned (asking the runtime costs more than a launch)


def _is_pinned(t: torch.Tensor) -> bool:
    key = t.untyped_storage().data_ptr()
    hit = _PINNED_STORAGES.get(key)
    if hit is None:
        if len(_PINNED_STORAGES) > 4096:
            _PINNED_STORAGES.clear()
        hit = _PINNED_STORAGES[key] = bool(t.is_pinned())
    return hit


def _ptr_readable(t: torch.Tensor, dtype=None) -> int:
    """A tensor a kernel may read in place: device memory or pinned host memory."""
    if not (t.is_cuda or _is_pinned(t)):
        raise ActQKVError(-1, "tensor is neither on the GPU nor in pinned host memory")
    if not t.is_contiguous():
        raise ActQKVError(-1, "tensor is not contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ActQKVError(-1, f"tensor dtype {t.dtype}, expected {dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def version() -> int:
    return load_library().actqkv_version()


def last_error() -> str:
    return load_library().actqkv_last_error().decode()


def stats_floats(shape: CShape) -> int:
    return load_library().actqkv_stats_floats(ctypes.byref(shape))


def workspace_bytes(shape: CShape, batch: int, m: int, nb_capacity: int, k_cap: int) -> int:
    n = load_library().actqkv_workspace_bytes(ctypes.byref(shape), batch, m, nb_capacity, k_cap)
    if n == 0:
        raise ActQKVError(-1, last_error())
    return n


def append_kv(shape: CShape, batch: int, m: int, k_new, v_new, pos0, k_cache, v_cache,
              cache_seq_stride: int, rep_keys, rep_seq_stride: int, nb_capacity: int, stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_append_kv(
        ctypes.byref(shape), batch, m, _ptr(k_new, st), _ptr(v_new, st), _ptr(pos0, torch.int32),
        _ptr(k_cache, st), _ptr(v_cache, st), cache_seq_stride, _ptr(rep_keys, st), rep_seq_stride,
        nb_capacity, _stream(stream)))


def append_kv_probe(shape: CShape, batch: int, q_tok, k_new, v_new, pos0, k_cache, v_cache,
                    cache_seq_stride: int, rep_keys, rep_seq_stride: int, nb_capacity: int, probe, probe_kv,
                    probe_norm, stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    f = torch.float32
    _check(load_library().actqkv_append_kv_probe(
        ctypes.byref(shape), batch, _ptr(q_tok, st), _ptr(k_new, st), _ptr(v_new, st), _ptr(pos0, torch.int32),
        _ptr(k_cache, st), _ptr(v_cache, st), cache_seq_stride, _ptr(rep_keys, st), rep_seq_stride,
        nb_capacity, _ptr(probe, f), _ptr(probe_kv, f), _ptr(probe_norm, f), _stream(stream)))


def decode_retrieve(shape: CShape, batch: int, q_tok, k_new, v_new, pos0, k_cache, v_cache,
                    cache_seq_stride: int, rep_keys, rep_seq_stride: int, nb_capacity: int, nb_begin: int,
                    nb_end, probe, probe_kv, probe_norm, scores, score_stride: int, k_cap: int,
                    budget_remaining, theta_rest_sum, idx, n_sel, theta, budget, stream=None,
                    flags: int = 0) -> None:
    """Cache update, probe, scores and selection of a decode step in one call; see the header."""
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    f, i32 = torch.float32, torch.int32
    _check(load_library().actqkv_decode_retrieve(
        ctypes.byref(shape), batch, _ptr(q_tok, st), _ptr(k_new, st), _ptr(v_new, st), _ptr(pos0, i32),
        _ptr(k_cache, st), _ptr(v_cache, st), cache_seq_stride, _ptr(rep_keys, st), rep_seq_stride,
        nb_capacity, nb_begin, _ptr(nb_end, i32), _ptr(probe, f), _ptr(probe_kv, f), _ptr(probe_norm, f),
        _ptr(scores, f), score_stride, k_cap, int(flags), _ptr(budget_remaining, f), _ptr(theta_rest_sum, f),
        _ptr(idx, i32), _ptr(n_sel, i32), _ptr(theta, f), _ptr(budget, f), _stream(stream)))


def decode_select_attention(shape: CShape, batch: int, q, k_cache, v_cache, seq_stride: int, nb_capacity: int,
                            n_ctx, scores, score_stride: int, nb_begin: int, nb_end, k_cap: int, budget_in,
                            theta_rest_sum, budget_after, idx, n_sel, theta, budget, out, lse, workspace,
                            stream=None, flags: int = 0) -> None:
    """Selection and attention of a decode step in one launch; see the header."""
    st = torch.bfloat16
    f, i32 = torch.float32, torch.int32
    _check(load_library().actqkv_decode_select_attention(
        ctypes.byref(shape), batch, _ptr(q, st), _ptr(k_cache, st), _ptr(v_cache, st), seq_stride, nb_capacity,
        _ptr(n_ctx, i32), _ptr(scores, f), score_stride, nb_begin, _ptr(nb_end, i32), k_cap, int(flags),
        _ptr(budget_in, f), _ptr(theta_rest_sum, f), _ptr(budget_after, f), _ptr(idx, i32), _ptr(n_sel, i32),
        _ptr(theta, f), _ptr(budget, f), _ptr(out, st), _ptr(lse, f), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def decode_layer(shape: CShape, batch: int, q, k_new, v_new, k_cache, v_cache, cache_seq_stride: int,
                 rep_keys, rep_seq_stride: int, nb_capacity: int, n_ctx, nb_begin: int, nb_end, scores,
                 score_stride: int, k_cap: int, budget_in, theta_rest_sum, budget_after, idx, n_sel, theta,
                 budget, out, lse, workspace, stream=None, flags: int = 0) -> None:
    """A whole layer of a decode step in one launch; see the header."""
    st, f, i32 = torch.bfloat16, torch.float32, torch.int32
    _check(load_library().actqkv_decode_layer(
        ctypes.byref(shape), batch, _ptr(q, st), _ptr(k_new, st), _ptr(v_new, st), _ptr(k_cache, st),
        _ptr(v_cache, st), cache_seq_stride, _ptr(rep_keys, st), rep_seq_stride, nb_capacity, _ptr(n_ctx, i32),
        nb_begin, _ptr(nb_end, i32), _ptr(scores, f), score_stride, k_cap, int(flags), _ptr(budget_in, f),
        _ptr(theta_rest_sum, f), _ptr(budget_after, f), _ptr(idx, i32), _ptr(n_sel, i32), _ptr(theta, f),
        _ptr(budget, f), _ptr(out, st), _ptr(lse, f), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def retrieval_attention_static(shape: CShape, batch: int, m: int, q, k_cache, v_cache, seq_stride: int,
                               nb_capacity: int, n_ctx, idx, n_sel, k_cap: int, out, lse, stream=None) -> None:
    """The attention with the library's own scratch array instead of a workspace; see the header."""
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_retrieval_attention_static(
        ctypes.byref(shape), batch, m, _ptr(q, st), _ptr(k_cache, st), _ptr(v_cache, st),
        seq_stride, nb_capacity, _ptr(n_ctx, torch.int32), _ptr(idx, torch.int32),
        _ptr(n_sel, torch.int32), k_cap, _ptr(out, st), _ptr(lse, torch.float32), _stream(stream)))


def retrieval_attention_teams(shape: CShape, batch: int, m: int, q, k_cache, v_cache, seq_stride: int,
                              nb_capacity: int, n_ctx, idx, n_sel, k_cap: int, out, lse, workspace,
                              first_cus: int, late_cus: int, stream=None, stream_late=None) -> None:
    """The attention on first_cus compute units, with an optional second team of late_cus workgroups
    launched on stream_late; see the header."""
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_retrieval_attention_teams(
        ctypes.byref(shape), batch, m, _ptr(q, st), _ptr(k_cache, st), _ptr(v_cache, st),
        seq_stride, nb_capacity, _ptr(n_ctx, torch.int32), _ptr(idx, torch.int32),
        _ptr(n_sel, torch.int32), k_cap, _ptr(out, st), _ptr(lse, torch.float32),
        _ptr(workspace), workspace.numel() * workspace.element_size(), int(first_cus), int(late_cus),
        _stream(stream), _stream(stream_late)))


def cutoff_budgets(batch: int, n_layers: int, k_mean: float, k_cap: int, theta, budget, count, budget_left=None,
                   stream=None) -> None:
    f = torch.float32
    _check(load_library().actqkv_cutoff_budgets(batch, n_layers, k_mean, k_cap, _ptr(theta, f), _ptr(budget, f),
                                                _ptr(count, torch.int32), _ptr(budget_left, f), _stream(stream)))


def cutoff_next_step(batch: int, n_layers: int, k_mean: float, theta_prior: float, theta_prev,
                     theta_sum, n_steps, budget_remaining, theta_rest_sum, stream=None) -> None:
    f = torch.float32
    _check(load_library().actqkv_cutoff_next_step(
        batch, n_layers, k_mean, theta_prior, _ptr(theta_prev, f), _ptr(theta_sum, f), _ptr(n_steps, f),
        _ptr(budget_remaining, f), _ptr(theta_rest_sum, f), _stream(stream)))


def copy_bytes(dst, src, stream=None) -> None:
    """Plain copy of src into dst by one kernel; either may be device memory or pinned host memory."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ActQKVError(-1, "copy_bytes: sizes differ")
    _check(load_library().actqkv_copy_bytes(_ptr_readable(dst), _ptr_readable(src), n, _stream(stream)))


def copy_bytes_at(dst, dst_byte: int, src, src_byte: int, n_bytes: int, stream=None) -> None:
    """copy_bytes between byte offsets of two tensors, without making views of them (a slice costs
    the host about as much as the launch); offsets and length are checked against the tensors."""
    if dst_byte < 0 or src_byte < 0 or n_bytes < 0 or dst_byte + n_bytes > dst.numel() * dst.element_size() \
            or src_byte + n_bytes > src.numel() * src.element_size():
        raise ActQKVError(-1, "copy_bytes_at: range outside a tensor")
    _check(load_library().actqkv_copy_bytes(_ptr_readable(dst) + dst_byte, _ptr_readable(src) + src_byte, n_bytes,
                                            _stream(stream)))


def build_probe(shape: CShape, batch: int, m: int, q_win, stats, update_stats, probe, probe_kv,
                probe_norm, weights, workspace, stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_build_probe(
        ctypes.byref(shape), batch, m, _ptr(q_win, st), _ptr(stats, torch.float32),
        int(update_stats), _ptr(probe, torch.float32), _ptr(probe_kv, torch.float32),
        _ptr(probe_norm, torch.float32), _ptr(weights, torch.float32), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def gather_blocks(shape: CShape, batch: int, k_store, v_store, store_seq_stride: int, nb_store: int,
                  idx, n_sel, k_cap: int, k_cache, v_cache, cache_seq_stride: int, nb_capacity: int,
                  slot0: int, idx_slots, stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_gather_blocks(
        ctypes.byref(shape), batch, _ptr_readable(k_store, st), _ptr_readable(v_store, st),
        store_seq_stride, nb_store, _ptr(idx, torch.int32), _ptr(n_sel, torch.int32), k_cap,
        _ptr(k_cache, st), _ptr(v_cache, st), cache_seq_stride, nb_capacity, slot0,
        _ptr(idx_slots, torch.int32), _stream(stream)))


def score_blocks(shape: CShape, batch: int, probe_kv, probe_norm, rep_keys, seq_stride: int,
                 nb_capacity: int, nb_begin: int, nb_end, scores, score_stride: int,
                 stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_score_blocks(
        ctypes.byref(shape), batch, _ptr(probe_kv, torch.float32), _ptr(probe_norm, torch.float32),
        _ptr(rep_keys, st), seq_stride, nb_capacity, nb_begin, _ptr(nb_end, torch.int32),
        _ptr(scores, torch.float32), score_stride, _stream(stream)))


def score_blocks_per_head(shape: CShape, batch: int, probe, rep_keys, seq_stride: int, nb_capacity: int,
                          nb_begin: int, nb_end, scores, score_stride: int, stream=None) -> None:
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    _check(load_library().actqkv_score_blocks_per_head(
        ctypes.byref(shape), batch, _ptr(probe, torch.float32), _ptr(rep_keys, st), seq_stride, nb_capacity,
        nb_begin, _ptr(nb_end, torch.int32), _ptr(scores, torch.float32), score_stride, _stream(stream)))


def select(batch: int, scores, score_stride: int, nb_capacity: int, nb_begin: int, nb_end,
           k_cap: int, budget_remaining, theta_rest_sum, idx, n_sel, theta=None, budget=None,
           stream=None, flags: int = 0) -> None:
    _check(load_library().actqkv_select(
        batch, _ptr(scores, torch.float32), score_stride, nb_capacity, nb_begin,
        _ptr(nb_end, torch.int32), k_cap, int(flags), _ptr(budget_remaining, torch.float32),
        _ptr(theta_rest_sum, torch.float32), _ptr(idx, torch.int32),
        _ptr(n_sel, torch.int32), _ptr(theta, torch.float32), _ptr(budget, torch.float32),
        _stream(stream)))


def retrieval_attention(shape: CShape, batch: int, m: int, q, k_cache, v_cache, seq_stride: int,
                        nb_capacity: int, n_ctx, idx, n_sel, k_cap: int, out, lse, workspace,
                        stream=None, per_head: bool = False) -> None:
    """per_head: idx [batch][Hk][k_cap], n_sel [batch][Hk] (actqkv_retrieval_attention_per_head)."""
    st = torch.float32 if shape.dtype == ACTQKV_F32 else torch.bfloat16
    lib = load_library()
    _check((lib.actqkv_retrieval_attention_per_head if per_head else lib.actqkv_retrieval_attention)(
        ctypes.byref(shape), batch, m, _ptr(q, st), _ptr(k_cache, st), _ptr(v_cache, st),
        seq_stride, nb_capacity, _ptr(n_ctx, torch.int32), _ptr(idx, torch.int32),
        _ptr(n_sel, torch.int32), k_cap, _ptr(out, st), _ptr(lse, torch.float32),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
