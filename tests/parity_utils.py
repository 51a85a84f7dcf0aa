"""Helpers shared by the GPU parity tests: widening to fp64, the comparison
rules and their tolerances.  Nothing here computes the method; the expected
values always come from oracle/."""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import actqkv_oracle as orc
from paper_2502_13542_amd.synth import LayerShape

# Tolerances.  The kernels accumulate in fp32; the oracle in fp64 on the same stored bits.
TOL_PROBE = 2e-4      # relative to the largest |probe| entry (fp32 running statistics, m terms)
TOL_WEIGHT = 5e-4     # relative to the largest weight
TOL_SCORE = 2e-5      # absolute; scores are cosines in [-1, 1], sums of <= 16K fp32 products
TOL_THETA = 2e-4      # absolute; theta <= ln(8192) ~ 9
TOL_BUDGET = 5e-4     # relative
TOL_OUT = {"fp32": 1e-4, "bf16": 2e-2}   # max over rows of max|diff| / max|ref| (the benchmark spec)
GAP_EXACT = 1e-3      # indices must match exactly when neighbouring scores differ by more


def f64(t) -> np.ndarray:
    if isinstance(t, torch.Tensor):
        return t.detach().float().cpu().numpy().astype(np.float64)
    return np.asarray(t, dtype=np.float64)


def rel_to_max(got, want) -> float:
    got, want = f64(got), f64(want)
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


def out_error(got, want) -> float:
    """max over query rows (and heads) of max_d |got - want| / max_d |want|."""
    got, want = f64(got), f64(want)
    num = np.abs(got - want).max(axis=-1)
    den = np.maximum(np.abs(want).max(axis=-1), 1e-30)
    return float((num / den).max())


def check_selection(gpu_idx: Sequence[int], gpu_count: int, res: Dict, k_cap: int,
                    tol: float = TOL_SCORE) -> bool:
    """Compares a selection from the GPU with the oracle's result `res` for the same
    probe.  Returns True when the lists are identical.  Identity is required whenever the
    scores around the cut are further apart than GAP_EXACT; otherwise the GPU's list must
    be a correct selection under scores perturbed by at most tol (near-ties may swap)."""
    elig, s = res["eligible"], res["scores"]
    gpu = [int(x) for x in gpu_idx[:gpu_count]]
    assert all(int(x) == -1 for x in gpu_idx[gpu_count:]), "unused index slots must be -1"
    assert gpu_count == len(gpu)
    if not elig:
        assert gpu_count == 0
        return True
    count = res["count"]
    # E: the rounding of B^l is taken in fp32 on the GPU; a budget within 1e-3 of a
    # half-integer may round either way
    frac = res["budget"] + 0.5 - math.floor(res["budget"] + 0.5)
    near_half = min(frac, 1.0 - frac) < 1e-3
    if not near_half:
        assert gpu_count == count, (gpu_count, count, res["budget"])
    else:
        assert abs(gpu_count - count) <= 1
    if gpu == res["idx"]:
        return True
    score_of = {b: float(v) for b, v in zip(elig, s)}
    assert len(set(gpu)) == len(gpu) and all(b in score_of for b in gpu), "not a set of eligible blocks"
    order = np.sort(s)[::-1]
    top = order[: max(count, gpu_count) + 1]
    gaps = -np.diff(top) if len(top) > 1 else np.array([1.0])
    assert gaps.min() <= GAP_EXACT, f"selection differs although all gaps exceed {GAP_EXACT}: {gpu} vs {res['idx']}"
    got = np.array([score_of[b] for b in gpu])
    assert (np.diff(got) <= tol).all(), "selection is not sorted by score"
    if gpu_count:
        kth = order[gpu_count - 1]
        assert got.min() >= kth - tol, "a selected block scores below the cut"
    return False


def oracle_windows(q, k, v, rep, shape: LayerShape, m: int, k_cap: int, cutoffs=None,
                   attend: Optional[Sequence[int]] = None) -> List[Dict]:
    """The oracle's prefill over CPU copies of the tensors."""
    f32 = lambda t: t.detach().float().cpu().numpy()   # exact for bf16 and fp32; widened per window
    return orc.prefill_layer(f32(q), f32(k), f32(v), f64(rep), m, shape.n_init, shape.n_local,
                             shape.block_size, k_cap, cutoffs, attend)
