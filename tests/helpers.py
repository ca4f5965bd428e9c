"""Shared helpers of the GPU parity tests: conversions, oracle adapters and the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import slim_oracle as so

# Tolerances of the parity bar -------------------------------------------------------------------
# bf16 outputs vs the oracle: max-abs 2e-2 and mean-abs 2e-3 (attention output, projections of O(1)
# magnitude).  For tensors whose magnitude is well above 1 (the residual stream after the FFN) the
# bf16 rounding of the exact result alone exceeds those numbers, so there the gate is
# max(literal, 1.5 x error of the oracle run with bf16 rounding at every stored tensor).
MAX_ABS, MEAN_ABS = 2e-2, 2e-3
SCORE_GAP = 1e-3           # blocks whose oracle score is within this of the cut may go either way
F32_MAX_ABS = 2e-4         # fp32 workloads: accumulation-order differences only


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def oracle_shape(wl, scoring: str = "unit", placement: str = "before") -> so.LayerShape:
    return so.LayerShape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.block, wl.unit, wl.window,
                         wl.rope_theta, wl.rms_eps, scoring, placement)


def oracle_weights(w: dict, dtype=np.float64) -> so.LayerWeights:
    return so.LayerWeights(**{k: v.detach().cpu().to(torch.float32).numpy().astype(dtype) for k, v in w.items()})


def errs(got: torch.Tensor, want: np.ndarray):
    d = np.abs(f64(got) - want)
    return float(d.max()), float(d.mean())


def assert_selection_matches(kept_gpu: np.ndarray, scores_ref: np.ndarray, n_keep: int, force_first=True,
                             force_last=True, gap=SCORE_GAP):
    """The GPU set must be sorted, unique, of the stated size, contain the forced blocks, and agree
    with the oracle's set on every block whose oracle score is not within `gap` of the cut.
    Returns (oracle set, number of blocks in the ambiguity band, number of differing blocks)."""
    nb = len(scores_ref)
    want = so.select_blocks(scores_ref, n_keep, force_first, force_last)
    assert kept_gpu.dtype == np.int32 and len(kept_gpu) == min(n_keep, nb)
    assert (np.diff(kept_gpu) > 0).all() and kept_gpu.min() >= 0 and kept_gpu.max() < nb
    if force_first:
        assert kept_gpu[0] == 0
    if force_last:
        assert kept_gpu[-1] == nb - 1
    cut = so.selection_cut(scores_ref, n_keep, force_first, force_last)
    diff = set(kept_gpu.tolist()) ^ set(want.tolist())
    band = 0
    if cut is not None:
        amb = np.abs(scores_ref - cut) < gap
        band = int(amb.sum())
        for j in diff:
            assert amb[j], f"block {j} differs but its score {scores_ref[j]} is {abs(scores_ref[j]-cut):.2e} from the cut"
    else:
        assert not diff
    return want, band, len(diff)


def bf16_floor(s, w, x, pos, kept, rows=None):
    """Error of the oracle with bf16 rounding at every stored tensor against the exact oracle, on the
    same kept set: how far any bf16 pipeline is from the exact result.  Returns (z_exact, max, mean)."""
    after = so.layer_after_selection_literal if s.placement == "after" else so.layer_after_selection
    z, _ = after(s, w, x, pos, kept, rows=rows)
    zb, _ = after(s, w, x, pos, kept, rows=rows, rounding="bf16")
    d = np.abs(z - zb)
    return z, float(d.max()), float(d.mean())
