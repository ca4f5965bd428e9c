"""Shared helpers of the GPU parity tests: conversions, oracle adapters and the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import slim_oracle as so

# Tolerances of the parity bar -------------------------------------------------------------------
# bf16 outputs vs the oracle: max-abs 2e-2 and mean-abs 2e-3 (attention output, projections of O(1)
# magnitude).  The residual stream is stored in bf16 twice on the way to the layer output (y = x' + Wo.o,
# then z = y + FFN(y)), and a value v stored in bf16 is off by up to half a unit in its last place,
# ulp(v) = 2^(floor(log2 |v|) - 7): 0.03 for |v| in [8, 16).  So the stated numbers are applied to everything
# but those two stores, and each store is allowed its half ulp, element by element, at the magnitude the
# exact oracle gives that element (assert_residual_close).  No rounding emulation is involved.
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


def ulp_bf16(a: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 numbers at the magnitude of each element of a (8 significant bits)."""
    m = np.maximum(np.abs(np.asarray(a, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(m)) - 7)


TAIL_FRACTION, TAIL_FACTOR = 2e-5, 1.3


def ffn_response_sigma(y_ref: np.ndarray, z_ref: np.ndarray, dy: np.ndarray | None = None, input_roundings: int = 0) -> np.ndarray:
    """Per row: the standard deviation of what a small random change of the FFN's input does to the FFN branch.
    The branch f = z - y reads the normalised row r = y / rms(y) and answers a small random change of r about as
    it answers r itself, with gain rms(f) / rms(r) = rms(f); a change e of the row y changes r by e / rms(y).
    Two such changes are counted: dy, the deviation of the GPU's y from the oracle's (itself held to its own bound;
    the normalisation amplifies it where the residual is small), and input_roundings further bf16 roundings of the
    FFN's input (the normalised row, when it is stored), each an error uniform over ulp(y_i) in element i.
    y_ref, z_ref come from the exact oracle."""
    f = z_ref - y_ref
    rms = lambda a: np.sqrt(np.mean(a * a, axis=1))
    var = input_roundings * np.mean(ulp_bf16(y_ref) ** 2, axis=1) / 12.0
    if dy is not None:
        var = var + np.mean(dy * dy, axis=1)
    return rms(f) * np.sqrt(var) / rms(y_ref)


def assert_residual_close(got, want: np.ndarray, stores: list, label: str = "", ffn_sigma=None):
    """got: a bf16 tensor of the residual stream; want: the exact oracle's value of it; stores: the exact
    oracle's values of every bf16-stored residual tensor whose rounding reaches `got` one to one (the tensor
    itself, and for z also y); ffn_sigma: per row, the standard deviation of the FFN branch's answer to the
    roundings of its input (ffn_response_sigma times the square root of their number), for z only.
    Element by element the bound is b = 2e-2 + half an ulp of each store + 5 ffn_sigma.  What the 2e-2 covers is a
    sum of thousands of independent roundings (Key/Query/Value states, probabilities, attention output, activations),
    close to Gaussian with a standard deviation of 3e-3 to 6e-3 at these shapes, so among 10^7 elements a few lie
    beyond any fixed multiple of it: at most TAIL_FRACTION of the elements may exceed b, none may exceed
    TAIL_FACTOR * b.  The mean: <= 2e-3 + the mean quarter ulp of each store (the expected size of a rounding error
    uniform over one ulp) + 0.8 ffn_sigma (the expected size of a Gaussian one).  Returns (max-abs, mean-abs)."""
    d = np.abs(f64(got) - want)
    half = sum(0.5 * ulp_bf16(np.abs(t) + MAX_ABS) for t in stores)      # ulp at the largest value that can be rounded
    sig = np.zeros(d.shape[0]) if ffn_sigma is None else ffn_sigma
    bound = MAX_ABS + half + 5.0 * sig[:, None]
    ratio = d / bound
    worst = int(np.argmax(ratio))
    frac = float((ratio > 1.0).mean())
    mean_bound = MEAN_ABS + float(np.mean(0.5 * half)) + 0.8 * float(sig.mean())
    print(f"   {label}: max-abs {d.max():.3e}, mean-abs {d.mean():.3e} (bound {mean_bound:.3e}); largest error/bound "
          f"{ratio.flat[worst]:.2f} at |value| {abs(want.flat[worst]):.2f}; {frac:.1e} of {d.size} elements above the bound", flush=True)
    assert ratio.flat[worst] <= TAIL_FACTOR and frac <= TAIL_FRACTION, (
        f"{label}: element {np.unravel_index(worst, d.shape)} off by {d.flat[worst]:.3e}, bound {bound.flat[worst]:.3e} at |value| "
        f"{abs(want.flat[worst]):.3f}; {frac:.2e} of the elements above their bound")
    assert d.mean() <= mean_bound, f"{label}: mean-abs {d.mean():.3e} above {mean_bound:.3e}"
    return float(d.max()), float(d.mean())


def score_rounding_scale(s: so.LayerShape, w: so.LayerWeights, x: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """Per block: the root-sum-square of the Hkv*d products qt_i * k_i behind its score (k = the representative
    key that wins the block, qt = the window query with Eq. 2's head mean folded in), from the exact oracle's own
    Key and Query states.  A bf16-stored factor is off by up to 2^-9 of its size and the errors of the products
    add in quadrature, so a score moves by about 2^-9 / sqrt(3) times this per rounded tensor (key, normalised
    row, window Query state): the scale of the tolerance where the stated 2e-3 is too small for the scores'
    size (biases, max pooling, single-token units)."""
    N = x.shape[0]
    h = so.rmsnorm(x, w.g_attn, s.rms_eps)
    k = so.project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, None, w.bk)
    w_eff = min(s.window, N)
    q_win = so.project_heads(h[N - w_eff:], w.wq, s.n_q_heads, s.head_dim, pos[N - w_eff:], s.rope_theta, True, None, w.bq)
    G = s.n_q_heads // s.n_kv_heads
    qt = so.window_query(q_win).reshape(s.n_kv_heads, G, s.head_dim).sum(axis=1) / s.n_q_heads      # [Hkv, d]
    nb = so.n_blocks(N, s.block)
    out = np.empty(nb)
    for j in range(nb):
        kb = k[j * s.block:min((j + 1) * s.block, N)]
        if s.scoring == "unit":
            reps = so.unit_keys(kb, s.unit)
        else:
            reps = (kb.mean(axis=0) if s.scoring == "avg" else kb.max(axis=0))[None]
        out[j] = np.sqrt(((reps * qt[None]) ** 2).sum(axis=(1, 2))).max()
    return out


def score_tolerance(s, w, x, pos) -> np.ndarray:
    """Per-block tolerance of a bf16 score against the exact oracle: the stated 2e-3 plus 2^-7 of the
    root-sum-square of the products behind it (four standard deviations of three rounded tensors)."""
    return 2e-3 + 2.0 ** -7 * score_rounding_scale(s, w, x, pos)


def bf16_floor(s, w, x, pos, kept, rows=None):
    """Information for the log, not a gate: error of the oracle with bf16 rounding at every stored tensor against
    the exact oracle on the same kept set.  Returns (z_exact, max, mean)."""
    after = so.layer_after_selection_literal if s.placement == "after" else so.layer_after_selection
    z, _ = after(s, w, x, pos, kept, rows=rows)
    zb, _ = after(s, w, x, pos, kept, rows=rows, rounding="bf16")
    d = np.abs(z - zb)
    return z, float(d.max()), float(d.mean())
