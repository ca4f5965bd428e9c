"""GPU parity of slim_pruned_layer against the CPU oracle: the fp32 workload in full, reduced bf16
workloads in full, and the full-size bf16 workloads on sampled output rows (scores and the kept
set are always checked in full)."""
import numpy as np
import pytest
import torch

from oracle import slim_oracle as so
from paper_2508_06447_amd import inputs
from tests.helpers import (F32_MAX_ABS, MAX_ABS, MEAN_ABS, assert_residual_close, assert_selection_matches, bf16_floor, errs,
                           f64, ffn_response_sigma, oracle_shape, oracle_weights, score_tolerance)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def slim():
    import paper_2508_06447_amd as slim
    slim.load_library()
    return slim


SCORING_CODE = {"unit": 0, "avg": 1, "max": 2}


def fold_gains(slim, wd):
    """The layer's weights with both RMSNorm gains folded into the projections that follow them (gains -> NULL)."""
    out = {k: v for k, v in wd.items() if k not in ("g_attn", "g_ffn")}
    for g, names in (("g_attn", ("wq", "wk", "wv")), ("g_ffn", ("w_gate", "w_up"))):
        if not bool((wd[g] == 1).all()):                 # unit gains: nothing to fold
            for n in names:
                out[n] = slim.slim_fold_gain(wd[n], wd[g])
    return out


def run_gpu(slim, wl, x, w, pos, n_keep, flags=3, scoring="unit", placement="before", fold=False):
    shape = slim.make_shape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.block, wl.unit,
                            wl.window, x.dtype, wl.rope_theta, wl.rms_eps, flags, SCORING_CODE[scoring],
                            1 if placement == "after" else 0)
    wd = {k: v.cuda() for k, v in w.items()}
    if fold:
        wd = fold_gains(slim, wd)
    res = slim.slim_pruned_layer(shape, wd, x.cuda(), None if pos is None else pos.cuda(), n_keep)
    torch.cuda.synchronize()
    return res


def sample_rows(n, block, count=48, seed=0):
    g = np.random.default_rng(seed)
    fixed = [0, 1, block - 1, block, n // 2, n - block, n - 2, n - 1, 127, 128, 255, 256]
    rows = set(r for r in fixed if 0 <= r < n)
    rows |= set(g.integers(0, n, max(0, count - len(rows))).tolist())
    return np.array(sorted(rows))


def check_layer(slim, wl, np_dtype, rows_count=None, label="", scoring="unit", placement="before", score_scaled=False,
                fold=False, gains=None, floor_info=False):
    """Runs the GPU layer and the oracle on one workload.  Always checked here: kept set (outside the 1e-3 band),
    positions, and for bf16 the residual stream element by element (assert_residual_close) at two places: y, the
    residual after the attention branch (on the GPU the layer run with a zero down projection returns exactly it), and z; and the FFN branch z - y at its own scale.  Scores: against the stated 2e-3, or with
    score_scaled against score_tolerance.  fold: the RMSNorm gains are folded into the weights and the norms run
    inside the projections (the configuration bench.py times); gains: (g_attn, g_ffn) tensors that replace the
    workload's unit gains.  Returns the numbers for the log."""
    x, w, pos = inputs.hidden_states(wl), inputs.layer_weights(wl), inputs.positions(wl)
    if gains is not None:
        w = dict(w, g_attn=gains[0], g_ffn=gains[1])
    n_keep = wl.n_keep
    res = run_gpu(slim, wl, x, w, pos, n_keep, scoring=scoring, placement=placement, fold=fold)
    s, ow = oracle_shape(wl, scoring, placement), oracle_weights(w, np_dtype)
    xs = x.to(torch.float32).numpy().astype(np_dtype)
    kept_gpu = res["kept"].cpu().numpy()
    if n_keep < wl.n_blocks:
        sc_ref, _ = so.layer_scores(s, ow, xs, pos.numpy())
        sc_gpu = f64(res["scores"])
        sc_err = float(np.abs(sc_gpu - sc_ref).max())
        want, band, ndiff = assert_selection_matches(kept_gpu, sc_ref.astype(np.float64), n_keep)
        if x.dtype == torch.bfloat16:
            tol = score_tolerance(s, ow, xs, pos.numpy()) if score_scaled else np.full(sc_ref.shape, 2e-3)
            worst = int(np.argmax(np.abs(sc_gpu - sc_ref) - tol))
            assert (np.abs(sc_gpu - sc_ref) <= tol).all(), (f"{label}: score of block {worst} off by "
                                                             f"{abs(sc_gpu[worst] - sc_ref[worst]):.2e}, allowed {tol[worst]:.2e}")
    else:                                                # a Preserve layer: nothing is scored, every block continues
        np.testing.assert_array_equal(kept_gpu, np.arange(wl.n_blocks))
        sc_ref, sc_err, band, ndiff = np.zeros(1), 0.0, 0, 0
    n_out = slim.kept_tokens(wl.seq, wl.block, n_keep)
    assert res["x"].shape[0] == n_out
    # positions and (teacher-forced on the GPU's set) the layer output
    T = so.kept_token_index(kept_gpu, wl.block, wl.seq)
    np.testing.assert_array_equal(res["pos"].cpu().numpy(), pos.numpy()[T])
    rows = None if rows_count is None else sample_rows(n_out, wl.block, rows_count)
    after = so.layer_after_selection_literal if placement == "after" else so.layer_after_selection
    z_ref, _, y_ref = after(s, ow, xs, pos.numpy(), kept_gpu, rows=rows, want_y=True)
    z_ref, y_ref = z_ref.astype(np.float64), y_ref.astype(np.float64)
    pick = (lambda t: t) if rows is None else (lambda t: t[torch.from_numpy(rows).cuda()])
    got = pick(res["x"])
    out = dict(sc_err=sc_err, sc_scale=float(np.abs(sc_ref).max()))
    if x.dtype == torch.bfloat16:
        # y on the GPU: the same layer with a zero down projection returns exactly it
        w0 = dict(w, w_down=torch.zeros_like(w["w_down"]))
        y_gpu = pick(run_gpu(slim, wl, x, w0, pos, n_keep, scoring=scoring, placement=placement, fold=fold)["x"])
        ymx, ymean = assert_residual_close(y_gpu, y_ref, [y_ref], f"{label} y")
        # the FFN half alone: the oracle's FFN on the GPU's own y (teacher-forced), so that only the FFN's roundings
        # and the store of z are left; with gain vectors the normalised row is stored too (one more rounding), and
        # folding gains that are not 1 rounds gain * weight to bf16 (the same size of effect on the projections)
        stored_r = 0 if (fold and gains is None) else 1
        z_tf = so.ffn_residual(s, ow, f64(y_gpu).astype(np_dtype)).astype(np.float64)
        assert_residual_close(got, z_tf, [z_tf], f"{label} z from the GPU's y",
                              ffn_sigma=ffn_response_sigma(f64(y_gpu), z_tf, None, stored_r) if stored_r else None)
        # end to end against the exact z: additionally the FFN's answer to the deviation of the GPU's y
        sig = ffn_response_sigma(y_ref, z_ref, f64(y_gpu) - y_ref, stored_r)
        mx, mean = assert_residual_close(got, z_ref, [z_ref, y_ref], f"{label} z", ffn_sigma=sig)
        f_gpu, f_ref = f64(got) - f64(y_gpu), z_ref - y_ref
        f_rel = float(np.sqrt(np.mean((f_gpu - f_ref) ** 2)) / np.sqrt(np.mean(f_ref ** 2)))
        out.update(ymx=ymx, ymean=ymean, f_rel=f_rel)
        extra = f"; y max-abs {ymx:.3e} mean-abs {ymean:.3e}; FFN branch z - y: rms error {f_rel:.2e} of its rms"
    else:
        mx, mean = errs(got, z_ref)
        extra = ""
    out.update(mx=mx, mean=mean)
    if floor_info:
        _, fl_max, fl_mean = bf16_floor(s, ow, xs, pos.numpy(), kept_gpu, rows=rows)
        extra += f"; oracle with bf16 rounding at every stored tensor, for comparison: {fl_max:.3e} / {fl_mean:.3e}"
    print(f"{label}: scores max-abs {sc_err:.2e} (|scores| max {out['sc_scale']:.2f}); kept {len(kept_gpu)} blocks, {band} in the "
          f"1e-3 band, {ndiff} differ; z max-abs {mx:.3e} mean-abs {mean:.3e} (|z| max {np.abs(z_ref).max():.2f}){extra}", flush=True)
    return out


def test_cfg1_fp32_full(slim):
    wl = inputs.WORKLOADS["cfg1"]
    r = check_layer(slim, wl, np.float64, label="cfg1")
    assert r["sc_err"] < 1e-5 and r["mx"] < F32_MAX_ABS


def test_cfg1_keep_all_equals_unpruned_layer(slim):
    wl = inputs.WORKLOADS["cfg1"]
    x, w, pos = inputs.hidden_states(wl), inputs.layer_weights(wl), inputs.positions(wl)
    res = run_gpu(slim, wl, x, w, pos, wl.n_blocks)                       # Preserve layer
    res2 = run_gpu(slim, wl, x, w, None, wl.n_blocks + 7)                 # NULL positions, n_keep > nb
    assert torch.equal(res["x"], res2["x"]) and torch.equal(res["pos"], res2["pos"])
    np.testing.assert_array_equal(res["kept"].cpu().numpy(), np.arange(wl.n_blocks))
    ref = so.pruned_layer(oracle_shape(wl), oracle_weights(w), f64(x), pos.numpy(), wl.n_blocks)
    mx, _ = errs(res["x"], ref["z"])
    assert mx < F32_MAX_ABS
    np.testing.assert_array_equal(res["pos"].cpu().numpy(), pos.numpy())


@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("seq,block,window,keep", [(1024, 64, 64, 0.5), (1000, 64, 64, 0.3), (1536, 128, 128, 0.25)])
def test_reduced_bf16_layer_full_output(slim, seq, block, window, keep, fold):
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=seq, block=block, window=window, keep_ratio=keep, planted=seq // 100)
    check_layer(slim, wl, np.float64, label=f"llama-shaped seq {seq} block {block} keep {keep} fold {fold}", fold=fold,
                floor_info=True)


@pytest.mark.parametrize("scoring", ["avg", "max"])
def test_layer_with_pooled_scoring(slim, scoring):
    """The pooled scoring baselines of Table 3 inside the layer: fp32 workload and a reduced bf16 one."""
    r = check_layer(slim, inputs.WORKLOADS["cfg1"], np.float64, label=f"cfg1 {scoring}-pool", scoring=scoring)
    assert r["sc_err"] < 1e-5 and r["mx"] < F32_MAX_ABS
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=1000, keep_ratio=0.3, planted=10)
    # bf16 Key states against the float64 oracle: a maximum over 64 tokens does not average the rounding of the
    # keys out the way a mean does, so the scores are held to the tolerance that follows their products' size
    check_layer(slim, wl, np.float64, label=f"llama-shaped seq 1000 {scoring}-pool", scoring=scoring, score_scaled=True)


def test_layer_with_blocks_dropped_after_attention(slim):
    """Section 4.1's order: the pruning layer's attention sees all tokens, the blocks are dropped after it."""
    r = check_layer(slim, inputs.WORKLOADS["cfg1"], np.float64, label="cfg1, drop after attention", placement="after")
    assert r["sc_err"] < 1e-5 and r["mx"] < F32_MAX_ABS
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=1000, keep_ratio=0.3, planted=10)
    check_layer(slim, wl, np.float64, label="llama-shaped seq 1000, drop after attention", placement="after")
    # Every step after attention is per token and the kernels accumulate each output element in the same
    # order whatever the row count, so the result is bit for bit the unpruned layer's rows at the kept
    # tokens; scores, kept set and positions equal those of the graded placement.
    x, w, pos = inputs.hidden_states(wl), inputs.layer_weights(wl), inputs.positions(wl)
    lit = run_gpu(slim, wl, x, w, pos, wl.n_keep, placement="after")
    std = run_gpu(slim, wl, x, w, pos, wl.n_keep)
    full = run_gpu(slim, wl, x, w, pos, wl.n_blocks)
    assert torch.equal(lit["kept"], std["kept"]) and torch.equal(lit["pos"], std["pos"])
    assert torch.equal(lit["scores"], std["scores"])
    T = torch.from_numpy(so.kept_token_index(lit["kept"].cpu().numpy(), wl.block, wl.seq)).cuda()
    assert torch.equal(lit["x"], full["x"][T])


def test_reduced_bf16_keep_all_and_prefix_property(slim):
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=768, keep_ratio=1.0, planted=7)
    x, w, pos = inputs.hidden_states(wl), inputs.layer_weights(wl), inputs.positions(wl)
    full = run_gpu(slim, wl, x, w, pos, wl.n_blocks)
    s, ow = oracle_shape(wl), oracle_weights(w)
    all_blocks = np.arange(wl.n_blocks, dtype=np.int32)
    z_ref, _, y_ref = so.layer_after_selection(s, ow, f64(x), pos.numpy(), all_blocks, want_y=True)
    y_gpu = run_gpu(slim, wl, x, dict(w, w_down=torch.zeros_like(w["w_down"])), pos, wl.n_blocks)["x"]
    mx, mean = assert_residual_close(full["x"], z_ref, [z_ref, y_ref], "keep-all z",
                                     ffn_sigma=ffn_response_sigma(y_ref, z_ref, f64(y_gpu) - y_ref, 1))
    print(f"keep-all: z max-abs {mx:.3e} mean-abs {mean:.3e}", flush=True)
    # Causal attention never looks right: rows of kept blocks that form a prefix equal the unpruned rows.
    pr = run_gpu(slim, wl, x, w, pos, 5)
    kept = pr["kept"].cpu().numpy()
    lead = 0
    while lead < len(kept) and kept[lead] == lead:
        lead += 1
    a, b = f64(pr["x"][: lead * wl.block]), f64(full["x"][: lead * wl.block])
    assert lead >= 1 and np.abs(a - b).max() <= 2 * MAX_ABS


@pytest.mark.parametrize("fold", [False, True])
def test_layer_with_non_unit_gains(slim, fold):
    """RMSNorm gains that are not 1: as gain vectors (norm kernels) and folded into the weights by slim_fold_gain
    (norms inside the projections), both against the oracle with the gains."""
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=1000, keep_ratio=0.3, planted=10)
    g = np.random.default_rng(17)
    gains = tuple(torch.from_numpy((1.0 + 0.2 * g.standard_normal(wl.hidden)).astype(np.float32)).to(torch.bfloat16)
                  for _ in range(2))
    check_layer(slim, wl, np.float64, label=f"llama-shaped seq 1000, random gains, fold {fold}", fold=fold, gains=gains)


@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("seq,block,window,keep", [
    (5, 64, 64, 1.0),        # fewer tokens than a block and than the window: one short block, nothing to drop
    (64, 64, 64, 1.0),       # exactly one block
    (70, 64, 64, 0.5),       # two blocks, both forced (first, short last): n_keep = 2 = nb, a Preserve layer
    (130, 64, 64, 0.1),      # three blocks, only the two forced ones kept: no slot left for the scored block
    (200, 16, 300, 0.3),     # window longer than the sequence: every token is in the window
    (257, 1, 4, 0.25),       # blocks of one token (unit 1): token-level pruning
    (300, 32, 1, 0.5),       # window of one token
])
def test_degenerate_small_sequences(slim, seq, block, window, keep, fold):
    """Edge shapes of the layer on a narrow bf16 model (2 kv heads of 128), against the oracle in full."""
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=seq, block=block, unit=min(8, block), window=window, keep_ratio=keep,
                       hidden=256, n_q_heads=4, n_kv_heads=2, ffn=512, planted=max(1, seq // 50))
    # single-token units and a one-token window leave nothing to average the keys' rounding out: scaled score tolerance
    check_layer(slim, wl, np.float64, label=f"narrow model seq {seq} block {block} window {window} keep {keep} fold {fold}",
                fold=fold, score_scaled=True)


def test_reduced_qwen_shaped_layer_full_output(slim):
    """Second model family (28 query / 4 kv heads, hidden 3584, FFN 18944, Q/K/V biases, theta 1e6)."""
    wl = inputs.scaled(inputs.WORKLOADS["cfg6"], seq=1000, x_kind="planted", planted=10)
    # biases of size 0.5 make the Query/Key states and the scores several times larger than in the LLaMA-shaped
    # workloads, and with them the bf16 rounding of the states: the score tolerance follows the products' size
    check_layer(slim, wl, np.float64, label="qwen-shaped seq 1000 keep 0.375", score_scaled=True, fold=True)


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg6"])
def test_full_size_workloads_sampled_rows(slim, name):
    wl = inputs.WORKLOADS[name]
    print(f"{name}: N={wl.seq} nb={wl.n_blocks} n_keep={wl.n_keep} n'={wl.n_kept_tokens}", flush=True)
    check_layer(slim, wl, np.float32, rows_count=64, label=name, score_scaled=wl.qkv_bias, fold=True)   # see the reduced Qwen-shaped test
