"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in the CPU oracle (a dropped term, a wrong
sign or index, a transposed operand, an off-by-one) and runs the pin tests against the damaged oracle: at least one
pin must fail.  Everything here runs on the CPU; nothing touches the GPU path."""
import inspect
import itertools
import math
import warnings

import numpy as np
import pytest

from oracle import slim_oracle as so
from tests import test_oracle_pins as pins

ORIG = {name: getattr(so, name) for name in dir(so) if inspect.isfunction(getattr(so, name))}


def pin_calls():
    """Every pin as (label, zero-argument callable), parametrised pins expanded over their argument sets."""
    calls = []
    for name, fn in sorted(vars(pins).items()):
        if not (name.startswith("test_") and inspect.isfunction(fn)):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        axes = []
        for m in marks:
            names = [a.strip() for a in m.args[0].split(",")]
            axes.append([dict(zip(names, v if len(names) > 1 else (v,))) for v in m.args[1]])
        for combo in itertools.product(*axes):
            kw = {}
            for part in combo:
                kw.update(part)
            calls.append((f"{name}[{kw}]", (lambda f=fn, k=kw: f(**k))))
    return calls


def failing_pins(stop_at_first=True):
    failed = []
    saved = pins.rng
    pins.rng = np.random.default_rng(1234)                       # the pins' shared generator, from its start
    try:
        for label, call in pin_calls():
            try:
                with np.errstate(all="ignore"), warnings.catch_warnings():
                    warnings.simplefilter("ignore")
                    call()
            except Exception as e:                               # an assertion, or a shape error the mistake causes
                failed.append((label, type(e).__name__))
                if stop_at_first:
                    break
    finally:
        pins.rng = saved
    return failed


# ------------------------------------------------------------------------------------------------ the mistakes
def m_rmsnorm_eps_outside(x, gain, eps):
    return gain * (x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps))


def m_rmsnorm_subtracts_mean(x, gain, eps):
    xc = x - x.mean(axis=-1, keepdims=True)
    return gain * (xc / np.sqrt(np.mean(xc * xc, axis=-1, keepdims=True) + eps))


def m_linear_not_transposed(h, W):
    return h @ W if W.shape[0] == W.shape[1] else h @ W.T


def m_rope_exponent_halved(pos, head_dim, theta, dtype):
    i = np.arange(head_dim // 2, dtype=np.float64)
    ang = pos.astype(np.float64)[:, None] * (theta ** (-1.0 * i / head_dim))[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def m_rope_angles_in_float32(pos, head_dim, theta, dtype):
    i = np.arange(head_dim // 2, dtype=np.float32)
    ang = pos.astype(np.float32)[:, None] * (np.float32(theta) ** (-2.0 * i / head_dim)).astype(np.float32)[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def m_rope_wrong_sign(x, cos, sin):
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([x1 * c + x2 * s, x2 * c - x1 * s], axis=-1)


def m_rope_interleaved_pairs(x, cos, sin):
    x1, x2 = x[..., 0::2], x[..., 1::2]
    c, s = cos[:, None, :], sin[:, None, :]
    out = np.empty_like(x)
    out[..., 0::2] = x1 * c - x2 * s
    out[..., 1::2] = x2 * c + x1 * s
    return out


def m_silu_wrong_sign(a):
    return a / (1.0 + np.exp(a))


def m_window_query_sum(q_win):
    return q_win.sum(axis=0)


def m_unit_keys_divide_by_unit(k_block, unit):
    return np.stack([k_block[s:s + unit].sum(axis=0) / unit for s in range(0, k_block.shape[0], unit)])


def _scores_variant(head_map, reduce_units):
    def f(q_win, k, block, unit):
        Hq, Hkv = q_win.shape[1], k.shape[1]
        q_l = ORIG["window_query"](q_win)
        N = k.shape[0]
        out = np.empty(so.n_blocks(N, block), dtype=k.dtype)
        for j in range(out.shape[0]):
            k_rep = ORIG["unit_keys"](k[j * block:min((j + 1) * block, N)], unit)
            k_rep_h = k_rep[:, [head_map(h, Hq, Hkv) for h in range(Hq)], :]
            out[j] = reduce_units(np.einsum("hd,mhd->mh", q_l, k_rep_h))
        return out
    return f


m_scores_interleaved_heads = _scores_variant(lambda h, Hq, Hkv: h % Hkv, lambda ph: ph.mean(axis=1).max())
m_scores_mean_over_units = _scores_variant(lambda h, Hq, Hkv: h // (Hq // Hkv), lambda ph: ph.mean(axis=1).mean())
m_scores_max_per_head = _scores_variant(lambda h, Hq, Hkv: h // (Hq // Hkv), lambda ph: ph.max(axis=0).mean())


def m_pooled_ignores_mode(q_win, k, block, pooling):
    return ORIG["block_scores_pooled"](q_win, k, block, "avg")


def _select_variant(forced_of, order_key, sort_result=True):
    def f(scores, n_keep, force_first=True, force_last=True):
        nb = scores.shape[0]
        if n_keep >= nb:
            return np.arange(nb, dtype=np.int32)
        forced = forced_of(nb, force_first, force_last)
        rest = [j for j in range(nb) if j not in forced]
        rest.sort(key=lambda j: order_key(scores, j))
        kept = list(forced | set(rest[:n_keep - len(forced)]))
        return np.asarray(sorted(kept) if sort_result else kept[::-1], dtype=np.int32)
    return f


_forced_ok = lambda nb, ff, fl: ({0} if ff else set()) | ({nb - 1} if fl else set())
m_select_forgets_last = _select_variant(lambda nb, ff, fl: {0} if ff else set(), lambda s, j: (-float(s[j]), j))
m_select_ties_to_higher_index = _select_variant(_forced_ok, lambda s, j: (-float(s[j]), -j))
m_select_lowest_scores = _select_variant(_forced_ok, lambda s, j: (float(s[j]), j))
m_select_unsorted = _select_variant(_forced_ok, lambda s, j: (-float(s[j]), j), sort_result=False)


def m_compact_renumbers_positions(src, pos, kept_blocks, block):
    T = ORIG["kept_token_index"](kept_blocks, block, src.shape[0])
    return src[T], np.arange(len(T), dtype=pos.dtype)


def m_kept_index_full_last_block(kept_blocks, block, n_tokens):
    parts = [np.minimum(np.arange(b * block, (b + 1) * block), n_tokens - 1) for b in kept_blocks]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)


def _attention_variant(mask_le=True, scaled=True, head_of=lambda h, G, Hkv: h // G, max_sub=True):
    def f(q, k, v, scale=None, rows=None, chunk=256, rounding=None):
        nq, Hq, d = q.shape
        n, Hkv, _ = k.shape
        G = Hq // Hkv
        if scale is None:
            scale = 1.0 / math.sqrt(d)
        if not scaled:
            scale = 1.0
        if rows is None:
            rows = np.arange(n)
        out = np.empty_like(q)
        for h in range(Hq):
            g = head_of(h, G, Hkv)
            s = (q[:, h, :] @ k[:, g, :].T) * scale
            j = np.arange(n)[None, :]
            vis = (j <= rows[:, None]) if mask_le else ((j < rows[:, None]) | (rows[:, None] == 0))
            s = np.where(vis, s, -np.inf)
            if max_sub:
                s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            out[:, h, :] = (p @ v[:, g, :]) / p.sum(axis=1, keepdims=True)
        return out
    return f


m_attention_excludes_diagonal = _attention_variant(mask_le=False)
m_attention_unscaled = _attention_variant(scaled=False)
m_attention_interleaved_heads = _attention_variant(head_of=lambda h, G, Hkv: h % Hkv)
m_attention_no_max_subtraction = _attention_variant(max_sub=False)


def m_decode_attention_unscaled(q, k, v, scale=None):
    return ORIG["decode_attention"](q, k, v, 1.0)


def m_swap_overlap_over_active(active_prev, candidate, memory, gamma):
    active_prev, candidate, memory = set(active_prev), set(candidate), set(memory)
    overlap = len(candidate & active_prev) / max(len(active_prev), 1)
    if overlap < gamma:
        active = set(candidate)
        offload = (active_prev - active) - memory
        return dict(active=active, offload=offload, load=active - active_prev, memory=memory | offload,
                    overlap=overlap, swapped=True)
    return dict(active=active_prev, offload=set(), load=set(), memory=memory, overlap=overlap, swapped=False)


def m_swap_offloads_blocks_already_in_memory(active_prev, candidate, memory, gamma):
    r = ORIG["kv_swap_step"](active_prev, candidate, memory, gamma)
    if r["swapped"]:
        r["offload"] = set(active_prev) - set(candidate)
    return r


def m_swap_not_strict(active_prev, candidate, memory, gamma):
    return ORIG["kv_swap_step"](active_prev, candidate, memory, np.nextafter(gamma, 2.0))


def _layer_variant(swap_gate_up=False, drop_attn_residual=False, drop_ffn_residual=False, v_gets_rope=False,
                   norm_reuses_attn_gain=False):
    def f(s, w, x, pos, kept_blocks, rows=None, rounding=None):
        xk, posk = ORIG["compact_tokens"](x, pos, kept_blocks, s.block)
        n = xk.shape[0]
        h = so.rmsnorm(xk, w.g_attn, s.rms_eps)
        k = so.project_heads(h, w.wk, s.n_kv_heads, s.head_dim, posk, s.rope_theta, True, rounding, w.bk)
        v = so.project_heads(h, w.wv, s.n_kv_heads, s.head_dim, posk, s.rope_theta, v_gets_rope, rounding, w.bv)
        if rows is None:
            rows = np.arange(n)
        q = so.project_heads(h[rows], w.wq, s.n_q_heads, s.head_dim, posk[rows], s.rope_theta, True, rounding, w.bq)
        o = so.causal_gqa_attention(q, k, v, rows=rows, rounding=rounding)
        y = so.linear(o.reshape(len(rows), -1), w.wo) + (0.0 if drop_attn_residual else xk[rows])
        r = so.rmsnorm(y, w.g_attn if norm_reuses_attn_gain else w.g_ffn, s.rms_eps)
        g, u = (w.w_up, w.w_gate) if swap_gate_up else (w.w_gate, w.w_up)
        z = so.linear(so.silu(so.linear(r, g)) * so.linear(r, u), w.w_down) + (0.0 if drop_ffn_residual else y)
        return z, posk
    return f


def m_layer_scores_window_from_the_front(s, w, x, pos, rounding=None):
    N = x.shape[0]
    h = so.rmsnorm(x, w.g_attn, s.rms_eps)
    k = so.project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bk)
    w_eff = min(s.window, N)
    q_win = so.project_heads(h[:w_eff], w.wq, s.n_q_heads, s.head_dim, pos[:w_eff], s.rope_theta, True, rounding, w.bq)
    return so.block_scores(q_win, k, s.block, s.unit), k


def m_project_heads_bias_after_rope(h, W, n_heads, head_dim, pos, theta, rope, rounding=None, bias=None):
    y = so.linear(h, W).reshape(h.shape[0], n_heads, head_dim)
    if rope:
        cos, sin = so.rope_cos_sin(pos, head_dim, theta, h.dtype)
        y = so.apply_rope(y, cos, sin)
    if bias is not None:
        y = y + bias.reshape(n_heads, head_dim)
    return y


def m_keep_count_floor(ratio, nb, n_forced=2):
    return int(min(nb, max(min(n_forced, nb), math.floor(ratio * nb))))


def m_model_prunes_for_the_next_layer(s, weights_of_layer, n_layers, x, pos, schedule, rounding=None):
    shifted = {l + 1: r for l, r in schedule.items()}
    return ORIG["prefill_model"](s, weights_of_layer, n_layers, x, pos, shifted, rounding)


def m_round_bf16_truncates(a):
    f = np.ascontiguousarray(a, dtype=np.float32)
    return (f.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32).astype(a.dtype, copy=False)


def m_n_blocks_floor(n_tokens, block):
    return max(1, n_tokens // block)


def m_all_unit_keys_zero_for_missing(k, block, unit):
    return np.nan_to_num(ORIG["all_unit_keys"](k, block, unit), nan=0.0)


def m_scores_from_unit_keys_interleaved_heads(q_win, k_rep):
    Hq, Hkv = q_win.shape[1], k_rep.shape[2]
    q_l = ORIG["window_query"](q_win)
    out = np.empty(k_rep.shape[0], dtype=k_rep.dtype)
    for j in range(k_rep.shape[0]):
        present = ~np.isnan(k_rep[j, :, 0, 0])
        k_rep_h = k_rep[j, present][:, [h % Hkv for h in range(Hq)], :]
        out[j] = np.einsum("hd,mhd->mh", q_l, k_rep_h).mean(axis=1).max()
    return out


def m_selection_cut_is_last_taken(scores, n_keep, force_first=True, force_last=True):
    nb = scores.shape[0]
    forced = ({0} if force_first else set()) | ({nb - 1} if force_last else set())
    rest = sorted((j for j in range(nb) if j not in forced), key=lambda j: (-float(scores[j]), j))
    take = n_keep - len(forced)
    if n_keep >= nb or take >= len(rest):
        return None
    return float(scores[rest[max(take - 1, 0)]])


def m_attention_ignores_rows(q, k, v, scale=None, rows=None, chunk=256, rounding=None):
    if rows is not None and len(rows) == k.shape[0]:
        rows = None
    return ORIG["causal_gqa_attention"](q, k, v, scale, None if rows is None else np.minimum(rows + 1, k.shape[0] - 1),
                                        chunk, rounding)


def m_literal_placement_attends_kept_keys_only(s, w, x, pos, kept_blocks, rows=None, rounding=None):
    return ORIG["layer_after_selection"](s, w, x, pos, kept_blocks, rows, rounding)


def m_decode_layer_forgets_its_own_kv(s, w, x_new, pos_new, k_ctx, v_ctx, rounding=None):
    x = x_new[None, :]
    pos = np.asarray([pos_new])
    h = so.rmsnorm(x, w.g_attn, s.rms_eps)
    q = so.project_heads(h, w.wq, s.n_q_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bq)
    k = so.project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bk)
    v = so.project_heads(h, w.wv, s.n_kv_heads, s.head_dim, pos, s.rope_theta, False, rounding, w.bv)
    o = so.decode_attention(q[0], k_ctx, v_ctx)
    y = x + so.linear(o.reshape(1, -1), w.wo)
    r = so.rmsnorm(y, w.g_ffn, s.rms_eps)
    z = y + so.linear(so.silu(so.linear(r, w.w_gate)) * so.linear(r, w.w_up), w.w_down)
    return z[0], k[0], v[0]


def m_active_token_index_unsorted(active_blocks, block, n_prompt):
    return ORIG["kept_token_index"](np.asarray(sorted(active_blocks, reverse=True), dtype=np.int64), block, n_prompt)


def m_pruned_layer_never_forces_the_last_block(s, w, x, pos, n_keep, force_first=True, force_last=True, rounding=None):
    return ORIG["pruned_layer"](s, w, x, pos, n_keep, force_first, False, rounding)


MISTAKES = [
    ("rmsnorm", m_rmsnorm_eps_outside), ("rmsnorm", m_rmsnorm_subtracts_mean),
    ("linear", m_linear_not_transposed),
    ("rope_cos_sin", m_rope_exponent_halved), ("rope_cos_sin", m_rope_angles_in_float32),
    ("apply_rope", m_rope_wrong_sign), ("apply_rope", m_rope_interleaved_pairs),
    ("silu", m_silu_wrong_sign),
    ("window_query", m_window_query_sum), ("unit_keys", m_unit_keys_divide_by_unit),
    ("block_scores", m_scores_interleaved_heads), ("block_scores", m_scores_mean_over_units),
    ("block_scores", m_scores_max_per_head), ("block_scores_pooled", m_pooled_ignores_mode),
    ("select_blocks", m_select_forgets_last), ("select_blocks", m_select_ties_to_higher_index),
    ("select_blocks", m_select_lowest_scores), ("select_blocks", m_select_unsorted),
    ("compact_tokens", m_compact_renumbers_positions), ("kept_token_index", m_kept_index_full_last_block),
    ("causal_gqa_attention", m_attention_excludes_diagonal), ("causal_gqa_attention", m_attention_unscaled),
    ("causal_gqa_attention", m_attention_interleaved_heads), ("causal_gqa_attention", m_attention_no_max_subtraction),
    ("decode_attention", m_decode_attention_unscaled),
    ("kv_swap_step", m_swap_overlap_over_active), ("kv_swap_step", m_swap_offloads_blocks_already_in_memory),
    ("kv_swap_step", m_swap_not_strict),
    ("layer_after_selection", _layer_variant(swap_gate_up=True)),
    ("layer_after_selection", _layer_variant(drop_attn_residual=True)),
    ("layer_after_selection", _layer_variant(drop_ffn_residual=True)),
    ("layer_after_selection", _layer_variant(v_gets_rope=True)),
    ("layer_after_selection", _layer_variant(norm_reuses_attn_gain=True)),
    ("layer_scores", m_layer_scores_window_from_the_front),
    ("project_heads", m_project_heads_bias_after_rope),
    ("n_keep_from_ratio", m_keep_count_floor),
    ("prefill_model", m_model_prunes_for_the_next_layer),
    ("round_bf16", m_round_bf16_truncates), ("n_blocks", m_n_blocks_floor),
    ("all_unit_keys", m_all_unit_keys_zero_for_missing),
    ("block_scores_from_unit_keys", m_scores_from_unit_keys_interleaved_heads),
    ("selection_cut", m_selection_cut_is_last_taken),
    ("causal_gqa_attention", m_attention_ignores_rows),
    ("layer_after_selection_literal", m_literal_placement_attends_kept_keys_only),
    ("decode_layer", m_decode_layer_forgets_its_own_kv),
    ("active_token_index", m_active_token_index_unsorted),
    ("pruned_layer", m_pruned_layer_never_forces_the_last_block),
]


def test_pins_pass_on_the_oracle_as_it_stands():
    assert failing_pins(stop_at_first=False) == []


@pytest.mark.parametrize("idx", range(len(MISTAKES)))
def test_a_planted_mistake_fails_some_pin(idx, monkeypatch):
    target, wrong = MISTAKES[idx]
    assert target in ORIG
    monkeypatch.setattr(so, target, wrong)
    failed = failing_pins()
    name = getattr(wrong, "__name__", "variant")
    print(f"{target} <- {name}: caught by {failed[0] if failed else None}")
    assert failed, f"no pin notices the mistake planted in {target} ({name})"
