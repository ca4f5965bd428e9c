"""CPU oracle for the SlimInfer pruned prefill layer.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition the HIP kernels are checked against.  Only the test-suite,
the smoke check and the benchmark's `cpu_baseline` leg may import it; the product package never does,
and this module imports nothing from the product package.

Everything is NumPy on the host.  Arithmetic runs in `dtype` (float64 unless the caller asks for
float32); RoPE angles are always formed in float64.  There is no blocking, fusion or re-association
beyond what the paper's definitions state, except that attention is evaluated for a chunk of query rows
at a time so the full score matrix is never held in memory (each row's arithmetic is unchanged).

Notation follows the paper (Section 4.2): prompt blocks B_j of `block` tokens, each split into M
TokenUnits of `unit` tokens; k_rep(j, m) is the unit's mean Key state (Eq. 1); q_l is the mean Query
state of the last `window` tokens; r_block is the block score (Eq. 2).

Pins (tests/test_oracle_*.py): brute-force softmax attention written with scalar loops; torch's CPU
scaled-dot-product attention; closed-form score cases; exhaustive selection on tiny inputs;
keep-ratio 1.0 equals the unpruned layer; gather commutation of the per-token steps; RoPE relative-
position property.  The one thing with no pin is whether the heuristic preserves model accuracy
(Table 1 needs LongBench and trained weights): "parity unpinned" for that claim only.

`rounding="bf16"` makes every function round its result to bfloat16 precision at the points where a
bf16 pipeline stores a tensor (after RMSNorm, after each projection, the softmax probabilities, the
attention output, the activation, both residual sums).  It is used only to measure how far any bf16
pipeline can be from the exact result, never as the parity reference.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------------------------------
# rounding hook (identity for the reference; bf16 grid for the "how far can bf16 be" measurement)
# --------------------------------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 value (ties to even); result keeps a's dtype."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    out = u.astype(np.uint32).view(np.float32)
    return out.astype(a.dtype, copy=False)


def _rnd(a, rounding):
    return round_bf16(a) if rounding == "bf16" else a


# --------------------------------------------------------------------------------------------------
# per-token layer math ("QKV Generation" and "FFN" boxes of Fig. 2)
# --------------------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """h_t = gain * x_t / sqrt(mean_c(x_t[c]^2) + eps), one row per token."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return gain * (x / np.sqrt(ms + eps))


def linear(h: np.ndarray, W: np.ndarray) -> np.ndarray:
    """y = h W^T with W stored [out_features, in_features] (no bias)."""
    return h @ W.T


def rope_cos_sin(pos: np.ndarray, head_dim: int, theta: float, dtype):
    """cos/sin of pos * theta^(-2i/d), i = 0..d/2-1.  Angles in float64, then cast."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate-half RoPE on x[n, H, d]: the pair is (i, i + d/2), rotated by the angle of index i."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


# --------------------------------------------------------------------------------------------------
# block-wise prompt token pruning (Section 4.2)
# --------------------------------------------------------------------------------------------------
def n_blocks(n_tokens: int, block: int) -> int:
    return (n_tokens + block - 1) // block


def n_keep_from_ratio(ratio: float, nb: int, n_forced: int = 2) -> int:
    """Retained block count for a keep ratio: ceil(ratio * nb), clamped to [forced, nb]."""
    return int(min(nb, max(min(n_forced, nb), math.ceil(ratio * nb - 1e-12))))


def window_query(q_win: np.ndarray) -> np.ndarray:
    """q_l: mean of the Query states of the local window.  q_win[w, Hq, d] -> [Hq, d]."""
    return q_win.mean(axis=0)


def unit_keys(k_block: np.ndarray, unit: int) -> np.ndarray:
    """Eq. (1): representative keys of one block.  k_block[len, Hkv, d] -> [M, Hkv, d];
    a short trailing unit is averaged over the tokens it actually has."""
    reps = []
    for s in range(0, k_block.shape[0], unit):
        reps.append(k_block[s:s + unit].mean(axis=0))
    return np.stack(reps)


def block_scores(q_win: np.ndarray, k: np.ndarray, block: int, unit: int) -> np.ndarray:
    """Eq. (2): r_j = max_m (1/H) sum_h q_l^h . k_rep^h(j, m), H = number of query heads;
    query head h reads kv head h // (Hq/Hkv).  No softmax, no 1/sqrt(d).
    q_win[w, Hq, d] (post-RoPE), k[N, Hkv, d] (post-RoPE) -> scores[nb]."""
    Hq, Hkv = q_win.shape[1], k.shape[1]
    G = Hq // Hkv
    q_l = window_query(q_win)                                   # [Hq, d]
    N = k.shape[0]
    out = np.empty(n_blocks(N, block), dtype=k.dtype)
    for j in range(out.shape[0]):
        k_rep = unit_keys(k[j * block:min((j + 1) * block, N)], unit)   # [M, Hkv, d]
        k_rep_h = np.repeat(k_rep, G, axis=1)                   # [M, Hq, d]: head h -> kv head h//G
        per_head = np.einsum("hd,mhd->mh", q_l, k_rep_h)        # q_l^h . k_rep^h(j, m)
        out[j] = per_head.mean(axis=1).max()
    return out


def block_scores_pooled(q_win: np.ndarray, k: np.ndarray, block: int, pooling: str) -> np.ndarray:
    """The two baselines of the block-scoring ablation (Table 3, "Block Importance Scoring Algorithm"):
    one representative key per block, either the average of the block's token key states ("avg") or
    their element-wise maximum ("max"), scored against the window query as in Eq. (2):
    r_j = (1/H) sum_h q_l^h . k_pool^h(j).  A short last block pools the tokens it has."""
    assert pooling in ("avg", "max")
    Hq, Hkv = q_win.shape[1], k.shape[1]
    G = Hq // Hkv
    q_l = window_query(q_win)                                   # [Hq, d]
    N = k.shape[0]
    out = np.empty(n_blocks(N, block), dtype=k.dtype)
    for j in range(out.shape[0]):
        kb = k[j * block:min((j + 1) * block, N)]               # [len, Hkv, d]
        k_pool = kb.mean(axis=0) if pooling == "avg" else kb.max(axis=0)
        k_pool_h = np.repeat(k_pool, G, axis=0)                 # [Hq, d]: head h -> kv head h//G
        out[j] = np.einsum("hd,hd->h", q_l, k_pool_h).mean()
    return out


def all_unit_keys(k: np.ndarray, block: int, unit: int) -> np.ndarray:
    """Eq. (1) for every block of the prompt: k[N, Hkv, d] -> k_rep[nb, M, Hkv, d], M = ceil(block/unit).
    Units that do not exist (short last block) are NaN.  This is what a decode step can keep on the GPU
    when the Key states themselves have been moved to CPU memory."""
    N = k.shape[0]
    nb, M = n_blocks(N, block), (block + unit - 1) // unit
    out = np.full((nb, M) + k.shape[1:], np.nan, dtype=k.dtype)
    for j in range(nb):
        reps = unit_keys(k[j * block:min((j + 1) * block, N)], unit)
        out[j, :reps.shape[0]] = reps
    return out


def block_scores_from_unit_keys(q_win: np.ndarray, k_rep: np.ndarray) -> np.ndarray:
    """Eq. (2) on stored representative keys.  q_win[w, Hq, d] are the Query states of the local window:
    the end of the prompt during prefill, the most recently decoded tokens during decoding (Section 4.2)."""
    Hq, Hkv = q_win.shape[1], k_rep.shape[2]
    q_l = window_query(q_win)
    out = np.empty(k_rep.shape[0], dtype=k_rep.dtype)
    for j in range(k_rep.shape[0]):
        present = ~np.isnan(k_rep[j, :, 0, 0])
        k_rep_h = np.repeat(k_rep[j, present], Hq // Hkv, axis=1)
        out[j] = np.einsum("hd,mhd->mh", q_l, k_rep_h).mean(axis=1).max()
    return out


def kv_swap_step(active_prev, candidate, memory, gamma: float):
    """Algorithm 1 (overlap-aware KV swapping), one inference step.  Sets of block indices:
    active_prev = B_active(t-1) (KV on the GPU), candidate = B_candidate(t), memory = B_Memory (KV present
    in the CPU pool).  Returns dict(active, offload, load, memory, overlap, swapped).  The CPU pool keeps
    what was once offloaded (prompt KV never changes), so B_Memory only grows; a block to load must be
    in it."""
    active_prev, candidate, memory = set(active_prev), set(candidate), set(memory)
    overlap = len(candidate & active_prev) / len(candidate)
    if overlap < gamma:
        active = set(candidate)
        offload = (active_prev - active) - memory
        load = active - active_prev
        assert load <= memory, "a block to prefetch must be in the CPU pool"
        return dict(active=active, offload=offload, load=load, memory=memory | offload, overlap=overlap,
                    swapped=True)
    return dict(active=active_prev, offload=set(), load=set(), memory=memory, overlap=overlap, swapped=False)


def select_blocks(scores: np.ndarray, n_keep: int, force_first: bool = True,
                  force_last: bool = True) -> np.ndarray:
    """Forced blocks (first = attention sink; last) are always kept; the remaining
    n_keep - #forced slots go to the other blocks in order (score descending, index ascending).
    Returns ascending int32 block indices; n_keep >= nb keeps everything."""
    nb = scores.shape[0]
    assert not np.isnan(scores).any(), "selection is undefined on NaN scores"
    if n_keep >= nb:
        return np.arange(nb, dtype=np.int32)
    forced = set()
    if force_first:
        forced.add(0)
    if force_last:
        forced.add(nb - 1)
    assert n_keep >= len(forced)
    rest = [j for j in range(nb) if j not in forced]
    rest.sort(key=lambda j: (-float(scores[j]), j))
    kept = sorted(forced | set(rest[:n_keep - len(forced)]))
    return np.asarray(kept, dtype=np.int32)


def selection_cut(scores: np.ndarray, n_keep: int, force_first: bool = True,
                  force_last: bool = True):
    """Midpoint between the last taken and the first not-taken score among non-forced blocks
    (None if nothing is dropped).  Blocks whose score lies within a tolerance of this cut may
    legitimately go either way when the scores carry rounding error."""
    nb = scores.shape[0]
    forced = ({0} if force_first else set()) | ({nb - 1} if force_last else set())
    rest = sorted((j for j in range(nb) if j not in forced), key=lambda j: (-float(scores[j]), j))
    take = n_keep - len(forced)
    if n_keep >= nb or take >= len(rest):
        return None
    if take == 0:
        return float(scores[rest[0]]) + 1.0
    return 0.5 * (float(scores[rest[take - 1]]) + float(scores[rest[take]]))


def kept_token_index(kept_blocks: np.ndarray, block: int, n_tokens: int) -> np.ndarray:
    """Token rows of the kept blocks, in ascending order (only the last block can be short)."""
    parts = [np.arange(b * block, min((b + 1) * block, n_tokens)) for b in kept_blocks]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)


def compact_tokens(src: np.ndarray, pos: np.ndarray, kept_blocks: np.ndarray, block: int):
    """Hidden-state pruning: keep only the rows of the kept blocks, and carry their original
    positions along (they are what RoPE must see afterwards)."""
    T = kept_token_index(kept_blocks, block, src.shape[0])
    return src[T], pos[T]


# --------------------------------------------------------------------------------------------------
# attention ("Attention" box of Fig. 2): causal softmax attention with grouped kv heads
# --------------------------------------------------------------------------------------------------
def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None,
                         rows: np.ndarray | None = None, chunk: int = 256,
                         rounding: str | None = None) -> np.ndarray:
    """o_i^h = sum_{j<=i} softmax_j(scale * q_i^h . k_j^{h//G}) v_j^{h//G}.

    q[nq, Hq, d], k/v[n, Hkv, d].  `rows[nq]` gives each query's index in the key sequence
    (default: nq == n and row i is query i), so a sample of rows can be evaluated on its own."""
    nq, Hq, d = q.shape
    n, Hkv, _ = k.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    if rows is None:
        assert nq == n
        rows = np.arange(n)
    out = np.empty_like(q)
    for h in range(Hq):
        kh, vh = k[:, h // G, :], v[:, h // G, :]
        for c0 in range(0, nq, chunk):
            r = rows[c0:c0 + chunk]
            jmax = int(r.max()) + 1
            s = (q[c0:c0 + chunk, h, :] @ kh[:jmax].T) * scale            # [c, jmax]
            s = np.where(np.arange(jmax)[None, :] <= r[:, None], s, -np.inf)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            den = p.sum(axis=1, keepdims=True)
            out[c0:c0 + chunk, h, :] = (_rnd(p, rounding) @ vh[:jmax]) / den
    return out


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Attention of one new token during decoding (Section 4.1: only the active blocks take part, every response
    token is retained): q[Hq, d] attends to ALL the keys it is given, k/v[n, Hkv, d] = the prompt tokens of the
    active blocks followed by the response tokens.  o^h = sum_j softmax_j(scale q^h . k_j^{h//G}) v_j^{h//G}."""
    Hq, d = q.shape
    n, Hkv, _ = k.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty_like(q)
    for h in range(Hq):
        s = (k[:, h // G, :] @ q[h]) * scale
        p = np.exp(s - s.max())
        out[h] = (p @ v[:, h // G, :]) / p.sum()
    return out


def active_token_index(active_blocks, block: int, n_prompt: int) -> np.ndarray:
    """Prompt token rows of a set of active blocks, ascending (the last prompt block can be short)."""
    return kept_token_index(np.asarray(sorted(active_blocks), dtype=np.int64), block, n_prompt)


# --------------------------------------------------------------------------------------------------
# the pruned prefill layer
# --------------------------------------------------------------------------------------------------
@dataclass
class LayerShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    block: int
    unit: int
    window: int
    rope_theta: float = 500000.0
    rms_eps: float = 1e-5
    scoring: str = "unit"          # "unit": Eq. (1)-(2); "avg" / "max": the pooled baselines of Table 3
    placement: str = "before"      # where a pruning layer drops the blocks: "before" its attention (the
                                   # graded path) or "after" it, as Section 4.1 words it


@dataclass
class LayerWeights:
    """All [out_features, in_features]; gains are vectors of length hidden."""
    g_attn: np.ndarray
    wq: np.ndarray
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray
    g_ffn: np.ndarray
    w_gate: np.ndarray
    w_up: np.ndarray
    w_down: np.ndarray
    # Biases of the Q/K/V projections (length = out_features), None for a model without them.  The
    # paper's second model family (Qwen2.5) has them; its LLaMA family does not.
    bq: np.ndarray | None = None
    bk: np.ndarray | None = None
    bv: np.ndarray | None = None

    def astype(self, dtype):
        return LayerWeights(*[None if getattr(self, f) is None else getattr(self, f).astype(dtype)
                              for f in self.__dataclass_fields__])


def project_heads(h, W, n_heads, head_dim, pos, theta, rope: bool, rounding=None, bias=None):
    """A projection (plus its bias, if the model has one) reshaped to heads, with RoPE at the tokens'
    own positions when asked."""
    y = linear(h, W)
    if bias is not None:
        y = y + bias
    y = y.reshape(h.shape[0], n_heads, head_dim)
    if rope:
        cos, sin = rope_cos_sin(pos, head_dim, theta, h.dtype)
        y = apply_rope(y, cos, sin)
    return _rnd(y, rounding)


def layer_scores(s: LayerShape, w: LayerWeights, x: np.ndarray, pos: np.ndarray, rounding=None):
    """Scoring inputs and Eq. (1)-(2) for one layer: Key states of all tokens, Query states of the
    last min(window, N) tokens (both post-RoPE), then the block scores.  Returns (scores, k)."""
    N = x.shape[0]
    h = _rnd(rmsnorm(x, w.g_attn, s.rms_eps), rounding)
    k = project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bk)
    w_eff = min(s.window, N)
    q_win = project_heads(h[N - w_eff:], w.wq, s.n_q_heads, s.head_dim, pos[N - w_eff:],
                          s.rope_theta, True, rounding, w.bq)
    if s.scoring != "unit":
        return block_scores_pooled(q_win, k, s.block, s.scoring), k
    return block_scores(q_win, k, s.block, s.unit), k


def ffn_residual(s: LayerShape, w: LayerWeights, y: np.ndarray, rounding=None) -> np.ndarray:
    """The "FFN" stage of Fig. 2 with its residual: z = y + Wd (silu(Wg r) * (Wu r)), r = RMSNorm(y)."""
    r = _rnd(rmsnorm(y, w.g_ffn, s.rms_eps), rounding)
    act = _rnd(silu(linear(r, w.w_gate)) * linear(r, w.w_up), rounding)
    return _rnd(y + linear(act, w.w_down), rounding)


def layer_after_selection(s: LayerShape, w: LayerWeights, x: np.ndarray, pos: np.ndarray,
                          kept_blocks: np.ndarray, rows: np.ndarray | None = None, rounding=None, want_y: bool = False):
    """Everything after the block set is known: compact, QKV for the kept tokens (RoPE with the
    original positions), causal GQA attention over the compacted sequence, output projection
    + residual, SwiGLU FFN + residual.  `rows` (indices into the compacted sequence) limits the
    output to a sample of rows; attention for a sampled row still sees every kept key before it.
    Returns (z[rows or n', hidden], pos'[n']), and with want_y also y, the residual stream between the
    attention branch and the FFN (an intermediate of the same computation, handed out unchanged)."""
    xk, posk = compact_tokens(x, pos, kept_blocks, s.block)
    n = xk.shape[0]
    h = _rnd(rmsnorm(xk, w.g_attn, s.rms_eps), rounding)
    k = project_heads(h, w.wk, s.n_kv_heads, s.head_dim, posk, s.rope_theta, True, rounding, w.bk)
    v = project_heads(h, w.wv, s.n_kv_heads, s.head_dim, posk, s.rope_theta, False, rounding, w.bv)
    if rows is None:
        rows = np.arange(n)
    q = project_heads(h[rows], w.wq, s.n_q_heads, s.head_dim, posk[rows], s.rope_theta, True, rounding, w.bq)
    o = _rnd(causal_gqa_attention(q, k, v, rows=rows, rounding=rounding), rounding)
    y = _rnd(xk[rows] + linear(o.reshape(len(rows), -1), w.wo), rounding)
    z = ffn_residual(s, w, y, rounding)
    return (z, posk, y) if want_y else (z, posk)


def layer_after_selection_literal(s: LayerShape, w: LayerWeights, x: np.ndarray, pos: np.ndarray,
                                  kept_blocks: np.ndarray, rows: np.ndarray | None = None, rounding=None,
                                  want_y: bool = False):
    """The placement Section 4.1 describes: the block decision is taken right after Attention, so the
    pruning layer's own attention still sees every incoming token, and the hidden states of the pruned
    blocks are dropped for everything that follows (this layer's output projection and FFN included).
    Queries are only needed for the kept tokens; their keys and values are those of all N tokens.
    `rows` indexes the compacted sequence as in layer_after_selection.  Returns (z, pos')."""
    N = x.shape[0]
    T = kept_token_index(kept_blocks, s.block, N)
    Tr = T if rows is None else T[rows]
    h = _rnd(rmsnorm(x, w.g_attn, s.rms_eps), rounding)
    k = project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bk)
    v = project_heads(h, w.wv, s.n_kv_heads, s.head_dim, pos, s.rope_theta, False, rounding, w.bv)
    q = project_heads(h[Tr], w.wq, s.n_q_heads, s.head_dim, pos[Tr], s.rope_theta, True, rounding, w.bq)
    o = _rnd(causal_gqa_attention(q, k, v, rows=Tr, rounding=rounding), rounding)
    y = _rnd(x[Tr] + linear(o.reshape(len(Tr), -1), w.wo), rounding)
    z = ffn_residual(s, w, y, rounding)
    return (z, pos[T], y) if want_y else (z, pos[T])


def pruned_layer(s: LayerShape, w: LayerWeights, x: np.ndarray, pos: np.ndarray, n_keep: int,
                 force_first: bool = True, force_last: bool = True, rounding=None):
    """One Slim layer: score -> select -> compact -> attention -> FFN on the kept tokens (placement
    "before"), or score -> select -> attention over all tokens -> compact -> FFN (placement "after").
    n_keep >= number of blocks makes it a Preserve layer (nothing dropped).
    Returns dict(z, pos, kept_blocks, scores)."""
    nb = n_blocks(x.shape[0], s.block)
    if n_keep >= nb:
        kept = np.arange(nb, dtype=np.int32)
        scores = None
    else:
        scores, _ = layer_scores(s, w, x, pos, rounding)
        kept = select_blocks(scores, n_keep, force_first, force_last)
    after = layer_after_selection_literal if s.placement == "after" else layer_after_selection
    z, posk = after(s, w, x, pos, kept, rounding=rounding)
    return dict(z=z, pos=posk, kept_blocks=kept, scores=scores)


def decode_layer(s: LayerShape, w: LayerWeights, x_new: np.ndarray, pos_new: int, k_ctx: np.ndarray, v_ctx: np.ndarray,
                 rounding=None):
    """One layer for one newly decoded token (Fig. 2, decoding phase): QKV generation for the token, attention of its
    Query over the context it is given -- the Key/Value states of the prompt tokens of the active blocks and of the
    earlier response tokens, k_ctx/v_ctx[n, Hkv, d] -- plus its own Key/Value, output projection and FFN.
    x_new[hidden], pos_new = the token's position.  Returns (z[hidden], k_new[Hkv, d], v_new[Hkv, d])."""
    x = x_new[None, :]
    pos = np.asarray([pos_new])
    h = _rnd(rmsnorm(x, w.g_attn, s.rms_eps), rounding)
    q = project_heads(h, w.wq, s.n_q_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bq)
    k = project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True, rounding, w.bk)
    v = project_heads(h, w.wv, s.n_kv_heads, s.head_dim, pos, s.rope_theta, False, rounding, w.bv)
    o = _rnd(decode_attention(q[0], np.concatenate([k_ctx, k]), np.concatenate([v_ctx, v])), rounding)
    y = _rnd(x + linear(o.reshape(1, -1), w.wo), rounding)
    r = _rnd(rmsnorm(y, w.g_ffn, s.rms_eps), rounding)
    act = _rnd(silu(linear(r, w.w_gate)) * linear(r, w.w_up), rounding)
    z = _rnd(y + linear(act, w.w_down), rounding)
    return z[0], k[0], v[0]


def prefill_model(s: LayerShape, weights_of_layer, n_layers: int, x: np.ndarray, pos: np.ndarray,
                  schedule: dict, rounding=None):
    """Preserve/Slim schedule (Section 4.1): layers run in order; layer l in `schedule` prunes its
    incoming sequence to ceil(schedule[l] * incoming blocks) blocks, and the surviving set then
    propagates unchanged until the next pruning layer.  `weights_of_layer(l)` supplies the weights.
    Returns (residual stream after the last layer, its positions, list of per-layer kept sets)."""
    kept_log = []
    for l in range(n_layers):
        nb = n_blocks(x.shape[0], s.block)
        n_keep = n_keep_from_ratio(schedule[l], nb) if l in schedule else nb
        res = pruned_layer(s, weights_of_layer(l), x, pos, n_keep, rounding=rounding)
        x, pos = res["z"], res["pos"]
        kept_log.append(res["kept_blocks"])
    return x, pos, kept_log
