"""Pins for the CPU oracle: every function is checked against something that is not itself --
a hand-worked example, a closed form, an invariant, brute force with scalar loops, or a library
routine (torch CPU ops in float64).  No GPU needed."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import slim_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


# ----------------------------------------------------------------------------- helpers
def brute_attention(q, k, v, scale):
    """Causal GQA attention with scalar loops and math.exp (float64)."""
    n, Hq, d = q.shape
    G = Hq // k.shape[1]
    out = np.zeros((n, Hq, d))
    for h in range(Hq):
        g = h // G
        for i in range(n):
            logits = [scale * sum(q[i, h, c] * k[j, g, c] for c in range(d)) for j in range(i + 1)]
            m = max(logits)
            e = [math.exp(l - m) for l in logits]
            den = sum(e)
            for c in range(d):
                out[i, h, c] = sum(e[j] * v[j, g, c] for j in range(i + 1)) / den
    return out


def torch_layer_unpruned(s, w, x, pos):
    """The unpruned layer composed from torch CPU library ops in float64 (HF-style RoPE)."""
    xt = torch.from_numpy(x)
    W = {f: None if getattr(w, f) is None else torch.from_numpy(getattr(w, f)) for f in w.__dataclass_fields__}
    n, d = x.shape[0], s.head_dim
    h = F.rms_norm(xt, (s.hidden,), W["g_attn"], s.rms_eps)
    q = F.linear(h, W["wq"], W["bq"]).view(n, s.n_q_heads, d).transpose(0, 1)
    k = F.linear(h, W["wk"], W["bk"]).view(n, s.n_kv_heads, d).transpose(0, 1)
    v = F.linear(h, W["wv"], W["bv"]).view(n, s.n_kv_heads, d).transpose(0, 1)
    inv = 1.0 / (s.rope_theta ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
    ang = torch.from_numpy(pos.astype(np.float64))[:, None] * inv[None, :]
    emb = torch.cat([ang, ang], dim=-1)
    cos, sin = emb.cos(), emb.sin()

    def rot(t):
        t1, t2 = t[..., : d // 2], t[..., d // 2:]
        return t * cos + torch.cat([-t2, t1], dim=-1) * sin

    q, k = rot(q), rot(k)
    o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True, enable_gqa=True)[0]
    o = o.transpose(0, 1).reshape(n, -1)
    y = xt + F.linear(o, W["wo"])
    r = F.rms_norm(y, (s.hidden,), W["g_ffn"], s.rms_eps)
    z = y + F.linear(F.silu(F.linear(r, W["w_gate"])) * F.linear(r, W["w_up"]), W["w_down"])
    return z.numpy()


def small_layer(seed=0, n=48, hidden=32, Hq=4, Hkv=2, d=8, ffn=40, block=8, unit=4, window=6):
    r = np.random.default_rng(seed)
    s = so.LayerShape(hidden, Hq, Hkv, d, ffn, block, unit, window, rope_theta=500000.0)
    mk = lambda *shp: 0.3 * r.standard_normal(shp)
    w = so.LayerWeights(g_attn=1.0 + 0.1 * r.standard_normal(hidden), wq=mk(Hq * d, hidden),
                        wk=mk(Hkv * d, hidden), wv=mk(Hkv * d, hidden), wo=mk(hidden, Hq * d),
                        g_ffn=1.0 + 0.1 * r.standard_normal(hidden), w_gate=mk(ffn, hidden),
                        w_up=mk(ffn, hidden), w_down=mk(hidden, ffn))
    x = r.standard_normal((n, hidden))
    pos = np.arange(n, dtype=np.int32)
    return s, w, x, pos


# ----------------------------------------------------------------------------- rounding helper
def test_round_bf16_matches_torch():
    a = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(so.round_bf16(a), want)
    assert so.round_bf16(a.astype(np.float64)).dtype == np.float64


# ----------------------------------------------------------------------------- per-token math
def test_rmsnorm_hand_and_invariants():
    x = np.array([[3.0, 4.0]])
    np.testing.assert_allclose(so.rmsnorm(x, np.ones(2), 0.0), x / math.sqrt(12.5), rtol=1e-15)
    np.testing.assert_allclose(so.rmsnorm(x, np.array([2.0, -1.0]), 0.5),
                               np.array([[6.0, -4.0]]) / math.sqrt(13.0), rtol=1e-15)
    y = rng.standard_normal((7, 33))
    h = so.rmsnorm(y, np.ones(33), 0.0)
    np.testing.assert_allclose(np.sqrt((h * h).mean(-1)), 1.0, rtol=1e-12)
    np.testing.assert_allclose(so.rmsnorm(5.0 * y, np.ones(33), 0.0), h, rtol=1e-12)
    g = rng.standard_normal(33)
    want = F.rms_norm(torch.from_numpy(y), (33,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(so.rmsnorm(y, g, 1e-5), want, rtol=1e-12)


def test_linear_is_x_wT():
    h, W = rng.standard_normal((3, 5)), rng.standard_normal((4, 5))
    want = np.array([[sum(h[i, c] * W[o, c] for c in range(5)) for o in range(4)] for i in range(3)])
    np.testing.assert_allclose(so.linear(h, W), want, rtol=1e-13)


def test_rope_closed_form_pairing():
    # d=4, theta=100: inv_freq = (1, 0.1).  Pair (0,2) turns by pos, pair (1,3) by pos/10.
    pos = np.array([0, 1, 7, 1000], dtype=np.int32)
    cos, sin = so.rope_cos_sin(pos, 4, 100.0, np.float64)
    for e, (a, b, f) in {0: (0, 2, 1.0), 1: (1, 3, 0.1)}.items():
        x = np.zeros((4, 1, 4))
        x[:, 0, e] = 1.0
        y = so.apply_rope(x, cos, sin)
        for t, p in enumerate(pos):
            want = np.zeros(4)
            want[a], want[b] = math.cos(p * f), math.sin(p * f)
            np.testing.assert_allclose(y[t, 0], want, atol=1e-12)
    # second element of the pair turns the same way: e_2 -> (-sin, cos)
    x = np.zeros((4, 1, 4))
    x[:, 0, 2] = 1.0
    y = so.apply_rope(x, cos, sin)
    np.testing.assert_allclose(y[2, 0], [-math.sin(7.0), 0, math.cos(7.0), 0], atol=1e-12)


def test_rope_identity_norm_and_relative_position():
    d, H, n = 16, 3, 9
    x = rng.standard_normal((n, H, d))
    c0, s0 = so.rope_cos_sin(np.zeros(n, np.int32), d, 500000.0, np.float64)
    np.testing.assert_array_equal(so.apply_rope(x, c0, s0), x)
    pos = rng.integers(0, 131072, n).astype(np.int32)
    c, s = so.rope_cos_sin(pos, d, 500000.0, np.float64)
    y = so.apply_rope(x, c, s)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # q_m . k_n depends only on m - n
    q, k = rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    dots = []
    for shift in (0, 5, 70000):
        cq, sq = so.rope_cos_sin(np.array([100 + shift]), d, 500000.0, np.float64)
        ck, sk = so.rope_cos_sin(np.array([37 + shift]), d, 500000.0, np.float64)
        dots.append(float((so.apply_rope(q, cq, sq) * so.apply_rope(k, ck, sk)).sum()))
    np.testing.assert_allclose(dots, dots[0], rtol=1e-9)


def test_rope_angles_are_float64_even_for_float32_data():
    pos = np.array([131071], dtype=np.int32)
    c32, s32 = so.rope_cos_sin(pos, 128, 500000.0, np.float32)
    i = 1
    ang = 131071.0 * 500000.0 ** (-2.0 * i / 128)
    assert abs(float(c32[0, i]) - math.cos(ang)) < 1e-7 and abs(float(s32[0, i]) - math.sin(ang)) < 1e-7


def test_silu_matches_library():
    a = rng.standard_normal(100) * 5
    np.testing.assert_allclose(so.silu(a), F.silu(torch.from_numpy(a)).numpy(), rtol=1e-13)


# ----------------------------------------------------------------------------- scoring (Eq. 1-2)
def _read_golden():
    q, k, r = [], [], []
    for line in open(os.path.join(GOLDEN, "score_example.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        {"q": q, "k": k, "r": r}[t[0]].append([float(v) for v in t[1:]])
    return np.array(q).reshape(2, 2, 2), np.array(k).reshape(8, 1, 2), np.array(r).ravel()


def test_scores_hand_worked_example():
    q, k, r = _read_golden()
    np.testing.assert_allclose(so.block_scores(q, k, block=4, unit=2), r, rtol=1e-15)
    np.testing.assert_allclose(so.unit_keys(k[:4], 2)[:, 0], [[2, 1], [0, -2]], rtol=1e-15)
    np.testing.assert_allclose(so.window_query(q), [[2, 0], [0, 2]], rtol=1e-15)


def brute_scores(q_win, k, block, unit):
    """Scalar loops in the re-associated order: per-token head-averaged dot, unit mean, block max."""
    w, Hq, d = q_win.shape
    N, Hkv, _ = k.shape
    G = Hq // Hkv
    tok = []
    for t in range(N):
        acc = 0.0
        for h in range(Hq):
            for c in range(d):
                ql = sum(q_win[i, h, c] for i in range(w)) / w
                acc += ql * k[t, h // G, c]
        tok.append(acc / Hq)
    out = []
    for b0 in range(0, N, block):
        b1 = min(b0 + block, N)
        best = -math.inf
        for u0 in range(b0, b1, unit):
            u1 = min(u0 + unit, b1)
            best = max(best, sum(tok[u0:u1]) / (u1 - u0))
        out.append(best)
    return np.array(out)


@pytest.mark.parametrize("N,block,unit,w,Hq,Hkv,d", [(24, 8, 4, 3, 4, 2, 4), (29, 8, 3, 5, 6, 2, 2),
                                                     (16, 16, 16, 1, 2, 2, 4), (10, 4, 1, 4, 2, 1, 6)])
def test_scores_match_scalar_brute_force_incl_ragged(N, block, unit, w, Hq, Hkv, d):
    q, k = rng.standard_normal((w, Hq, d)), rng.standard_normal((N, Hkv, d))
    np.testing.assert_allclose(so.block_scores(q, k, block, unit), brute_scores(q, k, block, unit),
                               rtol=1e-11, atol=1e-12)


def test_scores_closed_form_cases():
    w, Hq, Hkv, d, B, u, nb = 4, 4, 2, 8, 8, 4, 6
    q = rng.standard_normal((w, Hq, d))
    # all keys identical -> all scores identical
    k = np.tile(rng.standard_normal((1, Hkv, d)), (nb * B, 1, 1))
    r = so.block_scores(q, k, B, u)
    np.testing.assert_allclose(r, r[0], rtol=1e-12)
    # planted unit aligned with the group-summed query wins; scaling one block scales its score
    k = 0.01 * rng.standard_normal((nb * B, Hkv, d))
    ql = q.mean(0)
    qt = ql.reshape(Hkv, Hq // Hkv, d).sum(1)
    k[3 * B + 4:3 * B + 8] = 5.0 * qt
    r = so.block_scores(q, k, B, u)
    assert int(np.argmax(r)) == 3
    np.testing.assert_allclose(r[3], 5.0 * (qt * qt).sum() / Hq, rtol=1e-12)
    k2 = k.copy()
    k2[3 * B:4 * B] *= 2.5
    np.testing.assert_allclose(so.block_scores(q, k2, B, u)[3], 2.5 * r[3], rtol=1e-12)
    # unit == block is the dot with the block-mean key; unit == 1 is the per-token maximum
    k = rng.standard_normal((nb * B, Hkv, d))
    want = [(np.repeat(k[j * B:(j + 1) * B].mean(0), Hq // Hkv, 0) * ql).sum() / Hq for j in range(nb)]
    np.testing.assert_allclose(so.block_scores(q, k, B, B), want, rtol=1e-12)
    tok = (np.repeat(k, Hq // Hkv, 1) * ql[None]).sum((1, 2)) / Hq
    np.testing.assert_allclose(so.block_scores(q, k, B, 1), tok.reshape(nb, B).max(1), rtol=1e-12)
    # a max over units is never below the block-average score and never above the per-token max
    r8 = so.block_scores(q, k, B, u)
    assert (r8 >= np.array(want) - 1e-12).all() and (r8 <= tok.reshape(nb, B).max(1) + 1e-12).all()


def test_short_trailing_unit_is_averaged_over_its_own_tokens():
    # block 7, unit 3: units of 3, 3 and 1 tokens.  Only the lone token of the short unit carries a key, aligned
    # with the group-summed window query, so that unit wins and its mean is that token's key itself.
    w, Hq, Hkv, d, B, u = 2, 4, 2, 4, 7, 3
    q = rng.standard_normal((w, Hq, d))
    qt = q.mean(0).reshape(Hkv, Hq // Hkv, d).sum(1)
    k = np.zeros((2 * B, Hkv, d))
    k[2 * B - 1] = 3.0 * qt
    np.testing.assert_array_equal(so.unit_keys(k[B:], u)[2], k[2 * B - 1])
    r = so.block_scores(q, k, B, u)
    np.testing.assert_allclose(r, [0.0, 3.0 * (qt * qt).sum() / Hq], rtol=1e-12)
    # the same with a short last BLOCK: 9 tokens = a block of 7 and one of 2 (a single unit of 2 tokens)
    k = np.zeros((9, Hkv, d))
    k[7], k[8] = 1.0 * qt, 3.0 * qt
    np.testing.assert_allclose(so.block_scores(q, k, B, u)[1], 2.0 * (qt * qt).sum() / Hq, rtol=1e-12)


def test_scores_head_mapping_is_grouped_not_interleaved():
    # Hq=4, Hkv=2: heads 0,1 read kv head 0; heads 2,3 read kv head 1.
    d = 2
    q = np.zeros((1, 4, d))
    q[0, 1] = [1.0, 0.0]          # only query head 1 is non-zero -> must read kv head 0
    k = np.zeros((2, 2, d))
    k[:, 0] = [4.0, 0.0]
    k[:, 1] = [-100.0, 0.0]
    np.testing.assert_allclose(so.block_scores(q, k, 2, 1), [1.0], rtol=1e-15)   # 4 / Hq


def brute_pooled(q_win, k, block, pooling):
    """Scalar loops from the description of the two baselines (Table 3): one pooled key per block."""
    w, Hq, d = q_win.shape
    N, Hkv, _ = k.shape
    G = Hq // Hkv
    out = []
    for b0 in range(0, N, block):
        b1 = min(b0 + block, N)
        acc = 0.0
        for h in range(Hq):
            for c in range(d):
                ql = sum(q_win[i, h, c] for i in range(w)) / w
                vals = [k[t, h // G, c] for t in range(b0, b1)]
                acc += ql * (sum(vals) / len(vals) if pooling == "avg" else max(vals))
        out.append(acc / Hq)
    return np.array(out)


@pytest.mark.parametrize("pooling", ["avg", "max"])
@pytest.mark.parametrize("N,block,w,Hq,Hkv,d", [(24, 8, 3, 4, 2, 4), (29, 8, 5, 6, 2, 2), (10, 4, 4, 2, 1, 6)])
def test_pooled_scores_match_scalar_brute_force_incl_ragged(pooling, N, block, w, Hq, Hkv, d):
    q, k = rng.standard_normal((w, Hq, d)), rng.standard_normal((N, Hkv, d))
    np.testing.assert_allclose(so.block_scores_pooled(q, k, block, pooling), brute_pooled(q, k, block, pooling),
                               rtol=1e-11, atol=1e-12)


def test_pooled_scores_special_cases():
    w, Hq, Hkv, d, B, nb = 3, 4, 2, 8, 8, 5
    q = rng.standard_normal((w, Hq, d))
    k = rng.standard_normal((nb * B, Hkv, d))
    # average pooling is Eq. (1)-(2) with a single TokenUnit per block
    np.testing.assert_allclose(so.block_scores_pooled(q, k, B, "avg"), so.block_scores(q, k, B, B), rtol=1e-12)
    # keys constant inside each block: every pooling and every unit size agree
    kc = np.repeat(rng.standard_normal((nb, Hkv, d)), B, axis=0)
    ref = so.block_scores(q, kc, B, 1)
    np.testing.assert_allclose(so.block_scores_pooled(q, kc, B, "max"), ref, rtol=1e-12)
    np.testing.assert_allclose(so.block_scores_pooled(q, kc, B, "avg"), ref, rtol=1e-12)
    # d = 1, one head, positive query: max pooling is q times the largest key of the block; with a negative
    # query it still takes the element-wise maximum (the pooled key does not depend on the query)
    k1 = rng.standard_normal((4 * B, 1, 1))
    q1 = np.full((2, 1, 1), 0.7)
    np.testing.assert_allclose(so.block_scores_pooled(q1, k1, B, "max"), 0.7 * k1.reshape(4, B).max(1), rtol=1e-12)
    np.testing.assert_allclose(so.block_scores_pooled(-q1, k1, B, "max"), -0.7 * k1.reshape(4, B).max(1), rtol=1e-12)
    # the order of the tokens inside a block does not matter; raising a key element never lowers the score
    # where the query element is positive
    perm = np.concatenate([j * B + rng.permutation(B) for j in range(nb)])
    for pooling in ("avg", "max"):
        np.testing.assert_allclose(so.block_scores_pooled(q, k[perm], B, pooling),
                                   so.block_scores_pooled(q, k, B, pooling), rtol=1e-12)
    qpos = np.abs(q)
    k2 = k.copy()
    k2[5, 1, 3] += 10.0
    assert (so.block_scores_pooled(qpos, k2, B, "max") >= so.block_scores_pooled(qpos, k, B, "max") - 1e-12).all()
    # grouped head mapping, as in Eq. (2)
    qh = np.zeros((1, 4, 2)); qh[0, 1] = [1.0, 0.0]
    kh = np.zeros((2, 2, 2)); kh[:, 0] = [[4.0, 0.0], [2.0, 0.0]]; kh[:, 1] = [-100.0, 0.0]
    np.testing.assert_allclose(so.block_scores_pooled(qh, kh, 2, "max"), [1.0], rtol=1e-15)
    np.testing.assert_allclose(so.block_scores_pooled(qh, kh, 2, "avg"), [0.75], rtol=1e-15)


# ----------------------------------------------------------------------------- selection
def valid_selection(scores, kept, n_keep, ff, fl):
    nb = len(scores)
    forced = ({0} if ff else set()) | ({nb - 1} if fl else set())
    S = set(int(j) for j in kept)
    if len(kept) != min(n_keep, nb) or list(kept) != sorted(S) or not forced <= S:
        return False
    for a in S - forced:
        for b in set(range(nb)) - S:
            if not (scores[a] > scores[b] or (scores[a] == scores[b] and a < b)):
                return False
    return True


def test_select_exhaustive_small():
    for nb in range(2, 7):
        for vals in itertools.product([0.0, 1.0, -2.5], repeat=nb):
            sc = np.array(vals)
            for ff, fl in ((True, True), (True, False), (False, False)):
                for n_keep in range(int(ff) + int(fl), nb + 2):
                    kept = so.select_blocks(sc, n_keep, ff, fl)
                    assert kept.dtype == np.int32
                    assert valid_selection(sc, kept, n_keep, ff, fl), (vals, n_keep, ff, fl, kept)


def test_select_matches_sort_all_take_k_and_invariants():
    for _ in range(50):
        nb = int(rng.integers(3, 200))
        sc = np.round(rng.standard_normal(nb), 1)          # many ties
        n_keep = int(rng.integers(2, nb + 1))
        kept = so.select_blocks(sc, n_keep)
        order = np.lexsort((np.arange(1, nb - 1), -sc[1:nb - 1])) + 1
        want = np.sort(np.concatenate([[0, nb - 1], order[:n_keep - 2]])) if n_keep < nb else np.arange(nb)
        np.testing.assert_array_equal(kept, want)
        assert len(set(kept)) == len(kept) == n_keep and kept[0] == 0 and kept[-1] == nb - 1
        assert (np.diff(kept) > 0).all()


def test_selection_cut_band():
    sc = np.array([9.0, 0.5, 0.3, 0.7, 0.1, 9.0])
    assert so.selection_cut(sc, 4) == pytest.approx(0.4)         # takes 0.7, 0.5 ; next 0.3
    assert so.selection_cut(sc, 6) is None
    assert so.selection_cut(sc, 2) > 0.7


def test_keep_counts_of_the_workloads():
    assert [so.n_keep_from_ratio(r, nb) for r, nb in ((0.5, 32), (0.5, 128), (0.3, 512), (0.2, 1024))] \
        == [16, 64, 154, 205]
    assert [so.n_keep_from_ratio(r, nb) for r, nb in ((0.5, 512), (0.25, 256), (0.125, 64))] == [256, 64, 8]
    assert so.n_keep_from_ratio(0.0, 10) == 2 and so.n_keep_from_ratio(1.0, 10) == 10
    assert so.n_keep_from_ratio(0.5, 1) == 1


# ----------------------------------------------------------------------------- compaction
def test_compaction_is_indexing():
    N, B = 45, 8                                           # ragged last block (5 tokens)
    x = rng.standard_normal((N, 6))
    pos = (np.arange(N) * 3 + 1).astype(np.int32)
    kept = np.array([0, 2, 5], dtype=np.int32)
    xs, ps = so.compact_tokens(x, pos, kept, B)
    T = list(range(0, 8)) + list(range(16, 24)) + list(range(40, 45))
    np.testing.assert_array_equal(xs, x[T])
    np.testing.assert_array_equal(ps, pos[T])
    assert (np.diff(ps) > 0).all() and len(T) == (3 - 1) * B + (N - 5 * B)


# ----------------------------------------------------------------------------- attention
@pytest.mark.parametrize("n,Hq,Hkv,d", [(1, 1, 1, 2), (7, 2, 1, 4), (13, 6, 2, 3), (20, 4, 4, 8)])
def test_attention_vs_scalar_brute_force(n, Hq, Hkv, d):
    q, k, v = rng.standard_normal((n, Hq, d)), rng.standard_normal((n, Hkv, d)), rng.standard_normal((n, Hkv, d))
    got = so.causal_gqa_attention(q, k, v, chunk=5)
    np.testing.assert_allclose(got, brute_attention(q, k, v, 1 / math.sqrt(d)), rtol=1e-11, atol=1e-13)


def test_attention_vs_torch_sdpa_and_special_cases():
    n, Hq, Hkv, d = 70, 8, 2, 16
    q, k, v = rng.standard_normal((n, Hq, d)), rng.standard_normal((n, Hkv, d)), rng.standard_normal((n, Hkv, d))
    got = so.causal_gqa_attention(q, k, v, chunk=32)
    t = lambda a: torch.from_numpy(a).transpose(0, 1)[None]
    want = F.scaled_dot_product_attention(t(q), t(k), t(v), is_causal=True, enable_gqa=True)[0].transpose(0, 1)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)
    # row 0 attends only to itself
    np.testing.assert_allclose(got[0], np.repeat(v[0], Hq // Hkv, 0), rtol=1e-13)
    # equal logits -> running mean of V
    flat = so.causal_gqa_attention(np.zeros_like(q), k, v)
    run = np.cumsum(v, 0) / np.arange(1, n + 1)[:, None, None]
    np.testing.assert_allclose(flat, np.repeat(run, Hq // Hkv, 1), rtol=1e-12)
    # GQA == MHA on duplicated kv heads
    mha = so.causal_gqa_attention(q, np.repeat(k, 4, 1), np.repeat(v, 4, 1))
    np.testing.assert_allclose(got, mha, rtol=1e-13)
    # explicit scale, and a sample of rows equals those rows of the full result
    np.testing.assert_allclose(so.causal_gqa_attention(q, k, v, scale=0.0), flat, rtol=1e-12)
    rows = np.array([0, 3, 31, 32, 69])
    np.testing.assert_allclose(so.causal_gqa_attention(q[rows], k, v, rows=rows), got[rows], rtol=1e-12)


def test_attention_is_stable_for_large_logits():
    n, d = 5, 4
    q = np.full((n, 1, d), 300.0)
    k = np.full((n, 1, d), 300.0)
    k[2] *= 2
    v = np.arange(n * d, dtype=np.float64).reshape(n, 1, d)
    out = so.causal_gqa_attention(q, k, v)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out[4, 0], v[2, 0], rtol=1e-12)     # the huge logit takes everything


# ----------------------------------------------------------------------------- decode-time pieces
def test_scores_from_stored_unit_keys_equal_eq_1_2_incl_ragged():
    for (N, block, unit, w, Hq, Hkv, d) in [(24, 8, 4, 3, 4, 2, 4), (29, 8, 3, 5, 6, 2, 2), (10, 4, 1, 4, 2, 1, 6)]:
        q, k = rng.standard_normal((w, Hq, d)), rng.standard_normal((N, Hkv, d))
        kr = so.all_unit_keys(k, block, unit)
        assert kr.shape == (so.n_blocks(N, block), -(-block // unit), Hkv, d)
        np.testing.assert_allclose(so.block_scores_from_unit_keys(q, kr), brute_scores(q, k, block, unit),
                                   rtol=1e-11, atol=1e-12)
        # the stored means are the plain means of the units' tokens; missing units are marked
        np.testing.assert_allclose(kr[0, 0], k[:unit].mean(0), rtol=1e-13)
        last_len = N - (kr.shape[0] - 1) * block
        assert np.isnan(kr[-1, -(-last_len // unit):]).all() and not np.isnan(kr[-1, 0]).any()


def test_kv_swap_hand_worked_and_invariants():
    # worked by hand from Algorithm 1: 8 blocks, 4 active
    r = so.kv_swap_step({0, 1, 2, 3}, {0, 1, 4, 5}, {4, 5, 6, 7}, 0.9)
    assert r["overlap"] == 0.5 and r["swapped"]
    assert r["active"] == {0, 1, 4, 5} and r["offload"] == {2, 3} and r["load"] == {4, 5}
    assert r["memory"] == {2, 3, 4, 5, 6, 7}
    # block 2 already has a copy in the pool: its GPU memory is released without a transfer
    r = so.kv_swap_step({0, 1, 2, 3}, {0, 1, 4, 5}, {2, 4, 5, 6, 7}, 0.9)
    assert r["offload"] == {3} and r["load"] == {4, 5} and r["memory"] == {2, 3, 4, 5, 6, 7}
    # 3 of 4 candidates resident: 0.75 >= gamma 0.75 keeps the old set (the test is strict "<"), 0.76 swaps
    r = so.kv_swap_step({0, 1, 2, 3}, {0, 1, 2, 7}, {4, 5, 6, 7}, 0.75)
    assert not r["swapped"] and r["active"] == {0, 1, 2, 3} and not r["offload"] and not r["load"]
    assert so.kv_swap_step({0, 1, 2, 3}, {0, 1, 2, 7}, {4, 5, 6, 7}, 0.76)["swapped"]
    # the overlap is a fraction of the CANDIDATE set (Algorithm 1), not of the resident one: 3 of 4 candidates are
    # among 8 resident blocks -> 0.75, no swap at gamma 0.5 (3/8 would swap); 1 of 2 -> 0.5, swap at gamma 0.6
    r = so.kv_swap_step(set(range(8)), {0, 1, 2, 9}, {8, 9, 10}, 0.5)
    assert r["overlap"] == 0.75 and not r["swapped"]
    r = so.kv_swap_step(set(range(8)), {0, 9}, {8, 9, 10}, 0.6)
    assert r["overlap"] == 0.5 and r["swapped"] and r["load"] == {9} and r["offload"] == set(range(1, 8))
    # gamma = 0 never swaps; gamma > 1 always takes the candidate set, with nothing to move when it is the old set
    assert not so.kv_swap_step({0, 1}, {2, 3}, {2, 3}, 0.0)["swapped"]
    r = so.kv_swap_step({0, 1}, {0, 1}, {5}, 1.5)
    assert r["swapped"] and r["overlap"] == 1.0 and not r["offload"] and not r["load"]
    # random walks: set sizes stay fixed, every block is on the GPU or in the pool, traffic only on swaps
    g = np.random.default_rng(3)
    nb, na = 40, 10
    active, memory = set(range(na)), set(range(na, nb))
    for _ in range(200):
        cand = {0} | set(g.choice(np.arange(1, nb), na - 1, replace=False).tolist())
        prev = set(active)
        r = so.kv_swap_step(active, cand, memory, 0.6)
        active, memory = r["active"], r["memory"]
        assert len(active) == na and active in (cand, prev)
        assert set(range(nb)) == active | memory
        assert r["load"].isdisjoint(prev) and r["offload"] <= prev - active and len(r["load"]) == len(prev - active)
        assert r["swapped"] == (len(cand & prev) / na < 0.6)


# ----------------------------------------------------------------------------- the layer
def test_unpruned_layer_equals_torch_library_composition():
    s, w, x, pos = small_layer(seed=3)
    res = so.pruned_layer(s, w, x, pos, n_keep=10**6)
    np.testing.assert_allclose(res["z"], torch_layer_unpruned(s, w, x, pos), rtol=1e-9, atol=1e-11)
    np.testing.assert_array_equal(res["kept_blocks"], np.arange(6))
    np.testing.assert_array_equal(res["pos"], pos)


def test_keep_ratio_one_is_exactly_the_unpruned_layer():
    s, w, x, pos = small_layer(seed=4, n=45)              # ragged last block
    nb = so.n_blocks(45, s.block)
    a = so.pruned_layer(s, w, x, pos, n_keep=so.n_keep_from_ratio(1.0, nb))
    b = so.layer_after_selection(s, w, x, pos, np.arange(nb, dtype=np.int32))[0]
    np.testing.assert_array_equal(a["z"], b)
    np.testing.assert_allclose(a["z"], torch_layer_unpruned(s, w, x, pos), rtol=1e-9, atol=1e-11)


def test_the_intermediate_y_is_the_layer_with_a_zero_down_projection():
    """want_y hands out the residual stream between the two branches: it is what the layer returns when the FFN
    branch contributes nothing, in both placements and on sampled rows, and z is untouched by the request."""
    import dataclasses
    s, w, x, pos = small_layer(seed=21, n=45)
    kept = np.array([0, 2, 5], dtype=np.int32)
    w0 = dataclasses.replace(w, w_down=np.zeros_like(w.w_down))
    for fn in (so.layer_after_selection, so.layer_after_selection_literal):
        for rows in (None, np.array([0, 3, 9, 12])):
            z, p, y = fn(s, w, x, pos, kept, rows=rows, want_y=True)
            np.testing.assert_array_equal(z, fn(s, w, x, pos, kept, rows=rows)[0])
            np.testing.assert_array_equal(y, fn(s, w0, x, pos, kept, rows=rows)[0])
            assert np.abs(z - y).max() > 1e-3


def test_bf16_spacing_used_by_the_gpu_tolerances():
    from tests.helpers import ulp_bf16
    a = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-4, 4, 2000), [1.0, 2.0, 0.5, 7.999, 8.0, 15.99]])
    t = torch.from_numpy(np.abs(a)).to(torch.float32).to(torch.bfloat16)          # a bf16 value in the same binade or the next
    up = torch.nextafter(t, torch.tensor(float("inf"), dtype=torch.bfloat16))
    np.testing.assert_array_equal(ulp_bf16(t.double().numpy()), (up.double() - t.double()).numpy())
    assert ulp_bf16(np.array([8.0]))[0] == 0.0625 and ulp_bf16(np.array([-7.99]))[0] == 0.03125


def test_pruned_layer_uses_original_positions_and_kept_tokens_only():
    s, w, x, pos = small_layer(seed=5, n=64)
    res = so.pruned_layer(s, w, x, pos, n_keep=4)
    kept = res["kept_blocks"]
    assert len(kept) == 4 and kept[0] == 0 and kept[-1] == 7
    T = so.kept_token_index(kept, s.block, 64)
    np.testing.assert_array_equal(res["pos"], pos[T])
    # the same result from the library composition on the gathered rows with their old positions
    np.testing.assert_allclose(res["z"], torch_layer_unpruned(s, w, x[T], pos[T]), rtol=1e-9, atol=1e-11)
    # and it does differ from re-numbering the positions 0..n'-1 (RoPE sees the original ones)
    renum = torch_layer_unpruned(s, w, x[T], np.arange(len(T), dtype=np.int32))
    assert np.abs(renum - res["z"]).max() > 1e-3
    # scores used by the layer are Eq. (2) on that layer's own post-RoPE Q/K
    sc, k = so.layer_scores(s, w, x, pos)
    np.testing.assert_array_equal(sc, res["scores"])
    np.testing.assert_array_equal(so.select_blocks(sc, 4), kept)
    xt = torch.from_numpy(x)
    h = F.rms_norm(xt, (s.hidden,), torch.from_numpy(w.g_attn), s.rms_eps).numpy()
    c, sn = so.rope_cos_sin(pos, s.head_dim, s.rope_theta, np.float64)
    k_lib = so.apply_rope((h @ w.wk.T).reshape(64, s.n_kv_heads, s.head_dim), c, sn)
    q_lib = so.apply_rope((h @ w.wq.T).reshape(64, s.n_q_heads, s.head_dim), c, sn)[64 - s.window:]
    np.testing.assert_allclose(sc, brute_scores(q_lib, k_lib, s.block, s.unit), rtol=1e-9, atol=1e-12)


def test_prefix_selection_equals_prefix_of_unpruned_layer():
    s, w, x, pos = small_layer(seed=6, n=64)
    full = so.pruned_layer(s, w, x, pos, n_keep=8)["z"]
    z, p = so.layer_after_selection(s, w, x, pos, np.arange(3, dtype=np.int32))
    np.testing.assert_allclose(z, full[:24], rtol=1e-10, atol=1e-12)     # causal: never looks right
    # with the last block forced as well, every row before the last block is still a prefix row
    z2, _ = so.layer_after_selection(s, w, x, pos, np.array([0, 1, 2, 7], dtype=np.int32))
    np.testing.assert_allclose(z2[:24], full[:24], rtol=1e-10, atol=1e-12)
    assert np.abs(z2[24:] - full[56:]).max() > 1e-6


def test_sampled_rows_equal_rows_of_full_result():
    s, w, x, pos = small_layer(seed=7, n=64)
    kept = np.array([0, 2, 3, 6, 7], dtype=np.int32)
    full, _ = so.layer_after_selection(s, w, x, pos, kept)
    rows = np.array([0, 7, 8, 21, 39])
    part, _ = so.layer_after_selection(s, w, x, pos, kept, rows=rows)
    np.testing.assert_allclose(part, full[rows], rtol=1e-11, atol=1e-13)


def test_per_token_steps_commute_with_gather():
    s, w, x, pos = small_layer(seed=8, n=40)
    T = so.kept_token_index(np.array([0, 3, 4]), s.block, 40)
    h = so.rmsnorm(x, w.g_attn, s.rms_eps)
    np.testing.assert_array_equal(so.rmsnorm(x[T], w.g_attn, s.rms_eps), h[T])
    k_all = so.project_heads(h, w.wk, s.n_kv_heads, s.head_dim, pos, s.rope_theta, True)
    k_sub = so.project_heads(h[T], w.wk, s.n_kv_heads, s.head_dim, pos[T], s.rope_theta, True)
    np.testing.assert_allclose(k_sub, k_all[T], rtol=1e-12, atol=1e-14)


def test_bf16_rounding_mode_stays_close_and_on_grid():
    s, w, x, pos = small_layer(seed=9, n=32)
    a = so.pruned_layer(s, w, x, pos, n_keep=3)
    b = so.pruned_layer(s, w, x, pos, n_keep=3, rounding="bf16")
    np.testing.assert_array_equal(b["z"], so.round_bf16(b["z"]))
    assert 0 < np.abs(a["z"] - b["z"]).max() < 0.2


def test_placement_after_attention_is_the_unpruned_layer_at_the_kept_tokens():
    """Section 4.1's wording: the pruning layer's own attention still sees every token, the blocks are
    dropped afterwards.  Every later step is per token, so the result must be the rows of the unpruned
    layer (pinned above against the library composition) at the kept tokens, with the same kept set and
    scores as the graded placement."""
    import dataclasses
    s, w, x, pos = small_layer(seed=11, n=61)             # ragged last block
    pos = pos + 100
    lit = dataclasses.replace(s, placement="after")
    a = so.pruned_layer(lit, w, x, pos, n_keep=4)
    b = so.pruned_layer(s, w, x, pos, n_keep=4)
    np.testing.assert_array_equal(a["kept_blocks"], b["kept_blocks"])
    np.testing.assert_array_equal(a["scores"], b["scores"])
    np.testing.assert_array_equal(a["pos"], b["pos"])
    T = so.kept_token_index(a["kept_blocks"], s.block, 61)
    full = torch_layer_unpruned(s, w, x, pos)
    np.testing.assert_allclose(a["z"], full[T], rtol=1e-9, atol=1e-11)
    # it differs from the graded placement exactly where a kept token follows a dropped block
    first_gap = next(j for j in range(len(a["kept_blocks"])) if a["kept_blocks"][j] != j)
    lead = first_gap * s.block
    np.testing.assert_allclose(a["z"][:lead], b["z"][:lead], rtol=1e-9, atol=1e-11)
    assert np.abs(a["z"][lead:] - b["z"][lead:]).max() > 1e-3
    # keep-all: both placements are the unpruned layer; sampled rows equal rows of the full result
    nb = so.n_blocks(61, s.block)
    np.testing.assert_array_equal(so.pruned_layer(lit, w, x, pos, nb)["z"], so.pruned_layer(s, w, x, pos, nb)["z"])
    rows = np.array([0, 7, 8, 20, len(T) - 1])
    z_rows, _ = so.layer_after_selection_literal(lit, w, x, pos, a["kept_blocks"], rows=rows)
    np.testing.assert_allclose(z_rows, a["z"][rows], rtol=1e-12, atol=1e-13)


def test_qkv_biases_enter_before_rope_and_match_the_library_layer():
    """Second model family of the paper (Qwen2.5): Q/K/V projections carry a bias.  Pinned against the torch
    composition (F.linear with bias, HF-style RoPE afterwards); zero biases change nothing; the window
    query and the Key states that the scores read include the bias."""
    import dataclasses
    s, w, x, pos = small_layer(seed=21, n=40, Hq=6, Hkv=2)          # 3 query heads per kv head
    r = np.random.default_rng(5)
    wb = dataclasses.replace(w, bq=r.standard_normal(6 * 8), bk=r.standard_normal(2 * 8), bv=r.standard_normal(2 * 8))
    full = so.pruned_layer(s, wb, x, pos, n_keep=10**6)
    np.testing.assert_allclose(full["z"], torch_layer_unpruned(s, wb, x, pos), rtol=1e-9, atol=1e-11)
    assert np.abs(full["z"] - so.pruned_layer(s, w, x, pos, n_keep=10**6)["z"]).max() > 1e-2
    wz = dataclasses.replace(w, bq=np.zeros(48), bk=np.zeros(16), bv=np.zeros(16))
    np.testing.assert_array_equal(so.pruned_layer(s, wz, x, pos, 3)["z"], so.pruned_layer(s, w, x, pos, 3)["z"])
    # scores: keys and window queries with bias, by hand from the definitions
    h = so.rmsnorm(x, wb.g_attn, s.rms_eps)
    cos, sin = so.rope_cos_sin(pos, s.head_dim, s.rope_theta, np.float64)
    k = so.apply_rope((h @ wb.wk.T + wb.bk).reshape(40, 2, 8), cos, sin)
    q = so.apply_rope((h @ wb.wq.T + wb.bq).reshape(40, 6, 8), cos, sin)[-s.window:]
    np.testing.assert_allclose(so.layer_scores(s, wb, x, pos)[0], so.block_scores(q, k, s.block, s.unit), rtol=1e-12)
    # pruned layer with biases equals the library layer on the gathered rows when the kept set is a prefix
    res = so.layer_after_selection(s, wb, x, pos, np.array([0, 1, 2], dtype=np.int32))[0]
    np.testing.assert_allclose(res, torch_layer_unpruned(s, wb, x[:24], pos[:24]), rtol=1e-9, atol=1e-11)


def test_schedule_runs_pruning_layers_on_incoming_blocks():
    s, w, x, pos = small_layer(seed=10, n=64)
    ws = [w, small_layer(seed=11)[1], small_layer(seed=12)[1]]
    z, p, log = so.prefill_model(s, lambda l: ws[l], 3, x, pos, {1: 0.5, 2: 0.5})
    assert [len(k) for k in log] == [8, 4, 2] and z.shape == (16, s.hidden)
    r0 = so.pruned_layer(s, ws[0], x, pos, 8)
    r1 = so.pruned_layer(s, ws[1], r0["z"], r0["pos"], 4)
    r2 = so.pruned_layer(s, ws[2], r1["z"], r1["pos"], 2)
    np.testing.assert_array_equal(z, r2["z"])
    np.testing.assert_array_equal(p, r2["pos"])
    # the surviving positions are whole original blocks, first and last among them
    assert p[0] == 0 and p[-1] == 63 and all(p[i * 8] % 8 == 0 for i in range(2))


# --------------------------------------------------------------------------------------------- decode attention
def test_decode_attention_is_the_last_row_of_causal_attention_and_brute_force():
    """A new token sees every key it is given: that is the last row of causal attention over the same sequence
    (pinned above against scalar loops and torch), a scalar-loop brute force, and it does not depend on key order."""
    g = np.random.default_rng(21)
    n, Hq, Hkv, d = 37, 6, 2, 16
    q, k, v = g.standard_normal((n, Hq, d)), g.standard_normal((n, Hkv, d)), g.standard_normal((n, Hkv, d))
    full = so.causal_gqa_attention(q, k, v)
    got = so.decode_attention(q[-1], k, v)
    np.testing.assert_allclose(got, full[-1], rtol=1e-12, atol=1e-12)
    G = Hq // Hkv
    for h in range(Hq):
        w = [math.exp(sum(q[-1, h, c] * k[j, h // G, c] for c in range(d)) / math.sqrt(d)) for j in range(n)]
        for c in (0, d - 1):
            want = sum(w[j] * v[j, h // G, c] for j in range(n)) / sum(w)
            assert abs(got[h, c] - want) < 1e-12
    perm = g.permutation(n)
    np.testing.assert_allclose(so.decode_attention(q[-1], k[perm], v[perm]), got, rtol=1e-12, atol=1e-12)
    # one key: the output is that key's value; a custom scale of 0 averages the values
    np.testing.assert_allclose(so.decode_attention(q[-1], k[:1], v[:1]), np.repeat(v[0], G, axis=0), rtol=1e-12)
    np.testing.assert_allclose(so.decode_attention(q[-1], k, v, scale=0.0), np.repeat(v.mean(axis=0), G, axis=0), rtol=1e-12)
    # active blocks -> token rows (ragged last block)
    np.testing.assert_array_equal(so.active_token_index({2, 0, 4}, 8, 37), list(range(0, 8)) + list(range(16, 24)) + list(range(32, 37)))


def test_decode_layer_is_the_last_row_of_the_prefill_layer():
    """Decoding token n-1 with the Key/Value states of tokens 0..n-2 as its context is the unpruned prefill layer's
    last row (that layer is pinned above against a torch composition); the token's own K/V are those rows too."""
    g = np.random.default_rng(31)
    n, hidden, Hq, Hkv, d, ffn = 21, 48, 4, 2, 16, 80
    s = so.LayerShape(hidden, Hq, Hkv, d, ffn, 8, 4, 4, 10000.0, 1e-5)
    mk = lambda *shape: g.standard_normal(shape) * 0.2
    w = so.LayerWeights(1.0 + 0.1 * g.standard_normal(hidden), mk(Hq * d, hidden), mk(Hkv * d, hidden), mk(Hkv * d, hidden),
                        mk(hidden, Hq * d), 1.0 + 0.1 * g.standard_normal(hidden), mk(ffn, hidden), mk(ffn, hidden),
                        mk(hidden, ffn), mk(Hq * d), mk(Hkv * d), mk(Hkv * d))
    x = g.standard_normal((n, hidden))
    pos = np.sort(g.choice(500, n, replace=False))
    full = so.pruned_layer(s, w, x, pos, n_keep=99)                       # Preserve layer: every row
    h = so.rmsnorm(x, w.g_attn, s.rms_eps)
    k_all = so.project_heads(h, w.wk, Hkv, d, pos, s.rope_theta, True, None, w.bk)
    v_all = so.project_heads(h, w.wv, Hkv, d, pos, s.rope_theta, False, None, w.bv)
    z, k_new, v_new = so.decode_layer(s, w, x[-1], int(pos[-1]), k_all[:-1], v_all[:-1])
    np.testing.assert_allclose(z, full["z"][-1], rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(k_new, k_all[-1], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v_new, v_all[-1], rtol=1e-12, atol=1e-12)
    # with no context the token attends to itself only: attention output = its own value
    z0, _, v0 = so.decode_layer(s, w, x[0], int(pos[0]), k_all[:0], v_all[:0])
    np.testing.assert_allclose(z0, full["z"][0], rtol=1e-10, atol=1e-10)
