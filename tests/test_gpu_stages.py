"""GPU parity, stage by stage: every C entry point against the CPU oracle on the same seeded inputs,
element by element.  Sizes span several tiles and a ragged tail."""
import math

import numpy as np
import pytest
import torch

from oracle import slim_oracle as so
from paper_2508_06447_amd import inputs
from tests.helpers import MAX_ABS, MEAN_ABS, errs, f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def slim():
    import paper_2508_06447_amd as slim
    slim.load_library()
    return slim


def dev(t):
    return t.cuda()


def rand(shape, dtype, seed, scale=1.0):
    g = np.random.default_rng(seed)
    t = torch.from_numpy((scale * g.standard_normal(shape)).astype(np.float32))
    return t.to(dtype)


# ------------------------------------------------------------------------------------------ compaction
@pytest.mark.parametrize("N,block,row,dtype", [
    (512, 16, 256, torch.float32), (8192, 64, 4096, torch.bfloat16), (1000, 64, 1024, torch.bfloat16),
    (45, 8, 6, torch.float32), (45, 8, 3, torch.bfloat16), (333, 32, 10, torch.bfloat16), (64, 64, 8, torch.float32),
])
def test_compact_is_bit_exact(slim, N, block, row, dtype):
    print(f"compact N={N} block={block} row={row} {dtype}", flush=True)
    g = np.random.default_rng(N + row)
    nb = slim.n_blocks(N, block)
    src = rand((N, row), dtype, seed=N)
    pos = torch.from_numpy(np.sort(g.choice(10 * N, N, replace=False)).astype(np.int32))
    for n_keep in sorted({1, max(1, nb // 3), nb}):
        others = np.sort(g.choice(nb - 1, n_keep - 1, replace=False)) if n_keep > 1 else np.zeros(0, np.int64)
        kept = np.concatenate([others, [nb - 1]]).astype(np.int32)
        dst, pos_out = slim.slim_compact_tokens(dev(src), dev(torch.from_numpy(kept)), block, dev(pos))
        want_x, want_p = so.compact_tokens(src.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).numpy(),
                                           pos.numpy(), kept, block)
        got = dst.cpu().view(torch.int16 if dtype == torch.bfloat16 else torch.int32).numpy()
        np.testing.assert_array_equal(got, want_x)
        np.testing.assert_array_equal(pos_out.cpu().numpy(), want_p)
        assert dst.shape[0] == slim.kept_tokens(N, block, n_keep)
    # without the last block (N multiple of block only) and without positions
    if N % block == 0 and nb > 2:
        kept = np.array([0, nb - 2], dtype=np.int32)
        dst, p = slim.slim_compact_tokens(dev(src), dev(torch.from_numpy(kept)), block, None, want_pos=True)
        np.testing.assert_array_equal(f64(dst), f64(src)[so.kept_token_index(kept, block, N)])
        np.testing.assert_array_equal(p.cpu().numpy(), so.kept_token_index(kept, block, N))


def test_compact_3d_keys(slim):
    k = rand((640, 8, 128), torch.bfloat16, seed=5)
    kept = torch.tensor([0, 3, 4, 9], dtype=torch.int32)
    dst, _ = slim.slim_compact_tokens(dev(k), dev(kept), 64, None, want_pos=False)
    T = so.kept_token_index(kept.numpy(), 64, 640)
    assert torch.equal(dst.cpu(), k[T])


# ------------------------------------------------------------------------------------------ selection
@pytest.mark.parametrize("nb", [2, 3, 7, 32, 128, 512, 1024, 1025, 5000])
def test_select_bit_exact_including_ties(slim, nb):
    print(f"select nb={nb}", flush=True)
    g = np.random.default_rng(nb)
    cases = [g.standard_normal(nb).astype(np.float32),
             np.round(g.standard_normal(nb), 1).astype(np.float32),            # many ties
             np.zeros(nb, np.float32),                                         # all equal
             np.where(g.random(nb) < 0.5, -0.0, 0.0).astype(np.float32),       # signed zeros are equal
             (g.standard_normal(nb) * 10.0 ** g.integers(-30, 30, nb)).astype(np.float32),
             -np.abs(g.standard_normal(nb)).astype(np.float32)]
    for sc in cases:
        for flags in (3, 1, 0, 2):
            nf = bin(flags).count("1")
            for n_keep in sorted({max(nf, 1), nf + 1, max(nf, nb // 3), nb - 1, nb, nb + 5}):
                if n_keep < 1 or (n_keep < nb and n_keep < nf):
                    continue
                kept = slim.slim_select_topk_blocks(dev(torch.from_numpy(sc)), n_keep, flags).cpu().numpy()
                want = so.select_blocks(sc.astype(np.float64), n_keep, bool(flags & 1), bool(flags & 2))
                np.testing.assert_array_equal(kept, want, err_msg=f"nb={nb} n_keep={n_keep} flags={flags}")


# ------------------------------------------------------------------------------------------ scores
@pytest.mark.parametrize("N,block,unit,w,Hq,Hkv,d,dtype", [
    (512, 16, 8, 32, 4, 2, 64, torch.float32),
    (2048, 64, 8, 64, 32, 8, 128, torch.bfloat16),
    (1000, 64, 8, 4, 32, 8, 128, torch.bfloat16),        # ragged last block and unit
    (1536, 128, 8, 128, 32, 8, 128, torch.bfloat16),
    (300, 64, 64, 7, 8, 8, 32, torch.bfloat16),          # unit == block (average pooling)
    (130, 32, 1, 3, 4, 1, 16, torch.float32),            # unit == 1
    (700, 100, 24, 5, 6, 3, 8, torch.float32),           # nothing divides anything
])
def test_scores_match_oracle(slim, N, block, unit, w, Hq, Hkv, d, dtype):
    print(f"score N={N} B={block} u={unit} w={w} H={Hq}/{Hkv} d={d} {dtype}", flush=True)
    q, k = rand((w, Hq, d), dtype, seed=N), rand((N, Hkv, d), dtype, seed=N + 1)
    got = slim.slim_score_blocks(dev(q), dev(k), block, unit)
    want = so.block_scores(f64(q), f64(k), block, unit)
    scale = np.abs(want).max()
    np.testing.assert_allclose(f64(got), want, atol=2e-5 * max(scale, 1.0), rtol=1e-4)


@pytest.mark.parametrize("pooling", ["avg", "max"])
@pytest.mark.parametrize("N,block,w,Hq,Hkv,d,dtype", [
    (4096, 64, 64, 32, 8, 128, torch.bfloat16),
    (1000, 64, 4, 32, 8, 128, torch.bfloat16),           # ragged last block
    (777, 128, 9, 64, 64, 128, torch.bfloat16),          # Hkv*d = 8192: one token slice, chunks in two rounds
    (300, 50, 7, 8, 8, 32, torch.bfloat16),
    (130, 32, 3, 4, 1, 16, torch.float32),
    (700, 100, 5, 6, 3, 8, torch.float32),               # 6 chunks: not a power of two
    (5, 8, 2, 2, 2, 64, torch.float32),                  # one short block, fewer tokens than slices
])
def test_pooled_scores_match_oracle(slim, pooling, N, block, w, Hq, Hkv, d, dtype):
    print(f"pooled score {pooling} N={N} B={block} w={w} H={Hq}/{Hkv} d={d} {dtype}", flush=True)
    q, k = rand((w, Hq, d), dtype, seed=N), rand((N, Hkv, d), dtype, seed=N + 1)
    got = slim.slim_score_blocks_pooled(dev(q), dev(k), block, slim.POOL_AVG if pooling == "avg" else slim.POOL_MAX)
    want = so.block_scores_pooled(f64(q), f64(k), block, pooling)
    scale = np.abs(want).max()
    np.testing.assert_allclose(f64(got), want, atol=2e-5 * max(scale, 1.0), rtol=1e-4)
    if pooling == "avg":                                 # the single-TokenUnit special case of Eq. (1)-(2)
        same = slim.slim_score_blocks(dev(q), dev(k), block, block)
        np.testing.assert_allclose(f64(got), f64(same), atol=2e-5 * max(scale, 1.0), rtol=1e-4)


def test_scores_skewed_stage_input_and_selection(slim):
    wl = inputs.scaled(inputs.WORKLOADS["cfg3"], seq=4096)
    q, k = inputs.stage_qk(wl, skew=True)
    got = slim.slim_score_blocks(dev(q), dev(k), wl.block, wl.unit)
    want = so.block_scores(f64(q), f64(k), wl.block, wl.unit)
    np.testing.assert_allclose(f64(got), want, atol=2e-5 * np.abs(want).max(), rtol=1e-4)
    kept = slim.slim_select_topk_blocks(got, wl.n_keep).cpu().numpy()
    from tests.helpers import assert_selection_matches
    assert_selection_matches(kept, want, wl.n_keep, gap=1e-4)


# ------------------------------------------------------------------------------------------ per-token ops
@pytest.mark.parametrize("n,hidden,dtype", [(300, 4096, torch.bfloat16), (64, 256, torch.float32),
                                            (33, 1000, torch.bfloat16), (5, 10, torch.float32)])
def test_rmsnorm(slim, n, hidden, dtype):
    x, g = rand((n, hidden), dtype, seed=n, scale=3.0), rand((hidden,), dtype, seed=7) + 1.0
    got = slim.slim_rmsnorm(dev(x), dev(g), 1e-5)
    want = so.rmsnorm(f64(x), f64(g), 1e-5)
    tol = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-6
    np.testing.assert_allclose(f64(got), want, rtol=tol, atol=tol * 1e-2)


@pytest.mark.parametrize("n,H,d,dtype", [(257, 8, 128, torch.bfloat16), (100, 4, 64, torch.float32),
                                         (64, 32, 128, torch.bfloat16)])
def test_rope_with_large_positions(slim, n, H, d, dtype):
    g = np.random.default_rng(n)
    x = rand((n, H, d), dtype, seed=n)
    pos = torch.from_numpy(np.sort(g.choice(131072, n, replace=False)).astype(np.int32))
    pos[-1] = 131071
    got = slim.slim_rope(dev(x).clone(), dev(pos), 500000.0)
    c, s = so.rope_cos_sin(pos.numpy(), d, 500000.0, np.float64)
    want = so.apply_rope(f64(x), c, s)
    tol = 2.0 ** -8 if dtype == torch.bfloat16 else 2e-6
    np.testing.assert_allclose(f64(got), want, rtol=tol, atol=tol * 4)
    got0 = slim.slim_rope(dev(x).clone(), None, 500000.0)            # NULL positions = 0..n-1
    c, s = so.rope_cos_sin(np.arange(n), d, 500000.0, np.float64)
    np.testing.assert_allclose(f64(got0), so.apply_rope(f64(x), c, s), rtol=tol, atol=tol * 4)


@pytest.mark.parametrize("m,n,k,dtype", [
    (256, 256, 64, torch.bfloat16), (512, 1024, 4096, torch.bfloat16), (300, 520, 192, torch.bfloat16),
    (64, 4096, 4096, torch.bfloat16), (1, 8, 8, torch.bfloat16), (700, 260, 200, torch.bfloat16),
    (1300, 776, 128, torch.bfloat16), (3000, 512, 64, torch.bfloat16),   # several 256- and 128-token tiles
    (129, 264, 320, torch.bfloat16),     # one row past a 128-token tile, an odd number of k-tiles
    (257, 64, 448, torch.bfloat16),      # one row past a 256-token tile, a quarter of a feature tile
    (1000, 8, 128, torch.bfloat16),      # eight features: every weight row of the tile but eight is a clamped copy
    (130, 70, 50, torch.float32), (512, 688, 256, torch.float32),
])
def test_linear_all_epilogues(slim, m, n, k, dtype):
    print(f"linear m={m} n={n} k={k} {dtype}", flush=True)
    a, w, w2 = rand((m, k), dtype, 1), rand((n, k), dtype, 2, 0.05), rand((n, k), dtype, 3, 0.05)
    r = rand((m, n), dtype, 4)
    A, W, W2, R = f64(a), f64(w), f64(w2), f64(r)
    bf = dtype == torch.bfloat16
    rel = 2.0 ** -8 if bf else 1e-5
    plain = A @ W.T
    atol = rel * np.abs(plain).max()
    np.testing.assert_allclose(f64(slim.slim_linear(dev(a), dev(w))), plain, rtol=rel, atol=atol)
    np.testing.assert_allclose(f64(slim.slim_linear(dev(a), dev(w), residual=dev(r))), plain + R, rtol=rel,
                               atol=rel * np.abs(plain + R).max())
    rd = dev(r).clone()                                   # in place: residual aliases out
    slim.slim_linear(dev(a), dev(w), residual=rd, out=rd)
    np.testing.assert_allclose(f64(rd), plain + R, rtol=rel, atol=rel * np.abs(plain + R).max())
    sw = so.silu(plain) * (A @ W2.T)
    np.testing.assert_allclose(f64(slim.slim_swiglu_linear(dev(a), dev(w), dev(w2))), sw, rtol=rel,
                               atol=rel * np.abs(sw).max())


@pytest.mark.parametrize("m,n,k,lda,ldo", [(300, 520, 192, 256, 640), (1000, 264, 128, 136, 272), (64, 512, 256, 320, 520)])
def test_linear_with_row_strides(slim, m, n, k, lda, ldo):
    """Rows of a and of out / residual that are longer than what the call uses (lda > k_in, ldo > n_out), through the
    C ABI directly: the padding columns of out must stay untouched."""
    import ctypes
    print(f"linear strided m={m} n={n} k={k} lda={lda} ldo={ldo}", flush=True)
    lib = slim.load_library()
    bf = torch.bfloat16
    a_wide, w, w2 = dev(rand((m, lda), bf, 1)), dev(rand((n, k), bf, 2, 0.05)), dev(rand((n, k), bf, 3, 0.05))
    r_wide = dev(rand((m, ldo), bf, 4))
    A, W, W2, R = f64(a_wide)[:, :k], f64(w), f64(w2), f64(r_wide)[:, :n]
    P = lambda t: ctypes.c_void_p(t.data_ptr() if t is not None else 0)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rel = 2.0 ** -8
    for name, call, want in (
            ("plain", lambda o: lib.slim_linear(P(a_wide), lda, P(w), P(None), m, n, k, ldo, 1, P(o), st), A @ W.T),
            ("residual", lambda o: lib.slim_linear(P(a_wide), lda, P(w), P(r_wide), m, n, k, ldo, 1, P(o), st), A @ W.T + R),
            ("swiglu", lambda o: lib.slim_swiglu_linear(P(a_wide), lda, P(w), P(w2), m, n, k, ldo, 1, P(o), st),
             so.silu(A @ W.T) * (A @ W2.T))):
        out = torch.full((m, ldo), 7.0, dtype=bf, device="cuda")
        assert call(out) == 0, name
        torch.cuda.synchronize()
        np.testing.assert_allclose(f64(out)[:, :n], want, rtol=rel, atol=rel * np.abs(want).max(), err_msg=name)
        assert (f64(out)[:, n:] == 7.0).all(), f"{name}: wrote past n_out"


@pytest.mark.parametrize("m,n,k,dtype", [
    (1300, 3584, 256, torch.bfloat16), (64, 512, 3584, torch.bfloat16), (300, 520, 192, torch.bfloat16),
    (700, 260, 200, torch.bfloat16), (130, 70, 50, torch.float32),
])
def test_linear_with_bias(slim, m, n, k, dtype):
    print(f"linear+bias m={m} n={n} k={k} {dtype}", flush=True)
    a, w, b = rand((m, k), dtype, 1), rand((n, k), dtype, 2, 0.05), rand((n,), dtype, 3, 2.0)
    want = f64(a) @ f64(w).T + f64(b)
    rel = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-5
    np.testing.assert_allclose(f64(slim.slim_linear_bias(dev(a), dev(w), dev(b))), want, rtol=rel,
                               atol=rel * np.abs(want).max())


# ------------------------------------------------------------- projections with the RoPE / score epilogue
def test_rope_table_matches_float64_angles(slim):
    g = np.random.default_rng(3)
    pos = np.sort(g.choice(131072, 300, replace=False)).astype(np.int32)
    pos[-1] = 131071
    for theta in (500000.0, 1000000.0):
        t = slim.slim_rope_table(dev(torch.from_numpy(pos)), 300, 128, theta)
        c, s = so.rope_cos_sin(pos, 128, theta, np.float64)
        # angle formed and reduced in double, evaluated in float: 2^-24 * pi on the angle plus the float sincos
        np.testing.assert_allclose(f64(t)[:, :64], c, rtol=0, atol=4e-7)
        np.testing.assert_allclose(f64(t)[:, 64:], s, rtol=0, atol=4e-7)
    t0 = slim.slim_rope_table(None, 50, 128, 500000.0, device="cuda")
    c, s = so.rope_cos_sin(np.arange(50), 128, 500000.0, np.float64)
    np.testing.assert_allclose(f64(t0), np.concatenate([c, s], axis=1), rtol=0, atol=4e-7)


@pytest.mark.parametrize("m,heads,k,with_bias", [
    (64, 32, 4096, False),          # the window projection: one 128-token tile
    (1300, 8, 256, True),           # 256- and 128-token tiles, ragged last tile, bias
    (700, 3, 192, True),            # odd number of heads: the last 256-feature tile is half empty
    (3000, 4, 64, False),
    (1, 1, 64, True),
])
def test_linear_rope_epilogue_and_token_scores(slim, m, heads, k, with_bias):
    print(f"linear+rope m={m} heads={heads} k={k} bias={with_bias}", flush=True)
    bf, d = torch.bfloat16, 128
    g = np.random.default_rng(m + heads)
    a, w = rand((m, k), bf, 1), rand((heads * d, k), bf, 2, 0.05)
    b = rand((heads * d,), bf, 3, 1.0) if with_bias else None
    pos = np.sort(g.choice(40000, m, replace=False)).astype(np.int32)
    table = slim.slim_rope_table(dev(torch.from_numpy(pos)), m, d, 500000.0)
    want = so.project_heads(f64(a), f64(w), heads, d, pos, 500000.0, True, None, None if b is None else f64(b))
    got = slim.slim_linear_rope(dev(a), dev(w), None if b is None else dev(b), table, d)
    rel = 2.0 ** -8
    np.testing.assert_allclose(f64(got), want, rtol=rel, atol=rel * np.abs(want).max())
    # the two-kernel route (projection rounded to bf16, then rotated) agrees to bf16 rounding
    two = slim.slim_linear(dev(a), dev(w)) if b is None else slim.slim_linear_bias(dev(a), dev(w), dev(b))
    two = slim.slim_rope(two.view(m, heads, d), dev(torch.from_numpy(pos)), 500000.0)
    np.testing.assert_allclose(f64(two), want, rtol=2 * rel, atol=2 * rel * np.abs(want).max())
    # with a window query: same keys bit for bit, plus per-(token, head) dots of the stored keys with qt
    qt = torch.from_numpy(g.standard_normal(heads * d).astype(np.float32))
    got2, ts = slim.slim_linear_rope(dev(a), dev(w), None if b is None else dev(b), table, d, qt=dev(qt))
    assert torch.equal(got2, got)
    want_ts = np.einsum("mhd,hd->mh", f64(got), f64(qt).reshape(heads, d))
    np.testing.assert_allclose(f64(ts), want_ts, rtol=0, atol=2e-5 * max(1.0, np.abs(want_ts).max()))


@pytest.mark.parametrize("w,Hq,Hkv,hidden,with_bias,scaled", [
    (64, 32, 8, 4096, False, True),     # the LLaMA-shaped window: 4 splits of the reduction dimension
    (64, 28, 4, 3584, True, True),      # Qwen-shaped: bias, 56 chunks dealt unevenly to the waves
    (7, 4, 4, 128, True, False),        # fewer rows than one MFMA tile, 2 chunks for 4 waves
    (100, 8, 2, 256, False, True),      # two row tiles, the second ragged
    (256, 4, 1, 64, True, False),       # the largest window, a single chunk
    (1, 2, 2, 512, False, True),
])
def test_window_query_from_rows(slim, w, Hq, Hkv, hidden, with_bias, scaled):
    """qt from the window's hidden rows (split projection, rotation and means in float) against the oracle's
    projection + RoPE + window / head means in float64."""
    print(f"window query from rows w={w} Hq={Hq} Hkv={Hkv} hidden={hidden} bias={with_bias} scaled={scaled}", flush=True)
    bf, d, theta = torch.bfloat16, 128, 500000.0
    g = np.random.default_rng(w + Hq)
    big = rand((w + 3, hidden), bf, 11, 2.0)
    rows = big[3:]                                                            # a view into a larger buffer
    wq = rand((Hq * d, hidden), bf, 12, 0.05)
    b = rand((Hq * d,), bf, 13, 1.0) if with_bias else None
    pos = np.sort(g.choice(100000, w, replace=False)).astype(np.int32)
    table = slim.slim_rope_table(dev(torch.from_numpy(pos)), w, d, theta)
    x = f64(rows)
    rstd = 1.0 / np.sqrt((x * x).mean(axis=1) + 1e-5) if scaled else None
    xn = x * rstd[:, None] if scaled else x
    q = so.project_heads(xn, f64(wq), Hq, d, pos, theta, True, None, None if b is None else f64(b))
    want = so.window_query(q).reshape(Hkv, Hq // Hkv, d).sum(axis=1).reshape(-1) / Hq
    rows_gpu = dev(big)[3:]
    got = slim.slim_window_query_from_rows(rows_gpu, dev(wq), None if b is None else dev(b), table, Hq, Hkv,
                                           rstd=None if rstd is None else dev(torch.from_numpy(rstd.astype(np.float32))))
    # float accumulation over hidden * w * G products and the 4e-7 table: far inside a bf16 rounding of the states
    np.testing.assert_allclose(f64(got), want, rtol=0, atol=2e-5 * max(1.0, np.abs(q).max()))
    # the route through stored bf16 Query states agrees to the rounding of those states
    if not scaled:
        q_win = slim.slim_linear_rope(rows_gpu.contiguous(), dev(wq), None if b is None else dev(b), table, d)
        via = slim.slim_window_query(q_win, Hkv)
        assert (via - got).abs().max().item() < 2.0 ** -8 * max(1.0, np.abs(q).max())
    again = slim.slim_window_query_from_rows(rows_gpu, dev(wq), None if b is None else dev(b), table, Hq, Hkv,
                                             rstd=None if rstd is None else dev(torch.from_numpy(rstd.astype(np.float32))))
    assert torch.equal(got, again)


@pytest.mark.parametrize("N,block,unit,w,Hq,Hkv,hidden", [
    (1024, 64, 8, 64, 32, 8, 512), (1000, 64, 8, 4, 8, 2, 256), (1003, 64, 8, 16, 28, 4, 256), (333, 32, 5, 7, 4, 4, 128),
])
def test_key_first_pipeline_scores_match_oracle(slim, N, block, unit, w, Hq, Hkv, hidden):
    """Window query -> K projection with RoPE and score partials -> block scores, against Eq. 1-2 of the oracle
    on the oracle's own projections, and against slim_score_blocks on the same stored keys."""
    print(f"key-first scores N={N} block={block} unit={unit} w={w} Hq={Hq} Hkv={Hkv}", flush=True)
    bf, d, theta = torch.bfloat16, 128, 500000.0
    h = rand((N, hidden), bf, 5)
    wq, wk = rand((Hq * d, hidden), bf, 6, 0.05), rand((Hkv * d, hidden), bf, 7, 0.05)
    pos = np.arange(N, dtype=np.int32) * 3
    table = slim.slim_rope_table(dev(torch.from_numpy(pos)), N, d, theta)
    q_win = slim.slim_linear_rope(dev(h[N - w:]), dev(wq), None, table[N - w:], d)
    qt = slim.slim_window_query(q_win, Hkv)
    k, ts = slim.slim_linear_rope(dev(h), dev(wk), None, table, d, qt=qt)
    scores = slim.slim_score_blocks_from_token_scores(ts, block, unit)
    # qt against its definition on the GPU's window states
    ql = so.window_query(f64(q_win))                                         # [Hq, d]
    want_qt = ql.reshape(Hkv, Hq // Hkv, d).sum(axis=1).reshape(-1) / Hq
    np.testing.assert_allclose(f64(qt), want_qt, rtol=0, atol=1e-6 * max(1.0, np.abs(want_qt).max()))
    # scores: Eq. 1-2 on the stored (rounded) states
    want = so.block_scores(f64(q_win), f64(k), block, unit)
    scale = max(1.0, float(np.abs(want).max()))
    assert np.abs(f64(scores) - want).max() < 2e-5 * scale
    direct = slim.slim_score_blocks(q_win, k, block, unit)
    assert (scores - direct).abs().max().item() < 2e-5 * scale
    # and against the exact pipeline (float64 projections): bf16 rounding of the states only
    qe = so.project_heads(f64(h[N - w:]), f64(wq), Hq, d, pos[N - w:], theta, True)
    ke = so.project_heads(f64(h), f64(wk), Hkv, d, pos, theta, True)
    exact = so.block_scores(qe, ke, block, unit)
    qr = so.project_heads(f64(h[N - w:]), f64(wq), Hq, d, pos[N - w:], theta, True, "bf16")
    kr = so.project_heads(f64(h), f64(wk), Hkv, d, pos, theta, True, "bf16")
    floor = np.abs(so.block_scores(qr, kr, block, unit) - exact).max()      # what rounding the states to bf16 costs
    assert np.abs(f64(scores) - exact).max() < max(2e-3, 3.0 * floor) * max(1.0, float(np.abs(exact).max()))


@pytest.mark.parametrize("m,n,k", [(64, 512, 256), (1300, 776, 128), (300, 4096, 4096), (1, 8, 64)])
def test_rmsnorm_fused_into_projections(slim, m, n, k):
    """out = RMSNorm(a) . w^T from raw rows and their 1/rms applied to the accumulators, against the oracle's RMSNorm
    then projection; with a gain, the weights are folded first."""
    print(f"rmsnorm+linear m={m} n={n} k={k}", flush=True)
    bf, eps = torch.bfloat16, 1e-5
    a, w, w2 = rand((m, k), bf, 1, 3.0), rand((n, k), bf, 2, 0.05), rand((n, k), bf, 3, 0.05)
    b = rand((n,), bf, 4, 1.0)
    gain = (1.0 + 0.2 * rand((k,), torch.float32, 5)).to(bf)
    ones = np.ones(k)
    rel = 2.0 ** -8
    hn = so.rmsnorm(f64(a), ones, eps)
    rstd = slim.slim_row_rstd(dev(a), eps)
    np.testing.assert_allclose(f64(rstd), 1.0 / np.sqrt((f64(a) ** 2).mean(axis=1) + eps), rtol=2e-6)
    want = hn @ f64(w).T
    np.testing.assert_allclose(f64(slim.slim_rmsnorm_linear(dev(a), dev(w), rstd)), want, rtol=rel, atol=rel * np.abs(want).max())
    np.testing.assert_allclose(f64(slim.slim_rmsnorm_linear(dev(a), dev(w), rstd, bias=dev(b))), want + f64(b), rtol=rel,
                               atol=rel * np.abs(want + f64(b)).max())
    sw = so.silu(want) * (hn @ f64(w2).T)
    np.testing.assert_allclose(f64(slim.slim_rmsnorm_swiglu_linear(dev(a), dev(w), dev(w2), rstd)), sw, rtol=rel,
                               atol=rel * np.abs(sw).max())
    # gain folded into the weights: exact fold in bf16 rounding, then the same projection
    wf = slim.slim_fold_gain(dev(w), dev(gain))
    np.testing.assert_allclose(f64(wf), f64(w) * f64(gain)[None, :], rtol=2.0 ** -8, atol=0)
    want_g = so.rmsnorm(f64(a), f64(gain), eps) @ f64(w).T
    np.testing.assert_allclose(f64(slim.slim_rmsnorm_linear(dev(a), wf, rstd)), want_g, rtol=2 * rel,
                               atol=2 * rel * np.abs(want_g).max())
    # the fold also works in float and in place
    w32 = f64(w).astype(np.float32)
    got32 = slim.slim_fold_gain(dev(torch.from_numpy(w32)), dev(gain.to(torch.float32)))
    np.testing.assert_allclose(got32.cpu().numpy(), w32 * gain.to(torch.float32).numpy()[None, :], rtol=1e-6)


@pytest.mark.parametrize("m,n1,n2,k,bias,scaled", [
    (1300, 4096, 1024, 128, False, True), (700, 3584, 512, 192, True, True), (300, 260, 72, 64, False, False),
    (2000, 256, 256, 64, True, False),
])
def test_two_projections_in_one_launch_are_bit_identical_to_two_launches(slim, m, n1, n2, k, bias, scaled):
    print(f"linear pair m={m} n1={n1} n2={n2} k={k} bias={bias} scaled={scaled}", flush=True)
    bf = torch.bfloat16
    a, w1, w2 = dev(rand((m, k), bf, 1, 2.0)), dev(rand((n1, k), bf, 2, 0.05)), dev(rand((n2, k), bf, 3, 0.05))
    b1, b2 = (dev(rand((n1,), bf, 4)), dev(rand((n2,), bf, 5))) if bias else (None, None)
    rstd = slim.slim_row_rstd(a, 1e-5) if scaled else None
    o1, o2 = slim.slim_linear_pair(a, w1, w2, b1, b2, rstd)
    if scaled:
        r1, r2 = slim.slim_rmsnorm_linear(a, w1, rstd, bias=b1), slim.slim_rmsnorm_linear(a, w2, rstd, bias=b2)
    elif bias:
        r1, r2 = slim.slim_linear_bias(a, w1, b1), slim.slim_linear_bias(a, w2, b2)
    else:
        r1, r2 = slim.slim_linear(a, w1), slim.slim_linear(a, w2)
    assert torch.equal(o1, r1) and torch.equal(o2, r2)
    want = (so.rmsnorm(f64(a), np.ones(k), 1e-5) if scaled else f64(a)) @ f64(w2).T + (f64(b2) if bias else 0.0)
    np.testing.assert_allclose(f64(o2), want, rtol=2.0 ** -8, atol=2.0 ** -8 * np.abs(want).max())


def test_rmsnorm_and_rope_in_one_projection(slim):
    m, heads, k, d, theta, eps = 700, 4, 256, 128, 500000.0, 1e-5
    bf = torch.bfloat16
    a, w, b = rand((m, k), bf, 1, 5.0), rand((heads * d, k), bf, 2, 0.05), rand((heads * d,), bf, 3, 1.0)
    pos = (np.arange(m, dtype=np.int32) * 7) % 5000
    table = slim.slim_rope_table(dev(torch.from_numpy(pos)), m, d, theta)
    hn = so.rmsnorm(f64(a), np.ones(k), eps)
    want = so.project_heads(hn, f64(w), heads, d, pos, theta, True, None, f64(b))
    got = slim.slim_linear_rope(dev(a), dev(w), dev(b), table, d, rstd=slim.slim_row_rstd(dev(a), eps))
    np.testing.assert_allclose(f64(got), want, rtol=2.0 ** -8, atol=2.0 ** -8 * np.abs(want).max())


# ------------------------------------------------------------------------------------------ attention
@pytest.mark.parametrize("n,Hq,Hkv,d,dtype", [
    (1, 4, 1, 128, torch.bfloat16), (37, 4, 2, 128, torch.bfloat16), (128, 8, 8, 128, torch.bfloat16),
    (200, 4, 1, 128, torch.bfloat16), (1000, 8, 2, 128, torch.bfloat16), (1280, 32, 8, 128, torch.bfloat16),
    (256, 4, 2, 64, torch.float32), (77, 6, 3, 32, torch.float32), (130, 2, 1, 128, torch.float32),
])
def test_attention_matches_oracle(slim, n, Hq, Hkv, d, dtype):
    print(f"attn n={n} H={Hq}/{Hkv} d={d} {dtype}", flush=True)
    name = "bf16" if dtype == torch.bfloat16 else "fp32"
    q, k, v = inputs.stage_qkv(n, Hq, Hkv, d, name, seed=n)
    got = slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    want = so.causal_gqa_attention(f64(q), f64(k), f64(v))
    mx, mean = errs(got, want)
    print(f"   max-abs {mx:.3e} mean-abs {mean:.3e}", flush=True)
    if dtype == torch.bfloat16:
        assert mx <= MAX_ABS and mean <= MEAN_ABS
    else:
        assert mx <= 2e-5
    # explicit scale
    got2 = slim.slim_prefill_attn(dev(q), dev(k), dev(v), softmax_scale=0.05)
    mx2, _ = errs(got2, so.causal_gqa_attention(f64(q), f64(k), f64(v), scale=0.05))
    assert mx2 <= (MAX_ABS if dtype == torch.bfloat16 else 2e-5)


@pytest.mark.parametrize("n,q_scale", [(9856, 1.0), (26240, 1.0), (16384, 1.0), (9856, 2.5)])
def test_attention_full_size_sampled_rows(slim, n, q_scale):
    """slim_prefill_attn alone at the kept-token counts of the 32K, 131K and 32-layer workloads (32 query / 8 kv heads
    of 128), in the launch configuration the layer uses, on sampled rows that the oracle evaluates one by one: the
    first and last rows, rows on both sides of every boundary the kernel has (32-key unit, 64-query wave, 128-key
    tile, 256), rows of the last, short tile, and random ones.  q_scale 2.5: logits of +-15 and more, so that the
    softmax is carried by a few keys and the reference of the online softmax moves."""
    Hq, Hkv, d = 32, 8, 128
    print(f"attn full size n={n} H={Hq}/{Hkv} d={d} q x {q_scale}", flush=True)
    q, k, v = inputs.stage_qkv(n, Hq, Hkv, d, "bf16", seed=n % 1000 + int(10 * q_scale))
    if q_scale != 1.0:
        q = (q.float() * q_scale).to(torch.bfloat16)
    g = np.random.default_rng(n)
    edges = [0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, n // 2 - 1, n // 2, (n // 128) * 128 - 1,
             (n // 128) * 128, (n // 256) * 256 - 1, (n // 256) * 256, n - 65, n - 64, n - 33, n - 32, n - 2, n - 1]
    rows = np.array(sorted(set(r for r in edges if 0 <= r < n) | set(g.integers(0, n, 44).tolist())))
    assert len(rows) >= 64
    got = slim.slim_prefill_attn(dev(q), dev(k), dev(v))[torch.from_numpy(rows).cuda()]
    want = so.causal_gqa_attention(f64(q)[rows], f64(k), f64(v), rows=rows)
    mx, mean = errs(got, want)
    print(f"   {len(rows)} rows: max-abs {mx:.3e} mean-abs {mean:.3e}", flush=True)
    assert np.isfinite(f64(got)).all() and mx <= MAX_ABS and mean <= MEAN_ABS


def test_attention_peaked_logits_and_first_row(slim):
    n, Hq, Hkv, d = 300, 4, 2, 128
    q, k, v = inputs.stage_qkv(n, Hq, Hkv, d, "bf16", seed=9)
    q = q * 4.0                                             # logits up to ~ +-40: softmax nearly one-hot
    got = slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    want = so.causal_gqa_attention(f64(q), f64(k), f64(v))
    mx, mean = errs(got, want)
    assert np.isfinite(f64(got)).all() and mx <= 4e-2 and mean <= MEAN_ABS * 2
    np.testing.assert_array_equal(f64(got)[0], np.repeat(f64(v)[0], Hq // Hkv, 0))   # row 0 sees only key 0


@pytest.mark.parametrize("stair", [12.0, 160.0])
def test_attention_reference_moves_at_every_place(slim, stair):
    """Logits that climb a staircase along the keys (48 stairs at random keys, each about 12 binary orders high, or
    about 160: then exp2 of a logit taken against the old reference overflows): for every query the reference of the
    online softmax has to move at each stair below it, at whatever place in the key tile, unit and part of a unit the
    stair falls, in the full-tile loop and in the masked loop of the diagonal."""
    n, Hq, Hkv, d = 1500, 8, 2, 128
    print(f"attn staircase n={n} H={Hq}/{Hkv} d={d} stair {stair}", flush=True)
    q, k, v = inputs.stage_qkv(n, Hq, Hkv, d, "bf16", seed=77)
    g = np.random.default_rng(5)
    stairs = np.sort(g.choice(np.arange(1, n), 48, replace=False))
    level = torch.from_numpy(np.searchsorted(stairs, np.arange(n), side="right").astype(np.float32))
    q = (q.float() * 0.25)
    k = (k.float() * 0.25)
    q[:, :, 0] = 8.0
    k[:, :, 0] = stair * level[:, None]                  # exact in bf16 up to 48 stairs
    q, k = q.to(torch.bfloat16), k.to(torch.bfloat16)
    got = slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    want = so.causal_gqa_attention(f64(q), f64(k), f64(v))
    mx, mean = errs(got, want)
    print(f"   max-abs {mx:.3e} mean-abs {mean:.3e}", flush=True)
    assert np.isfinite(f64(got)).all() and mx <= 4e-2 and mean <= MEAN_ABS * 2


def test_kernels_are_deterministic(slim):
    q, k, v = inputs.stage_qkv(700, 8, 2, 128, "bf16", seed=3)
    a = slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    b = slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    assert torch.equal(a, b)
    x, w = rand((300, 512), torch.bfloat16, 1), rand((384, 512), torch.bfloat16, 2)
    assert torch.equal(slim.slim_linear(dev(x), dev(w)), slim.slim_linear(dev(x), dev(w)))


def test_error_paths_on_device_tensors(slim):
    q, k, v = inputs.stage_qkv(16, 4, 2, 96, "bf16", seed=1)
    with pytest.raises(slim.SlimError) as e:
        slim.slim_prefill_attn(dev(q), dev(k), dev(v))
    assert e.value.code == -2
    sc = torch.zeros(8, device="cuda")
    with pytest.raises(slim.SlimError) as e:
        slim.slim_select_topk_blocks(sc, 1, 3)
    assert e.value.code == -1
    with pytest.raises(ValueError):
        slim.slim_rmsnorm(torch.zeros(4, 8), torch.ones(8), 1e-5)          # host tensor is refused
