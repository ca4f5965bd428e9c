"""The C-ABI library loads and exports every symbol that include/slim.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2508_06447_amd as slim
    if not os.path.exists(slim.LIB_PATH):
        from paper_2508_06447_amd.build import build_lib
        build_lib(verbose=False)
    return slim.load_library()


def declared_symbols(header="slim.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slim_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    import paper_2508_06447_amd as slim
    names = declared_symbols()
    assert len(names) >= 14 and set(names) == set(slim.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_the_probes_live_in_a_library_and_header_of_their_own(lib):
    """The method's ABI (slim.h, libslim.so) holds no measurement helper; bench.py's probes are declared in
    slim_probe.h and exported by libslim_probe.so only."""
    import paper_2508_06447_amd as slim
    assert not [n for n in declared_symbols() if "probe" in n]
    names = declared_symbols("slim_probe.h")
    assert set(names) == set(slim.PROBE_EXPORTS) and len(names) == 3
    plib = slim.load_probe_library()
    for n in names:
        assert getattr(plib, n) is not None
        assert not hasattr(lib, n)
    assert plib.slim_probe_mfma_flops(2, 3) == 2 * 8 * 3 * 8 * 2.0 * 32 * 32 * 16
    assert plib.slim_probe_copy(None, None, 16, None) == -1


def test_status_strings_and_host_only_helpers(lib):
    assert lib.slim_status_string(0) == b"ok"
    assert b"invalid" in lib.slim_status_string(-1)
    assert b"unsupported" in lib.slim_status_string(-2)
    assert b"workspace" in lib.slim_status_string(-3)
    assert lib.slim_last_hip_error() == b""
    # n' = (n_keep-1)*block + length of the last block
    assert lib.slim_kept_tokens(512, 16, 16) == 256
    assert lib.slim_kept_tokens(32768, 64, 154) == 9856
    assert lib.slim_kept_tokens(131072, 128, 205) == 26240
    assert lib.slim_kept_tokens(45, 8, 3) == 21 and lib.slim_kept_tokens(45, 8, 6) == 45
    assert lib.slim_score_blocks_workspace_bytes(8, 128) == 4096


def test_argument_errors_are_reported_before_anything_is_enqueued(lib):
    import paper_2508_06447_amd as slim
    null = ctypes.c_void_p(0)
    assert lib.slim_score_blocks(null, null, 8, 2, 2, 1, 8, 4, 2, 1, null, null, 0, null) == -1
    assert lib.slim_select_topk_blocks(null, 4, 2, 3, null, null) == -1
    assert lib.slim_compact_tokens(null, null, null, 1, 4, 8, 8, 1, null, null, null) == -1
    assert lib.slim_prefill_attn(null, null, null, 4, 2, 1, 128, 0.0, 1, null, null) == -1
    one = ctypes.c_void_p(256)            # non-null, never dereferenced on these paths
    assert lib.slim_prefill_attn(one, one, one, 4, 3, 2, 128, 0.0, 1, one, null) == -1      # Hq % Hkv
    assert lib.slim_prefill_attn(one, one, one, 4, 2, 1, 96, 0.0, 1, one, null) == -2       # head_dim
    assert lib.slim_prefill_attn(one, one, one, 4, 2, 1, 128, 0.0, 7, one, null) == -2      # dtype
    assert lib.slim_select_topk_blocks(one, 8, 1, 3, one, null) == -1                       # fewer than forced
    assert lib.slim_score_blocks(one, one, 8, 2, 2, 1, 8, 4, 8, 1, one, one, 4096, null) == -1   # unit > block
    assert lib.slim_score_blocks(one, one, 8, 2, 2, 1, 8, 4, 2, 1, one, one, 0, null) == -3      # workspace
    assert lib.slim_linear(one, 8, one, null, 4, 4, 12, 4, 1, one, null) == -1                    # lda < k
    assert lib.slim_linear(one, 12, one, null, 4, 4, 12, 4, 1, one, null) == -2                   # k % 8
    assert lib.slim_unit_keys(one, 100, 8, 128, 64, 128, 1, one, null) == -1                      # unit > block
    assert lib.slim_unit_keys(one, 100, 8, 128, 64, 8, 1, ctypes.c_void_p(260), null) == -2       # k_rep alignment
    assert lib.slim_score_blocks_from_unit_keys(one, one, 100, 4, 32, 8, 128, 64, 8, 1, one, one, 0, null) == -3
    assert lib.slim_kv_swap_workspace_bytes(512, 128) == 4352 and lib.slim_kv_swap_workspace_bytes(0, 4) == 0
    swap = lambda n_cand, gamma, block_bytes, ws: lib.slim_kv_swap(one, n_cand, 512, gamma, one, one, one, 128, one,
                                                                  one, block_bytes, one, one, ws, null)
    assert swap(0, 0.9, 4096, 4096) == -1 and swap(4, 1.5, 4096, 4096) == -1 and swap(4, float("nan"), 4096, 4096) == -1
    assert swap(4, 0.9, 4100, 4096) == -2 and swap(4, 0.9, 4096, 1024) == -3
    # key-first pipeline, fused norms, paired projections: checks that need no GPU
    fl = ctypes.c_float
    assert lib.slim_rope_table(null, 8, 128, fl(5e5), null, null) == -1                            # no output
    assert lib.slim_rope_table(null, 8, 127, fl(5e5), one, null) == -1                             # odd head_dim
    assert lib.slim_window_query(one, 4, 6, 4, 128, 1, one, null) == -1                            # Hq % Hkv
    assert lib.slim_window_query_from_rows_workspace_bytes(64, 32) == 4 * 64 * 32 * 128 * 4
    assert lib.slim_window_query_from_rows_workspace_bytes(0, 32) == 0
    wqr = lambda window, k_in, Hq, ws: lib.slim_window_query_from_rows(one, k_in, one, null, null, one, window, Hq, 4, k_in,
                                                                       one, one, ws, null)
    assert wqr(64, 4096, 6, 1 << 30) == -1 and wqr(257, 4096, 8, 1 << 30) == -2 and wqr(64, 4000, 8, 1 << 30) == -2
    assert wqr(64, 4096, 8, 4096) == -3
    rope = lambda head_dim, k_in, dtype: lib.slim_linear_rope(one, k_in, one, null, one, 64, 8, head_dim, k_in, 8 * head_dim,
                                                              dtype, null, one, null, null, null)
    assert rope(64, 4096, 1) == -2 and rope(128, 4000, 1) == -2 and rope(128, 4096, 0) == -2       # head_dim, k % 64, fp32
    assert lib.slim_linear_rope(one, 4096, one, null, one, 64, 8, 128, 4096, 1024, 1, null, one, one, null, null) == -1  # qt without token_scores
    assert lib.slim_score_blocks_from_token_scores(one, 100, 8, 64, 65, one, null) == -1            # unit > block
    assert lib.slim_row_rstd(null, 4, 64, fl(1e-5), 1, one, null) == -1
    assert lib.slim_rmsnorm_linear(one, 4096, one, null, null, 64, 64, 4096, 64, 1, one, null) == -1     # no rstd
    assert lib.slim_rmsnorm_linear(one, 4096, one, null, one, 64, 64, 4096, 64, 0, one, null) == -2      # fp32
    assert lib.slim_rmsnorm_swiglu_linear(one, 4096, one, null, one, 64, 64, 4096, 64, 1, one, null) == -1   # no w_up
    assert lib.slim_fold_gain(one, null, 8, 8, 1, one, null) == -1
    assert lib.slim_gemv(one, null, one, null, null, null, 64, 4100, 1, one, null) == -2            # k % 8
    assert lib.slim_gemv(one, null, one, null, null, null, 64, 32768, 1, one, null) == -2           # token does not fit LDS
    assert lib.slim_gemv(null, null, one, null, null, null, 64, 4096, 1, one, null) == -1
    assert lib.slim_decode_attn_workspace_bytes(128, 16, 32) == (128 + 1) * 32 * 130 * 4 and lib.slim_decode_attn_workspace_bytes(0, 0, 32) == 0
    assert lib.slim_decode_attn(one, one, 262144, 0, one, 128, 64, 32768, null, null, 0, 32, 8, 96, fl(0), 1, one, one, 1 << 30, null) == -2   # head_dim
    assert lib.slim_decode_attn(one, one, 1024, 0, one, 128, 64, 32768, null, null, 0, 32, 8, 128, fl(0), 1, one, one, 1 << 30, null) == -1   # slot too small
    assert lib.slim_decode_attn(one, one, 262144, 0, one, 128, 64, 32768, null, null, 0, 32, 8, 128, fl(0), 1, one, one, 16, null) == -3
    pair = lambda m, b1, b2: lib.slim_linear_pair(one, 4096, one, b1, 4096, 4096, one, one, b2, 1024, 1024, one, null, m,
                                                  4096, 1, null)
    assert pair(512, one, null) == -1 and pair(64, null, null) == -2                               # one bias only; m <= 128
    shape = slim.make_shape(4096, 32, 8, 128, 14336, 64, 8, 64, __import__("torch").bfloat16)
    need = slim.pruned_layer_workspace_bytes(shape, 32768, 154)
    assert need > 32768 * 4096 * 2
    w = slim.LayerWeights(*([256] * 9))
    args = (ctypes.byref(shape), ctypes.byref(w), one, null, 32768, 154, one, one, one, null, one)
    assert lib.slim_pruned_layer(*args, need - 1, null) == -3
    assert lib.slim_pruned_layer(ctypes.byref(shape), ctypes.byref(w), one, null, 32768, 1, one, one, one, null,
                                 one, need, null) == -1
    bad = slim.make_shape(4096, 32, 8, 96, 14336, 64, 8, 64, __import__("torch").bfloat16)
    assert slim.pruned_layer_workspace_bytes(bad, 1024, 4) == 0
