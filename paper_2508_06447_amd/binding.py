"""ctypes binding of libslim.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their data pointers, sizes
and the current HIP stream to the C entry point of the same name, and raises on a non-zero status.
No arithmetic of the method happens here, and there is no fallback: if the library or a GPU is
missing, the call fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslim.so")
PROBE_LIB_PATH = os.path.join(_HERE, "libslim_probe.so")

F32, BF16 = 0, 1
POOL_AVG, POOL_MAX = 1, 2
PRUNE_BEFORE_ATTENTION, PRUNE_AFTER_ATTENTION = 0, 1
FORCE_FIRST, FORCE_LAST = 1, 2

EXPORTS = (
    "slim_status_string", "slim_last_hip_error", "slim_score_blocks_workspace_bytes", "slim_score_blocks",
    "slim_score_blocks_static",
    "slim_score_blocks_pooled", "slim_unit_keys", "slim_score_blocks_from_unit_keys",
    "slim_kv_swap_workspace_bytes", "slim_kv_swap", "slim_decode_attn_workspace_bytes", "slim_decode_attn", "slim_gemv", "slim_decode_layer_workspace_bytes",
    "slim_decode_layer",
    "slim_rope_table", "slim_window_query", "slim_window_query_from_rows_workspace_bytes", "slim_window_query_from_rows",
    "slim_linear_rope", "slim_score_blocks_from_token_scores",
    "slim_linear_pair", "slim_row_rstd", "slim_rmsnorm_linear", "slim_rmsnorm_swiglu_linear", "slim_fold_gain",
    "slim_select_topk_blocks", "slim_compact_tokens", "slim_prefill_attn", "slim_rmsnorm", "slim_rope",
    "slim_linear", "slim_linear_bias", "slim_swiglu_linear", "slim_kept_tokens", "slim_pruned_layer_workspace_bytes",
    "slim_pruned_layer", "slim_prefill_model_tokens", "slim_prefill_model_workspace_bytes", "slim_prefill_model",
)
PROBE_EXPORTS = ("slim_probe_mfma_flops", "slim_probe_mfma", "slim_probe_copy")   # libslim_probe.so, include/slim_probe.h


class SlimError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: status {code} ({detail})")


class LayerShape(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("ffn", C.c_int), ("block", C.c_int), ("unit", C.c_int), ("window", C.c_int),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int), ("flags", C.c_uint),
                ("scoring", C.c_int), ("placement", C.c_int)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w_gate", "w_up", "w_down",
                                          "bq", "bk", "bv")]


_lib = None


def load_library(path: str | None = None) -> C.CDLL:
    """Load libslim.so (built by `python -m paper_2508_06447_amd.build`).  Fails loudly if absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} not found: build it with __graft_entry__.build() or "
                                "`python paper_2508_06447_amd/build.py`")
    lib = C.CDLL(p)
    vp, i, f, sz, u = C.c_void_p, C.c_int, C.c_float, C.c_size_t, C.c_uint
    lib.slim_status_string.restype = C.c_char_p
    lib.slim_status_string.argtypes = [i]
    lib.slim_last_hip_error.restype = C.c_char_p
    lib.slim_last_hip_error.argtypes = []
    lib.slim_score_blocks_workspace_bytes.restype = sz
    lib.slim_score_blocks_workspace_bytes.argtypes = [i, i]
    lib.slim_score_blocks.argtypes = [vp, vp, i, i, i, i, i, i, i, i, vp, vp, sz, vp]
    lib.slim_score_blocks_static.argtypes = [vp, vp, i, i, i, i, i, i, i, i, vp, vp]
    lib.slim_score_blocks_pooled.argtypes = [vp, vp, i, i, i, i, i, i, i, i, vp, vp, sz, vp]
    lib.slim_unit_keys.argtypes = [vp, i, i, i, i, i, i, vp, vp]
    lib.slim_score_blocks_from_unit_keys.argtypes = [vp, vp, i, i, i, i, i, i, i, i, vp, vp, sz, vp]
    lib.slim_kv_swap_workspace_bytes.restype = sz
    lib.slim_kv_swap_workspace_bytes.argtypes = [i, i]
    lib.slim_kv_swap.argtypes = [vp, i, i, C.c_double, vp, vp, vp, i, vp, vp, sz, vp, vp, sz, vp]
    lib.slim_decode_attn_workspace_bytes.restype = sz
    lib.slim_decode_attn_workspace_bytes.argtypes = [i, i, i]
    lib.slim_decode_attn.argtypes = [vp, vp, sz, sz, vp, i, i, i, vp, vp, i, i, i, i, f, i, vp, vp, sz, vp]
    lib.slim_gemv.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp, vp]
    lib.slim_decode_layer_workspace_bytes.restype = sz
    lib.slim_decode_layer_workspace_bytes.argtypes = [C.POINTER(LayerShape), i, i]
    lib.slim_decode_layer.argtypes = [C.POINTER(LayerShape), C.POINTER(LayerWeights), vp, i, vp, sz, sz, vp, i, i, vp, vp, i, vp, vp,
                                      vp, sz, vp]
    lib.slim_rope_table.argtypes = [vp, i, i, f, vp, vp]
    lib.slim_window_query.argtypes = [vp, i, i, i, i, i, vp, vp]
    lib.slim_window_query_from_rows_workspace_bytes.restype = sz
    lib.slim_window_query_from_rows_workspace_bytes.argtypes = [i, i]
    lib.slim_window_query_from_rows.argtypes = [vp, i, vp, vp, vp, vp, i, i, i, i, vp, vp, sz, vp]
    lib.slim_linear_rope.argtypes = [vp, i, vp, vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, vp]
    lib.slim_row_rstd.argtypes = [vp, i, i, f, i, vp, vp]
    lib.slim_linear_pair.argtypes = [vp, i, vp, vp, i, i, vp, vp, vp, i, i, vp, vp, i, i, i, vp]
    lib.slim_rmsnorm_linear.argtypes = [vp, i, vp, vp, vp, i, i, i, i, i, vp, vp]
    lib.slim_rmsnorm_swiglu_linear.argtypes = [vp, i, vp, vp, vp, i, i, i, i, i, vp, vp]
    lib.slim_fold_gain.argtypes = [vp, vp, i, i, i, vp, vp]
    lib.slim_score_blocks_from_token_scores.argtypes = [vp, i, i, i, i, vp, vp]
    lib.slim_select_topk_blocks.argtypes = [vp, i, i, u, vp, vp]
    lib.slim_compact_tokens.argtypes = [vp, vp, vp, i, i, i, i, i, vp, vp, vp]
    lib.slim_prefill_attn.argtypes = [vp, vp, vp, i, i, i, i, f, i, vp, vp]
    lib.slim_rmsnorm.argtypes = [vp, vp, i, i, f, i, vp, vp]
    lib.slim_rope.argtypes = [vp, vp, i, i, i, f, i, vp]
    lib.slim_linear.argtypes = [vp, i, vp, vp, i, i, i, i, i, vp, vp]
    lib.slim_linear_bias.argtypes = [vp, i, vp, vp, i, i, i, i, i, vp, vp]
    lib.slim_swiglu_linear.argtypes = [vp, i, vp, vp, i, i, i, i, i, vp, vp]
    lib.slim_kept_tokens.argtypes = [i, i, i]
    lib.slim_pruned_layer_workspace_bytes.restype = sz
    lib.slim_pruned_layer_workspace_bytes.argtypes = [C.POINTER(LayerShape), i, i]
    lib.slim_pruned_layer.argtypes = [C.POINTER(LayerShape), C.POINTER(LayerWeights), vp, vp, i, i, vp, vp, vp, vp,
                                      vp, sz, vp]
    ip = C.POINTER(C.c_int)
    lib.slim_prefill_model_tokens.argtypes = [C.POINTER(LayerShape), i, ip, i]
    lib.slim_prefill_model_workspace_bytes.restype = sz
    lib.slim_prefill_model_workspace_bytes.argtypes = [C.POINTER(LayerShape), i, ip, i]
    lib.slim_prefill_model.argtypes = [C.POINTER(LayerShape), C.POINTER(LayerWeights), i, ip, vp, vp, i, vp, vp, vp,
                                       vp, sz, vp]
    for name in EXPORTS:
        getattr(lib, name)                      # every declared symbol must resolve
    if path is None:
        _lib = lib
    return lib


def _check(code: int, where: str):
    if code != 0:
        lib = load_library()
        detail = lib.slim_status_string(code).decode()
        if code == -4:
            detail += ": " + lib.slim_last_hip_error().decode()
        raise SlimError(code, where, detail)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: torch.Tensor | None, name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def n_blocks(n_tokens: int, block: int) -> int:
    return (n_tokens + block - 1) // block


def kept_tokens(n_tokens: int, block: int, n_keep: int) -> int:
    return load_library().slim_kept_tokens(n_tokens, block, n_keep)


def slim_score_blocks(q_win: torch.Tensor, k: torch.Tensor, block: int, unit: int,
                      scores: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """q_win[w,Hq,d], k[N,Hkv,d] -> scores[nb] float32 (Eq. 1-2)."""
    lib = load_library()
    w, Hq, d = q_win.shape
    N, Hkv, _ = k.shape
    if scores is None:
        scores = torch.empty(n_blocks(N, block), dtype=torch.float32, device=k.device)
    need = lib.slim_score_blocks_workspace_bytes(Hkv, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=k.device)
    _check(lib.slim_score_blocks(_dev(q_win, "q_win"), _dev(k, "k"), N, w, Hq, Hkv, d, block, unit, _dtype_code(k),
                                 _dev(scores, "scores"), _dev(workspace, "workspace"), workspace.numel(), _stream()),
           "slim_score_blocks")
    return scores


def slim_score_blocks_static(q_win: torch.Tensor, k: torch.Tensor, block: int, unit: int,
                             scores: torch.Tensor) -> torch.Tensor:
    """slim_score_blocks without a workspace: the library's own per-GPU scratch array carries the window query.
    The caller passes every buffer, `scores` included, so the call allocates nothing."""
    lib = load_library()
    w, Hq, d = q_win.shape
    N, Hkv, _ = k.shape
    _check(lib.slim_score_blocks_static(_dev(q_win, "q_win"), _dev(k, "k"), N, w, Hq, Hkv, d, block, unit,
                                        _dtype_code(k), _dev(scores, "scores"), _stream()), "slim_score_blocks_static")
    return scores


def slim_score_blocks_pooled(q_win: torch.Tensor, k: torch.Tensor, block: int, pooling: int,
                             scores: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """q_win[w,Hq,d], k[N,Hkv,d] -> scores[nb] float32 with one average- or max-pooled key per block (Table 3)."""
    lib = load_library()
    w, Hq, d = q_win.shape
    N, Hkv, _ = k.shape
    if scores is None:
        scores = torch.empty(n_blocks(N, block), dtype=torch.float32, device=k.device)
    need = lib.slim_score_blocks_workspace_bytes(Hkv, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=k.device)
    _check(lib.slim_score_blocks_pooled(_dev(q_win, "q_win"), _dev(k, "k"), N, w, Hq, Hkv, d, block, pooling,
                                        _dtype_code(k), _dev(scores, "scores"), _dev(workspace, "workspace"),
                                        workspace.numel(), _stream()), "slim_score_blocks_pooled")
    return scores


def slim_unit_keys(k: torch.Tensor, block: int, unit: int, k_rep: torch.Tensor | None = None) -> torch.Tensor:
    """k[N,Hkv,d] -> k_rep[nb, M, Hkv*d] float32 (Eq. 1 for every TokenUnit; missing units are zeros)."""
    lib = load_library()
    N, Hkv, d = k.shape
    M = (block + unit - 1) // unit
    if k_rep is None:
        k_rep = torch.empty(n_blocks(N, block), M, Hkv * d, dtype=torch.float32, device=k.device)
    _check(lib.slim_unit_keys(_dev(k, "k"), N, Hkv, d, block, unit, _dtype_code(k), _dev(k_rep, "k_rep"), _stream()),
           "slim_unit_keys")
    return k_rep


def slim_score_blocks_from_unit_keys(q_win: torch.Tensor, k_rep: torch.Tensor, n_tokens: int, n_kv_heads: int,
                                     block: int, unit: int, scores: torch.Tensor | None = None,
                                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """q_win[w,Hq,d], k_rep[nb,M,Hkv*d] float32 -> scores[nb] float32 (Eq. 2 on stored unit keys)."""
    lib = load_library()
    w, Hq, d = q_win.shape
    if scores is None:
        scores = torch.empty(n_blocks(n_tokens, block), dtype=torch.float32, device=k_rep.device)
    need = lib.slim_score_blocks_workspace_bytes(n_kv_heads, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=k_rep.device)
    _check(lib.slim_score_blocks_from_unit_keys(_dev(q_win, "q_win"), _dev(k_rep, "k_rep"), n_tokens, w, Hq, n_kv_heads,
                                                d, block, unit, _dtype_code(q_win), _dev(scores, "scores"),
                                                _dev(workspace, "workspace"), workspace.numel(), _stream()),
           "slim_score_blocks_from_unit_keys")
    return scores


def slim_decode_attn(q: torch.Tensor, gpu_pool: torch.Tensor, block_of_slot: torch.Tensor, block: int, n_prompt_tokens: int,
                     n_kv_heads: int, k_response: torch.Tensor | None = None, v_response: torch.Tensor | None = None,
                     layer_offset: int = 0, softmax_scale: float = 0.0, out: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """q[Hq,d] attends to the prompt tokens of the blocks in the slot pool and to the response tokens.
    gpu_pool[n_slots, ...]: per slot K[block,Hkv,d] then V[block,Hkv,d] at byte layer_offset."""
    lib = load_library()
    Hq, d = q.shape
    ns = block_of_slot.numel()
    slot_bytes = gpu_pool[0].numel() * gpu_pool.element_size() if ns else 0
    n_resp = 0 if k_response is None else k_response.shape[0]
    if out is None:
        out = torch.empty_like(q)
    need = lib.slim_decode_attn_workspace_bytes(ns, n_resp, Hq)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib.slim_decode_attn(_dev(q, "q"), _dev(gpu_pool, "gpu_pool"), slot_bytes, layer_offset,
                                _dev(block_of_slot, "block_of_slot"), ns, block, n_prompt_tokens, _dev(k_response, "k_response"),
                                _dev(v_response, "v_response"), n_resp, Hq, n_kv_heads, d, softmax_scale, _dtype_code(q),
                                _dev(out, "out"), _dev(workspace, "workspace"), workspace.numel(), _stream()),
           "slim_decode_attn")
    return out


def slim_gemv(w: torch.Tensor, x: torch.Tensor, w_up: torch.Tensor | None = None, scale: torch.Tensor | None = None,
              bias: torch.Tensor | None = None, residual: torch.Tensor | None = None, out: torch.Tensor | None = None):
    """Single-token projection w . x (scaled, + bias, + residual) or silu(w . x) * (w_up . x); x[k_in] -> [n_out]."""
    lib = load_library()
    n_out, k_in = w.shape
    if out is None:
        out = torch.empty(n_out, dtype=x.dtype, device=x.device)
    _check(lib.slim_gemv(_dev(w, "w"), _dev(w_up, "w_up"), _dev(x, "x"), _dev(scale, "scale"), _dev(bias, "bias"),
                         _dev(residual, "residual"), n_out, k_in, _dtype_code(x), _dev(out, "out"), _stream()), "slim_gemv")
    return out


def slim_decode_layer(shape: LayerShape, weights: dict, x_new: torch.Tensor, position: int, gpu_pool: torch.Tensor,
                      block_of_slot: torch.Tensor, n_prompt_tokens: int, k_response: torch.Tensor, v_response: torch.Tensor,
                      n_response: int, layer_offset: int = 0, workspace: torch.Tensor | None = None):
    """One layer for one decoded token.  k_response/v_response[>= n_response+1, Hkv, d]: row n_response is written.
    Returns (x_out[hidden], q[Hq, d])."""
    lib = load_library()
    ns = block_of_slot.numel()
    slot_bytes = gpu_pool[0].numel() * gpu_pool.element_size() if ns else 0
    x_out = torch.empty_like(x_new)
    q = torch.empty(shape.n_q_heads, shape.head_dim, dtype=x_new.dtype, device=x_new.device)
    need = lib.slim_decode_layer_workspace_bytes(C.byref(shape), ns, n_response)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x_new.device)
    wstruct = make_weights(weights)
    _check(lib.slim_decode_layer(C.byref(shape), C.byref(wstruct), _dev(x_new, "x_new"), position, _dev(gpu_pool, "gpu_pool"),
                                 slot_bytes, layer_offset, _dev(block_of_slot, "block_of_slot"), ns, n_prompt_tokens,
                                 _dev(k_response, "k_response"), _dev(v_response, "v_response"), n_response,
                                 _dev(x_out, "x_out"), _dev(q, "q"), _dev(workspace, "workspace"), workspace.numel(),
                                 _stream()), "slim_decode_layer")
    return x_out, q


def slim_rope_table(pos: torch.Tensor | None, n: int, head_dim: int, theta: float,
                    device=None) -> torch.Tensor:
    """table[n, head_dim] float32: cos then sin of the rotation angles of every position (None = 0..n-1)."""
    lib = load_library()
    dev = pos.device if pos is not None else device
    table = torch.empty(n, head_dim, dtype=torch.float32, device=dev)
    _check(lib.slim_rope_table(_dev(pos, "pos"), n, head_dim, theta, _dev(table, "table"), _stream()), "slim_rope_table")
    return table


def slim_window_query(q_win: torch.Tensor, n_kv_heads: int) -> torch.Tensor:
    """q_win[w,Hq,d] -> qt[Hkv*d] float32: mean over the window, head mean of Eq. (2) folded into kv groups."""
    lib = load_library()
    w, Hq, d = q_win.shape
    qt = torch.empty(n_kv_heads * d, dtype=torch.float32, device=q_win.device)
    _check(lib.slim_window_query(_dev(q_win, "q_win"), w, Hq, n_kv_heads, d, _dtype_code(q_win), _dev(qt, "qt"), _stream()),
           "slim_window_query")
    return qt


def slim_window_query_from_rows(rows: torch.Tensor, wq: torch.Tensor, bias: torch.Tensor | None, table: torch.Tensor,
                                n_q_heads: int, n_kv_heads: int, rstd: torch.Tensor | None = None) -> torch.Tensor:
    """qt[Hkv*128] float32 of Eq. (2) from the window's hidden rows [w, k_in] (row stride = rows.stride(0)): projection,
    rotation with table[w,128] and the window / head means without Query states in between."""
    lib = load_library()
    w, k_in = rows.shape
    qt = torch.empty(n_kv_heads * 128, dtype=torch.float32, device=rows.device)
    nbytes = lib.slim_window_query_from_rows_workspace_bytes(w, n_q_heads)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=rows.device)
    _check(lib.slim_window_query_from_rows(_dev(rows, "rows"), rows.stride(0), _dev(wq, "wq"), _dev(bias, "bias"),
                                           _dev(rstd, "rstd"), _dev(table, "table"), w, n_q_heads, n_kv_heads, k_in,
                                           _dev(qt, "qt"), _dev(ws, "workspace"), ws.numel(), _stream()),
           "slim_window_query_from_rows")
    return qt


def slim_linear_rope(a: torch.Tensor, w: torch.Tensor, bias: torch.Tensor | None, table: torch.Tensor, head_dim: int,
                     qt: torch.Tensor | None = None, rstd: torch.Tensor | None = None):
    """RoPE(a . w^T + bias) as [m, heads, head_dim]; with qt also the per-(token, head) score partials [m, heads];
    with rstd (from slim_row_rstd) the rows of a are raw and the projection is that of their RMSNorm (unit gain)."""
    lib = load_library()
    m, k_in = a.shape
    n_out = w.shape[0]
    heads = n_out // head_dim
    out = torch.empty(m, heads, head_dim, dtype=a.dtype, device=a.device)
    ts = torch.empty(m, heads, dtype=torch.float32, device=a.device) if qt is not None else None
    _check(lib.slim_linear_rope(_dev(a, "a"), a.stride(0), _dev(w, "w"), _dev(bias, "bias"), _dev(table, "table"), m, heads,
                                head_dim, k_in, n_out, _dtype_code(a), _dev(rstd, "rstd"), _dev(out, "out"), _dev(qt, "qt"),
                                _dev(ts, "ts"), _stream()), "slim_linear_rope")
    return (out, ts) if qt is not None else out


def slim_score_blocks_from_token_scores(token_scores: torch.Tensor, block: int, unit: int) -> torch.Tensor:
    """token_scores[N, Hkv] float32 -> scores[nb] float32 (unit means, block maximum)."""
    lib = load_library()
    N, H = token_scores.shape
    scores = torch.empty(n_blocks(N, block), dtype=torch.float32, device=token_scores.device)
    _check(lib.slim_score_blocks_from_token_scores(_dev(token_scores, "token_scores"), N, H, block, unit,
                                                   _dev(scores, "scores"), _stream()), "slim_score_blocks_from_token_scores")
    return scores


def slim_linear_pair(a: torch.Tensor, w_1: torch.Tensor, w_2: torch.Tensor, bias_1: torch.Tensor | None = None,
                     bias_2: torch.Tensor | None = None, rstd: torch.Tensor | None = None):
    """(a . w_1^T + bias_1, a . w_2^T + bias_2), rows scaled by rstd if given, in one launch."""
    lib = load_library()
    m, k_in = a.shape
    n1, n2 = w_1.shape[0], w_2.shape[0]
    o1 = torch.empty(m, n1, dtype=a.dtype, device=a.device)
    o2 = torch.empty(m, n2, dtype=a.dtype, device=a.device)
    _check(lib.slim_linear_pair(_dev(a, "a"), a.stride(0), _dev(w_1, "w_1"), _dev(bias_1, "bias_1"), n1, n1, _dev(o1, "o1"),
                                _dev(w_2, "w_2"), _dev(bias_2, "bias_2"), n2, n2, _dev(o2, "o2"), _dev(rstd, "rstd"), m, k_in,
                                _dtype_code(a), _stream()), "slim_linear_pair")
    return o1, o2


def slim_row_rstd(x: torch.Tensor, eps: float) -> torch.Tensor:
    """rstd[t] = 1/sqrt(mean(x[t,:]^2) + eps), float32."""
    lib = load_library()
    n, hidden = x.shape
    rstd = torch.empty(n, dtype=torch.float32, device=x.device)
    _check(lib.slim_row_rstd(_dev(x, "x"), n, hidden, eps, _dtype_code(x), _dev(rstd, "rstd"), _stream()), "slim_row_rstd")
    return rstd


def slim_rmsnorm_linear(a: torch.Tensor, w: torch.Tensor, rstd: torch.Tensor, bias: torch.Tensor | None = None) -> torch.Tensor:
    """RMSNorm(a) . w^T (+ bias) with unit gain: raw rows, their rstd applied to the accumulators."""
    lib = load_library()
    m, k_in = a.shape
    n_out = w.shape[0]
    out = torch.empty(m, n_out, dtype=a.dtype, device=a.device)
    _check(lib.slim_rmsnorm_linear(_dev(a, "a"), a.stride(0), _dev(w, "w"), _dev(bias, "bias"), _dev(rstd, "rstd"), m, n_out,
                                   k_in, n_out, _dtype_code(a), _dev(out, "out"), _stream()), "slim_rmsnorm_linear")
    return out


def slim_rmsnorm_swiglu_linear(a: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor, rstd: torch.Tensor) -> torch.Tensor:
    """silu(RMSNorm(a) . w_gate^T) * (RMSNorm(a) . w_up^T) with unit gain, as slim_rmsnorm_linear."""
    lib = load_library()
    m, k_in = a.shape
    n_out = w_gate.shape[0]
    out = torch.empty(m, n_out, dtype=a.dtype, device=a.device)
    _check(lib.slim_rmsnorm_swiglu_linear(_dev(a, "a"), a.stride(0), _dev(w_gate, "w_gate"), _dev(w_up, "w_up"),
                                          _dev(rstd, "rstd"), m, n_out, k_in, n_out, _dtype_code(a), _dev(out, "out"),
                                          _stream()), "slim_rmsnorm_swiglu_linear")
    return out


def slim_fold_gain(w: torch.Tensor, gain: torch.Tensor) -> torch.Tensor:
    """w[n, k] * gain[k], rounded to w's dtype: an RMSNorm gain folded into the projection that follows it."""
    lib = load_library()
    n_out, k_in = w.shape
    out = torch.empty_like(w)
    _check(lib.slim_fold_gain(_dev(w, "w"), _dev(gain, "gain"), n_out, k_in, _dtype_code(w), _dev(out, "out"), _stream()),
           "slim_fold_gain")
    return out


def _pinned(t: torch.Tensor, name: str):
    """Address of a pinned host tensor; under HIP's unified addressing the GPU reads it at the same address."""
    if t.is_cuda or not t.is_pinned():
        raise ValueError(f"{name} must be a pinned host tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def slim_kv_swap(candidate: torch.Tensor, gamma: float, slot_of_block: torch.Tensor, block_of_slot: torch.Tensor,
                 in_memory: torch.Tensor, gpu_pool: torch.Tensor, host_pool: torch.Tensor,
                 info: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """One step of Algorithm 1 on device state.  gpu_pool[n_slots, ...] on the GPU, host_pool[n_blocks, ...] pinned
    host memory with the same payload shape; the int32 maps are updated in place.  Returns info[8] (device)."""
    lib = load_library()
    nb, ns = slot_of_block.numel(), block_of_slot.numel()
    block_bytes = gpu_pool[0].numel() * gpu_pool.element_size()
    if host_pool.shape[0] != nb or gpu_pool.shape[0] != ns or \
            host_pool[0].numel() * host_pool.element_size() != block_bytes:
        raise ValueError("pool shapes do not match the maps")
    for t, name in ((candidate, "candidate"), (slot_of_block, "slot_of_block"), (block_of_slot, "block_of_slot"),
                    (in_memory, "in_memory")):
        if t.dtype != torch.int32:
            raise TypeError(f"{name} must be int32")
    dev = slot_of_block.device
    if info is None:
        info = torch.empty(8, dtype=torch.int32, device=dev)
    need = lib.slim_kv_swap_workspace_bytes(nb, ns)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib.slim_kv_swap(_dev(candidate, "candidate"), candidate.numel(), nb, float(gamma),
                            _dev(slot_of_block, "slot_of_block"), _dev(block_of_slot, "block_of_slot"),
                            _dev(in_memory, "in_memory"), ns, _dev(gpu_pool, "gpu_pool"), _pinned(host_pool, "host_pool"),
                            block_bytes, _dev(info, "info"), _dev(workspace, "workspace"), workspace.numel(), _stream()),
           "slim_kv_swap")
    return info


def slim_select_topk_blocks(scores: torch.Tensor, n_keep: int, force_flags: int = FORCE_FIRST | FORCE_LAST,
                            kept: torch.Tensor | None = None) -> torch.Tensor:
    """scores[nb] float32 -> ascending int32 indices of the kept blocks."""
    lib = load_library()
    nb = scores.numel()
    if kept is None:
        kept = torch.empty(min(max(n_keep, 1), nb), dtype=torch.int32, device=scores.device)
    _check(lib.slim_select_topk_blocks(_dev(scores, "scores"), nb, n_keep, force_flags, _dev(kept, "kept"), _stream()),
           "slim_select_topk_blocks")
    return kept


def slim_compact_tokens(src: torch.Tensor, kept: torch.Tensor, block: int, pos_in: torch.Tensor | None = None,
                        want_pos: bool = True, n_out: int | None = None):
    """src[N, row] -> (dst[n', row], pos_out[n'] or None).  `kept` is a device int32 tensor; n' is
    computed on the host assuming the short last block (if any) is among the kept ones unless given."""
    lib = load_library()
    N = src.shape[0]
    row = src[0].numel()
    n_keep = kept.numel()
    if n_out is None:
        n_out = lib.slim_kept_tokens(N, block, n_keep)
    dst = torch.empty((n_out,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    pos_out = torch.empty(n_out, dtype=torch.int32, device=src.device) if want_pos else None
    _check(lib.slim_compact_tokens(_dev(src, "src"), _dev(pos_in, "pos_in"), _dev(kept, "kept"), n_keep, block, N,
                                   row, _dtype_code(src), _dev(dst, "dst"), _dev(pos_out, "pos_out"), _stream()),
           "slim_compact_tokens")
    return dst, pos_out


def slim_prefill_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, softmax_scale: float = 0.0,
                      out: torch.Tensor | None = None) -> torch.Tensor:
    """q[n,Hq,d], k/v[n,Hkv,d] -> out[n,Hq,d], causal GQA attention."""
    lib = load_library()
    n, Hq, d = q.shape
    Hkv = k.shape[1]
    if out is None:
        out = torch.empty_like(q)
    _check(lib.slim_prefill_attn(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), n, Hq, Hkv, d, softmax_scale,
                                 _dtype_code(q), _dev(out, "out"), _stream()), "slim_prefill_attn")
    return out


def slim_rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float, out: torch.Tensor | None = None) -> torch.Tensor:
    lib = load_library()
    n, hidden = x.shape
    if out is None:
        out = torch.empty_like(x)
    _check(lib.slim_rmsnorm(_dev(x, "x"), _dev(gain, "gain"), n, hidden, eps, _dtype_code(x), _dev(out, "out"),
                            _stream()), "slim_rmsnorm")
    return out


def slim_rope(x: torch.Tensor, pos: torch.Tensor | None, theta: float) -> torch.Tensor:
    """In place on x[n,H,d]."""
    lib = load_library()
    n, H, d = x.shape
    _check(lib.slim_rope(_dev(x, "x"), _dev(pos, "pos"), n, H, d, theta, _dtype_code(x), _stream()), "slim_rope")
    return x


def slim_linear(a: torch.Tensor, w: torch.Tensor, residual: torch.Tensor | None = None,
                out: torch.Tensor | None = None) -> torch.Tensor:
    """a[m,k] . w[n,k]^T (+ residual[m,n])."""
    lib = load_library()
    m, k = a.shape
    n = w.shape[0]
    if out is None:
        out = torch.empty((m, n), dtype=a.dtype, device=a.device)
    _check(lib.slim_linear(_dev(a, "a"), k, _dev(w, "w"), _dev(residual, "residual"), m, n, k, n, _dtype_code(a),
                           _dev(out, "out"), _stream()), "slim_linear")
    return out


def slim_linear_bias(a: torch.Tensor, w: torch.Tensor, bias: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """a[m,k] . w[n,k]^T + bias[n]."""
    lib = load_library()
    m, k = a.shape
    n = w.shape[0]
    if out is None:
        out = torch.empty((m, n), dtype=a.dtype, device=a.device)
    _check(lib.slim_linear_bias(_dev(a, "a"), k, _dev(w, "w"), _dev(bias, "bias"), m, n, k, n, _dtype_code(a),
                                _dev(out, "out"), _stream()), "slim_linear_bias")
    return out


def slim_swiglu_linear(a: torch.Tensor, w_gate: torch.Tensor, w_up: torch.Tensor,
                       out: torch.Tensor | None = None) -> torch.Tensor:
    lib = load_library()
    m, k = a.shape
    n = w_gate.shape[0]
    if out is None:
        out = torch.empty((m, n), dtype=a.dtype, device=a.device)
    _check(lib.slim_swiglu_linear(_dev(a, "a"), k, _dev(w_gate, "w_gate"), _dev(w_up, "w_up"), m, n, k, n,
                                  _dtype_code(a), _dev(out, "out"), _stream()), "slim_swiglu_linear")
    return out


def make_shape(hidden, n_q_heads, n_kv_heads, head_dim, ffn, block, unit, window, dtype: torch.dtype,
               rope_theta=500000.0, rms_eps=1e-5, flags=FORCE_FIRST | FORCE_LAST, scoring=0, placement=0) -> LayerShape:
    """scoring: 0 = TokenUnits (Eq. 1-2), POOL_AVG, POOL_MAX (the pooled baselines of Table 3);
    placement: PRUNE_BEFORE_ATTENTION (measured path) or PRUNE_AFTER_ATTENTION (Section 4.1's order)."""
    code = BF16 if dtype == torch.bfloat16 else F32
    return LayerShape(hidden, n_q_heads, n_kv_heads, head_dim, ffn, block, unit, window, rope_theta, rms_eps, code,
                      flags, scoring, placement)


def make_weights(w: dict) -> LayerWeights:
    """`w` maps the field names of slim_layer_weights to GPU tensors (kept alive by the caller); the
    biases bq/bk/bv may be absent (NULL), and so may the gains g_attn/g_ffn once they are folded into the
    projections that follow them (slim_fold_gain)."""
    return LayerWeights(*[_dev(w.get(n), n) for n, _ in LayerWeights._fields_])


def pruned_layer_workspace_bytes(shape: LayerShape, n_tokens: int, n_keep: int) -> int:
    return load_library().slim_pruned_layer_workspace_bytes(C.byref(shape), n_tokens, n_keep)


def slim_pruned_layer(shape: LayerShape, weights: dict, x: torch.Tensor, pos: torch.Tensor | None, n_keep: int,
                      workspace: torch.Tensor | None = None, out: dict | None = None, want_scores: bool = True):
    """One pruned prefill layer.  Returns dict(x=[n',hidden], pos=[n'], kept=[n_keep], scores=[nb] or None).
    `out` may carry preallocated x / pos / kept / scores tensors (for timing loops)."""
    lib = load_library()
    N = x.shape[0]
    nb = n_blocks(N, shape.block)
    prune = n_keep < nb
    n_out = lib.slim_kept_tokens(N, shape.block, n_keep) if prune else N
    dev = x.device
    out = dict(out) if out else {}
    if "x" not in out:
        out["x"] = torch.empty((n_out, shape.hidden), dtype=x.dtype, device=dev)
    if "pos" not in out:
        out["pos"] = torch.empty(n_out, dtype=torch.int32, device=dev)
    if "kept" not in out:
        out["kept"] = torch.empty(min(n_keep, nb), dtype=torch.int32, device=dev)
    if "scores" not in out:
        out["scores"] = torch.empty(nb, dtype=torch.float32, device=dev) if (want_scores and prune) else None
    need = lib.slim_pruned_layer_workspace_bytes(C.byref(shape), N, n_keep)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    wstruct = make_weights(weights)
    _check(lib.slim_pruned_layer(C.byref(shape), C.byref(wstruct), _dev(x, "x"), _dev(pos, "pos"), N, n_keep,
                                 _dev(out["x"], "x_out"), _dev(out["pos"], "pos_out"), _dev(out["kept"], "kept"),
                                 _dev(out["scores"], "scores"), _dev(workspace, "workspace"), workspace.numel(),
                                 _stream()), "slim_pruned_layer")
    return out


def schedule_keep_counts(n_tokens: int, block: int, n_layers: int, schedule: dict) -> list:
    """Per-layer n_keep for a {layer: keep ratio of the incoming blocks} schedule (0 = Preserve layer):
    ceil(ratio * incoming blocks), at least the two forced blocks."""
    import math
    out, n = [], n_tokens
    for l in range(n_layers):
        nb = n_blocks(n, block)
        if l in schedule:
            keep = int(min(nb, max(min(2, nb), math.ceil(schedule[l] * nb - 1e-12))))
            out.append(keep)
            n = load_library().slim_kept_tokens(n, block, keep)
        else:
            out.append(0)
    return out


def slim_prefill_model(shape: LayerShape, layer_weights: list, x: torch.Tensor, pos: torch.Tensor | None,
                       n_keep: list, workspace: torch.Tensor | None = None, out: dict | None = None):
    """All layers in order (Preserve layers where n_keep[l] == 0).  `layer_weights` is a list of dicts of GPU
    tensors.  Returns dict(x=[n_final, hidden], pos=[n_final], kept=concatenated kept sets of the pruning layers)."""
    lib = load_library()
    L = len(layer_weights)
    N = x.shape[0]
    keep_arr = (C.c_int * L)(*[int(k) for k in n_keep])
    n_final = lib.slim_prefill_model_tokens(C.byref(shape), L, keep_arr, N)
    if n_final <= 0:
        raise SlimError(-1, "slim_prefill_model", "invalid schedule")
    warr = (LayerWeights * L)(*[make_weights(w) for w in layer_weights])
    dev = x.device
    out = dict(out) if out else {}
    if "x" not in out:
        out["x"] = torch.empty((n_final, shape.hidden), dtype=x.dtype, device=dev)
    if "pos" not in out:
        out["pos"] = torch.empty(n_final, dtype=torch.int32, device=dev)
    if "kept" not in out:
        out["kept"] = torch.empty(max(1, sum(int(k) for k in n_keep)), dtype=torch.int32, device=dev)
    need = lib.slim_prefill_model_workspace_bytes(C.byref(shape), L, keep_arr, N)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib.slim_prefill_model(C.byref(shape), warr, L, keep_arr, _dev(x, "x"), _dev(pos, "pos"), N,
                                  _dev(out["x"], "x_out"), _dev(out["pos"], "pos_out"), _dev(out["kept"], "kept"),
                                  _dev(workspace, "workspace"), workspace.numel(), _stream()), "slim_prefill_model")
    return out


_probe_lib = None


def load_probe_library() -> C.CDLL:
    """Load libslim_probe.so: the measurement probes of bench.py, kept out of the method's library."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise FileNotFoundError(f"{PROBE_LIB_PATH} not found: build it with __graft_entry__.build()")
        lib = C.CDLL(PROBE_LIB_PATH)
        lib.slim_probe_mfma_flops.restype = C.c_double
        lib.slim_probe_mfma_flops.argtypes = [C.c_int, C.c_int]
        lib.slim_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        lib.slim_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        _probe_lib = lib
    return _probe_lib


def probe_mfma(n_workgroups: int, iters: int, sink: torch.Tensor, random_operands: bool = False) -> float:
    """Enqueue the register-only MFMA loop; returns its flop count."""
    lib = load_probe_library()
    _check(lib.slim_probe_mfma(n_workgroups, iters, int(random_operands), _dev(sink, "sink"), _stream()),
           "slim_probe_mfma")
    return lib.slim_probe_mfma_flops(n_workgroups, iters)


def probe_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Enqueue a plain device copy of src into dst; returns the bytes copied."""
    nbytes = src.numel() * src.element_size()
    _check(load_probe_library().slim_probe_copy(_dev(src, "src"), _dev(dst, "dst"), nbytes, _stream()), "slim_probe_copy")
    return nbytes
