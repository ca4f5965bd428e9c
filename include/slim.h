/*
 * libslim -- the pruned prefill layer of SlimInfer (arXiv 2508.06447) for AMD MI355X (gfx950).
 *
 * C ABI.  Conventions shared by every entry point:
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless marked "host".
 *     The library never allocates, frees or keeps a pointer after the call returns.  What it keeps between
 *     calls is derived, immutable once computed and guarded for concurrent callers: device properties, the
 *     one-time raising of kernels' LDS limits, a memo of tile-schedule choices per problem shape, and the
 *     per-device address of the scratch array of slim_score_blocks_static.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call only enqueues
 *     kernels on that stream; it never synchronises with the host.
 *   - `dtype`: SLIM_F32 (0) = IEEE binary32, SLIM_BF16 (1) = bfloat16.  It is the type of every
 *     activation and weight tensor of the call.  Block scores are always float; indices are int32.
 *   - Tensors are dense row-major; "x[n, H, d]" means d is contiguous.
 *   - Return value: SLIM_OK (0) or a negative error code.  Argument errors (INVALID_ARG, UNSUPPORTED,
 *     WORKSPACE_TOO_SMALL) are found before the first launch: nothing has been enqueued.  SLIM_HIP_ERROR means
 *     the runtime refused a launch; a call that enqueues several kernels (the layer, the model, the decode
 *     layer, the two-kernel stage calls) may then already have enqueued the earlier ones, and its outputs
 *     and workspace are undefined.
 *   - Calls on different streams may overlap as long as their buffers (workspace included) are
 *     distinct.
 *
 * Notation (Section 4.2 of the paper): the N prompt tokens are split into blocks of `block`
 * tokens (nb = ceil(N/block)); each block into TokenUnits of `unit` tokens; q_l is the mean Query
 * state of the last `window` tokens; Hq / Hkv are the numbers of query / key-value heads and
 * query head h reads kv head h / (Hq/Hkv).
 */
#ifndef SLIM_H
#define SLIM_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SLIM_F32 = 0, SLIM_BF16 = 1 };

enum {
    SLIM_OK = 0,
    SLIM_INVALID_ARG = -1,        /* null pointer, non-positive size, Hq % Hkv != 0, bad n_keep ... */
    SLIM_UNSUPPORTED = -2,        /* a shape or dtype the kernels do not cover (see each call)      */
    SLIM_WORKSPACE_TOO_SMALL = -3,
    SLIM_HIP_ERROR = -4           /* a launch failed; slim_last_hip_error() has the runtime's text  */
};

/* Force flags for slim_select_topk_blocks / layer flags. */
enum { SLIM_FORCE_FIRST = 1u, SLIM_FORCE_LAST = 2u };

const char* slim_status_string(int code);
/* Text of the last HIP runtime error seen by this thread inside the library ("" if none). */
const char* slim_last_hip_error(void);

/* ------------------------------------------------------------------------------------------------
 * Block importance scores -- Eq. (1) and Eq. (2), Section 4.2.
 *   k_rep(j,m) = mean of the Key states of TokenUnit m of block j               (Eq. 1)
 *   scores[j]  = max_m (1/Hq) sum_h  q_l^h . k_rep^{h/(Hq/Hkv)}(j,m)             (Eq. 2)
 * with q_l^h the mean over the `window` rows of q_win.  Plain dot products: no softmax, no
 * 1/sqrt(d).  A short last block / last unit is averaged over the tokens it really has.
 *   q_win  [window, Hq, d]  Query states of the local window (post-RoPE), dtype
 *   k      [N, Hkv, d]      Key states of all prompt tokens (post-RoPE), dtype
 *   scores [nb]             out, float
 *   workspace               >= slim_score_blocks_workspace_bytes(Hkv, d) bytes, 256-byte aligned;
 *                           holds the head-group-summed window query between the two kernels.
 * Errors: INVALID_ARG (null, sizes < 1, Hq % Hkv, unit > block), UNSUPPORTED ((Hkv*d) % 8 != 0 for
 * bf16 or % 4 for f32, or Hkv*d > 8192), WORKSPACE_TOO_SMALL.
 */
size_t slim_score_blocks_workspace_bytes(int n_kv_heads, int head_dim);
int slim_score_blocks(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads,
                      int n_kv_heads, int head_dim, int block, int unit, int dtype, float* scores,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * slim_score_blocks for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results (bit for bit) as slim_score_blocks, minus the workspace: the head-group-summed window query
 * goes through a 32 KiB array that lives in the library's device image (one copy per GPU, held until the
 * process ends).  The call allocates and frees nothing.  The first call on a device looks up that
 * device's copy of the array (one runtime query, no allocation; make that first call outside a capture).
 * Limit: Hkv * head_dim <= 8192 (UNSUPPORTED beyond, as for slim_score_blocks).  Every call on one GPU
 * shares that GPU's array: calls that overlap on one GPU (different streams, or different threads)
 * race on it, so serialise them; the array keeps the last call's window query and every call overwrites
 * all of it that it reads.  Other errors as slim_score_blocks.
 */
int slim_score_blocks_static(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads,
                             int n_kv_heads, int head_dim, int block, int unit, int dtype, float* scores,
                             void* stream);

/* ------------------------------------------------------------------------------------------------
 * Pooled block scores -- the two baselines of the scoring ablation (Table 3, "Block Importance
 * Scoring Algorithm"): one representative key per block, the average of its token Key states
 * (SLIM_POOL_AVG, which is Eq. 1-2 with a single TokenUnit per block) or their element-wise maximum
 * (SLIM_POOL_MAX), scored like Eq. (2):  scores[j] = (1/Hq) sum_h q_l^h . k_pool^{h/(Hq/Hkv)}(j).
 * Arguments, layouts, workspace and errors as slim_score_blocks (no unit); INVALID_ARG for another
 * pooling value.
 */
enum { SLIM_POOL_AVG = 1, SLIM_POOL_MAX = 2 };
int slim_score_blocks_pooled(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads,
                             int n_kv_heads, int head_dim, int block, int pooling, int dtype,
                             float* scores, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * The same scores from stored representative keys -- Section 4.2 in its decode-time form: during
 * decoding the window is the most recently decoded tokens, and the Key states of inactive prompt blocks
 * may live in CPU memory (Section 4.3), so Eq. (1) is evaluated once and kept on the GPU.
 *   slim_unit_keys:  k[N, Hkv, d] (dtype) -> k_rep[nb, M, Hkv*d] float, M = ceil(block/unit); entry (j, m)
 *                    is Eq. (1) for TokenUnit m of block j, averaged over the tokens it really has; units
 *                    past the end of the prompt are written as zeros and never read.
 *   slim_score_blocks_from_unit_keys:  Eq. (2) on k_rep with the window q_win[window, Hq, d] (dtype);
 *                    scores[nb] float.  Equal to slim_score_blocks on the same keys up to the order of
 *                    the float additions.  Workspace as slim_score_blocks.
 * k_rep is caller-owned, 16-byte aligned, nb*M*Hkv*d floats.  Errors as slim_score_blocks.
 */
int slim_unit_keys(const void* k, int n_tokens, int n_kv_heads, int head_dim, int block, int unit, int dtype,
                   float* k_rep, void* stream);
int slim_score_blocks_from_unit_keys(const void* q_win, const float* k_rep, int n_tokens, int window,
                                     int n_q_heads, int n_kv_heads, int head_dim, int block, int unit,
                                     int dtype, float* scores, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* ------------------------------------------------------------------------------------------------
 * Block selection -- last paragraph of Section 4.2: the first block (attention sink) is always
 * kept; here the last block can be forced as well.  The remaining n_keep - #forced slots go to the
 * other blocks by (score descending, block index ascending).  n_keep counts the forced blocks.
 *   scores      [n_blocks] float (NaN: unspecified which blocks win)
 *   kept_blocks [min(n_keep, n_blocks)] out, int32, ascending
 * n_keep >= n_blocks keeps every block.  Errors: INVALID_ARG (null, n_blocks < 1,
 * n_keep < #forced blocks).
 */
int slim_select_topk_blocks(const float* scores, int n_blocks, int n_keep, unsigned force_flags,
                            int* kept_blocks, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Hidden-state pruning -- Section 4.1 ("Slim layers"): rows of the kept blocks are gathered into a
 * dense shorter sequence, original positions ride along for RoPE.
 *   src         [N, row_elems] dtype          dst     [n', row_elems] out
 *   pos_in      [N] int32 or NULL (= 0..N-1)  pos_out [n'] int32 out, or NULL
 *   kept_blocks [n_keep] int32, ascending, device.  An entry outside [0, nb) is skipped.
 * n' = sum of the kept blocks' lengths (only block nb-1 can be short).  dst must not overlap src.
 * Errors: INVALID_ARG (null src/dst/kept, sizes < 1, n_keep > nb).
 */
int slim_compact_tokens(const void* src, const int* pos_in, const int* kept_blocks, int n_keep,
                        int block, int n_tokens, int row_elems, int dtype, void* dst, int* pos_out,
                        void* stream);

/* ------------------------------------------------------------------------------------------------
 * Causal grouped-query prefill attention over a (compacted) sequence -- the "Attention" stage of
 * Fig. 2:  out[i,h,:] = sum_{j<=i} softmax_j(scale * q[i,h,:].k[j,g,:]) v[j,g,:],  g = h/(Hq/Hkv).
 *   q, out [n, Hq, d]   k, v [n, Hkv, d]   all dtype;  softmax_scale 0 => 1/sqrt(d)
 * Causality is in sequence index (rows are in ascending original position after compaction).
 * Errors: INVALID_ARG, UNSUPPORTED (bf16: d != 128; f32: d > 128 or d % 4 != 0).
 */
int slim_prefill_attn(const void* q, const void* k, const void* v, int n, int n_q_heads,
                      int n_kv_heads, int head_dim, float softmax_scale, int dtype, void* out,
                      void* stream);

/* ------------------------------------------------------------------------------------------------
 * Per-token building blocks of the layer ("QKV Generation" and "FFN" of Fig. 2).  Exposed so that
 * each kernel can be checked and timed on its own.
 */
/* out[t,:] = gain * x[t,:] / sqrt(mean(x[t,:]^2) + eps).  x, out [n, hidden], gain [hidden]. */
int slim_rmsnorm(const void* x, const void* gain, int n, int hidden, float eps, int dtype,
                 void* out, void* stream);
/* In-place rotate-half RoPE on x[n, H, d] at positions pos[n] (NULL = 0..n-1):
 * pair (i, i+d/2) is turned by pos * theta^(-2i/d); angles are formed in double precision. */
int slim_rope(void* x, const int* pos, int n, int n_heads, int head_dim, float theta, int dtype,
              void* stream);
/* out[m, n_out] = a[m, k_in] . w[n_out, k_in]^T (+ residual[m, n_out] if not NULL; may alias out).
 * Row strides in elements: lda for a, ldo for out and residual.  bf16 needs k_in % 8 == 0. */
int slim_linear(const void* a, int lda, const void* w, const void* residual, int m, int n_out,
                int k_in, int ldo, int dtype, void* out, void* stream);
/* out[m, n_out] = a . w^T + bias[n_out] (the Q/K/V projections of models that carry a bias; the sum is
 * formed in float and rounded once).  bias: n_out elements of dtype, 16-byte aligned. */
int slim_linear_bias(const void* a, int lda, const void* w, const void* bias, int m, int n_out, int k_in,
                     int ldo, int dtype, void* out, void* stream);
/* out[m, n_out] = silu(a . w_gate^T) * (a . w_up^T), both weights [n_out, k_in]. */
int slim_swiglu_linear(const void* a, int lda, const void* w_gate, const void* w_up, int m,
                       int n_out, int k_in, int ldo, int dtype, void* out, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Key-first scoring pipeline: the same Eq. (1)-(2) scores and the same rotated Key/Query states ("QKV
 * Generation" of Fig. 2), with RoPE and the per-token part of the score folded into the projection's
 * epilogue so that the Key states are written once and not re-read for scoring.  slim_pruned_layer uses
 * these kernels for the Key projection of bf16 heads of 128; they are exposed to be checked and timed on
 * their own.
 *   slim_rope_table:   table[n, head_dim] float; row t = cos of the head_dim/2 rotation angles of position
 *                      pos[t] (NULL = 0..n-1), then their sines; angle i = pos * theta^(-2i/head_dim), formed and
 *                      reduced to [-pi, pi] in double, evaluated in float (within 4e-7 of the double result).
 *   slim_window_query: qt[Hkv*d] float = (1/(window*Hq)) sum over the window rows and over the query heads of
 *                      each kv group of q_win[window, Hq, d]: Eq. (2)'s q_l with its head mean folded in.
 *   slim_window_query_from_rows (+ _workspace_bytes): the same qt, straight from the hidden rows of the window:
 *                      qt = (1/(window*Hq)) sum over rows t and heads of the group of RoPE_t(rows[t] . wq_h^T *
 *                      rstd[t] + bq_h), with no Query states written in between (the projection is kept in float
 *                      through the rotation and the means, so it differs from projecting to bf16 first by that
 *                      rounding).  rows[window, k_in] bf16 with row stride lda; wq [Hq*128, k_in]; bias NULL = none;
 *                      rstd[window] as for slim_linear_rope (NULL = rows are used as they are); table[window, 128] =
 *                      slim_rope_table of the window rows' positions.  The projection is a skinny product whose
 *                      reduction dimension is split over workgroups; the partial sums go through `workspace` and are
 *                      added in a fixed order.  bf16, head_dim 128, k_in % 64 == 0, lda % 8 == 0, window <= 256,
 *                      16-byte aligned pointers: UNSUPPORTED otherwise; WORKSPACE_TOO_SMALL.
 *   slim_linear_rope:  out[m, n_heads, 128] = RoPE(a[m, k_in] . w^T + bias) (bias NULL = none), rotation in float
 *                      on the unrounded projection, one rounding.  With qt != NULL (then n_heads = Hkv) also
 *                      token_scores[m, n_heads] float = the rounded key of (token, head) dotted with qt's slice.
 *                      rstd != NULL: a holds raw residual rows, rstd[m] their 1/rms from slim_row_rstd, and the
 *                      projection is that of their RMSNorm with unit gain (see slim_rmsnorm_linear); NULL: a is
 *                      used as it is.
 *                      bf16 only; head_dim 128; k_in % 64 == 0; lda, ldo (elements) % 8 == 0; all pointers 16-byte
 *                      aligned.  UNSUPPORTED otherwise.
 *   slim_score_blocks_from_token_scores: scores[nb] = max over the block's TokenUnits of the mean over the
 *                      unit's tokens of sum_h token_scores[t, h]; equal to slim_score_blocks on the same keys up
 *                      to the order of the float additions.
 */
int slim_rope_table(const int* pos, int n, int head_dim, float theta, float* table, void* stream);
int slim_window_query(const void* q_win, int window, int n_q_heads, int n_kv_heads, int head_dim, int dtype,
                      float* qt, void* stream);
size_t slim_window_query_from_rows_workspace_bytes(int window, int n_q_heads);
int slim_window_query_from_rows(const void* rows, int lda, const void* wq, const void* bias, const float* rstd,
                                const float* table, int window, int n_q_heads, int n_kv_heads, int k_in,
                                float* qt, void* workspace, size_t workspace_bytes, void* stream);
int slim_linear_rope(const void* a, int lda, const void* w, const void* bias, const float* table, int m,
                     int n_heads, int head_dim, int k_in, int ldo, int dtype, const float* rstd, void* out,
                     const float* qt, float* token_scores, void* stream);
int slim_score_blocks_from_token_scores(const float* token_scores, int n_tokens, int n_kv_heads, int block,
                                        int unit, float* scores, void* stream);

/* ------------------------------------------------------------------------------------------------
 * RMSNorm fused into the projection that consumes it (the norms in front of "QKV Generation" and "FFN" of
 * Fig. 2).  slim_row_rstd reads the rows once and leaves rstd[t] = 1/sqrt(mean(x[t,:]^2) + eps) (float); the
 * projections then read the RAW rows and scale their accumulators by rstd[m] before the epilogue:
 *   out = RMSNorm(a) . w^T (+ bias),   or   silu(RMSNorm(a) . w_gate^T) * (RMSNorm(a) . w_up^T),
 * with a UNIT gain, and the normalised rows are never written or re-read (the two-kernel route also rounds them
 * to bf16 first; this one does not).  A model's gain vector g is folded into the weights once with
 * slim_fold_gain: out[n, k] = w[n, k] * g[k] (rounded to dtype), since (g * x_hat) . w^T = x_hat . (w * g)^T.
 * The projections: bf16 only, k_in % 64 == 0, lda % 8 == 0, 16-byte aligned pointers; UNSUPPORTED otherwise.
 * slim_row_rstd and slim_fold_gain take either dtype; slim_fold_gain's out may alias w.
 */
int slim_row_rstd(const void* x, int n, int hidden, float eps, int dtype, float* rstd, void* stream);
int slim_rmsnorm_linear(const void* a, int lda, const void* w, const void* bias, const float* rstd, int m,
                        int n_out, int k_in, int ldo, int dtype, void* out, void* stream);
int slim_rmsnorm_swiglu_linear(const void* a, int lda, const void* w_gate, const void* w_up, const float* rstd,
                               int m, int n_out, int k_in, int ldo, int dtype, void* out, void* stream);
int slim_fold_gain(const void* w, const void* gain, int n_out, int k_in, int dtype, void* out, void* stream);
/* Two projections of the same rows in one launch (the layer's Query and Value projections: one launch of
 * n_1 + n_2 features fills the chip better than one of n_1 and one of n_2):
 *   out_1[m, n_1] = s . (a . w_1^T) + bias_1,   out_2[m, n_2] = s . (a . w_2^T) + bias_2,
 * s = rstd[m] (fused RMSNorm as above) or 1 when rstd is NULL; both biases or neither.  Results are bit-identical
 * to the two single launches.  bf16 only, m > 128, k_in % 64 == 0, lda % 8 == 0, 16-byte aligned pointers;
 * UNSUPPORTED otherwise. */
int slim_linear_pair(const void* a, int lda, const void* w_1, const void* bias_1, int n_1, int ldo_1, void* out_1,
                     const void* w_2, const void* bias_2, int n_2, int ldo_2, void* out_2, const float* rstd,
                     int m, int k_in, int dtype, void* stream);

/* ------------------------------------------------------------------------------------------------
 * The pruned prefill layer: score -> select -> compact -> attention -> FFN on the kept tokens.
 */
typedef struct slim_layer_shape {
    int hidden, n_q_heads, n_kv_heads, head_dim, ffn;
    int block, unit, window;
    float rope_theta, rms_eps;
    int dtype;
    unsigned flags;               /* SLIM_FORCE_FIRST | SLIM_FORCE_LAST */
    int scoring;                  /* 0 = TokenUnits (Eq. 1-2), SLIM_POOL_AVG, SLIM_POOL_MAX (Table 3) */
    int placement;                /* SLIM_PRUNE_BEFORE_ATTENTION (0) or SLIM_PRUNE_AFTER_ATTENTION       */
} slim_layer_shape;

/* Where a pruning layer drops the blocks.  BEFORE (the measured path): score, select, compact, then
 * attention over the kept tokens only.  AFTER (the order Section 4.1 words: the decision is taken
 * right after Attention): Query, Key and Value states and attention for all N tokens, then the
 * attention output and the residual are compacted, and the output projection and FFN run on the kept
 * tokens.  Scores, kept set and positions are the same in both; AFTER needs a larger workspace. */
enum { SLIM_PRUNE_BEFORE_ATTENTION = 0, SLIM_PRUNE_AFTER_ATTENTION = 1 };

typedef struct slim_layer_weights {   /* device pointers, [out_features, in_features] row-major */
    /* g_attn / g_ffn: RMSNorm gains [hidden], or NULL when the gain has been folded into wq, wk, wv / w_gate,
     * w_up (slim_fold_gain; nothing to fold for unit gains).  With NULL only the row statistics are computed,
     * the projections apply them to their accumulators, and no normalised copy of the hidden states is
     * written (bf16, hidden % 64 == 0; UNSUPPORTED otherwise). */
    const void *g_attn, *wq, *wk, *wv, *wo, *g_ffn, *w_gate, *w_up, *w_down;
    const void *bq, *bk, *bv;         /* biases of the Q/K/V projections ([out_features], 16-byte aligned)
                                         or NULL: the paper's LLaMA models have none, its Qwen2.5 models do */
} slim_layer_weights;

/* Tokens left after keeping n_keep of the blocks of an n_tokens sequence (last block among them). */
int slim_kept_tokens(int n_tokens, int block, int n_keep);

size_t slim_pruned_layer_workspace_bytes(const slim_layer_shape* s, int n_tokens, int n_keep);

/* One layer.  With n_keep >= nb it is a Preserve layer (no scoring, nothing dropped).  Otherwise:
 * Key states of all N tokens and Query states of the last `window` tokens are formed, blocks are
 * scored (Eq. 1-2) and selected, hidden rows / positions / keys of the kept blocks are compacted,
 * and attention, projections and the SwiGLU FFN run on the n' kept tokens only.
 *   s, w            host structs (w holds device pointers)
 *   x_in [N, hidden], pos_in [N] int32 (NULL = 0..N-1)
 *   x_out [n', hidden] out, pos_out [n'] out, kept_blocks_out [min(n_keep, nb)] out (may be NULL
 *   for a Preserve layer), scores_out [nb] float out or NULL.
 *   workspace: >= slim_pruned_layer_workspace_bytes(...) bytes, 256-byte aligned.
 * x_out must not overlap x_in.  Without SLIM_FORCE_LAST, N must be a multiple of block.
 * Errors: as the stage calls, plus WORKSPACE_TOO_SMALL.
 */
int slim_pruned_layer(const slim_layer_shape* s, const slim_layer_weights* w, const void* x_in,
                      const int* pos_in, int n_tokens, int n_keep, void* x_out, int* pos_out,
                      int* kept_blocks_out, float* scores_out, void* workspace,
                      size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Preserve/Slim schedule -- Section 4.1: the layers run in order; a layer whose n_keep[l] is smaller
 * than its incoming block count prunes its incoming sequence to n_keep[l] blocks (forced blocks
 * included), and the surviving set then propagates unchanged until the next pruning layer.
 * Because whole blocks are kept in order, the compacted sequence is re-blocked by `block` and its
 * blocks are the surviving original ones.
 *   layers   host array [n_layers] of slim_layer_weights (device pointers inside)
 *   n_keep   host array [n_layers]; 0 or >= incoming blocks = Preserve layer
 *   x_in [N, hidden], pos_in [N] int32 or NULL (= 0..N-1)
 *   x_out [n_final, hidden], pos_out [n_final] int32 (NULL allowed), n_final = slim_prefill_model_tokens(...)
 *   kept_blocks_out: int32, the kept sets of the pruning layers one after another (each in the block
 *                    numbering of that layer's incoming sequence), or NULL
 *   workspace >= slim_prefill_model_workspace_bytes(...), 256-byte aligned
 * Output = residual stream after the last layer (no final norm).  Errors as slim_pruned_layer.
 */
int slim_prefill_model_tokens(const slim_layer_shape* s, int n_layers, const int* n_keep, int n_tokens);
size_t slim_prefill_model_workspace_bytes(const slim_layer_shape* s, int n_layers, const int* n_keep,
                                          int n_tokens);
int slim_prefill_model(const slim_layer_shape* s, const slim_layer_weights* layers, int n_layers,
                       const int* n_keep, const void* x_in, const int* pos_in, int n_tokens, void* x_out,
                       int* pos_out, int* kept_blocks_out, void* workspace, size_t workspace_bytes,
                       void* stream);

/* ------------------------------------------------------------------------------------------------
 * Overlap-aware KV swapping -- Algorithm 1, Section 4.3, one inference step, decided and carried out on
 * the GPU without a host round trip:
 *   overlap = |candidate ∩ active| / |candidate|   (double; a repeated candidate counts once)
 *   overlap <  gamma: active <- candidate;  B_offload = (active_prev \ active) \ B_Memory is copied from its
 *                     GPU slots to the CPU pool and joins B_Memory;  B_load = active \ active_prev is copied
 *                     from the CPU pool into the slots that became free
 *   overlap >= gamma: nothing changes.
 * A block is "active" iff slot_of_block[b] >= 0.  The call enqueues two kernels on `stream` (pass the
 * stream the transfer should overlap compute from; the paper uses a second stream for it).
 *   candidate      [n_candidates] int32, device (for instance the output of slim_select_topk_blocks)
 *   slot_of_block  [n_blocks] int32, device, in/out: GPU slot of an active block, -1 otherwise
 *   block_of_slot  [n_slots]  int32, device, in/out: inverse map, -1 = free slot
 *   in_memory      [n_blocks] int32, device, in/out: 1 when the CPU pool holds the block (B_Memory); only
 *                  ever set, never cleared (the prompt's KV does not change once written)
 *   gpu_pool       [n_slots, block_bytes]  device
 *   host_pool      [n_blocks, block_bytes] HOST memory that is pinned and device-mapped (hipHostMalloc),
 *                  passed by its device-visible address; block b lives at offset b*block_bytes
 *   block_bytes    payload of one block (its K and V rows, of one layer or of every layer that shares the
 *                  block set); multiple of 16; both pools 16-byte aligned
 *   info           [8] int32, device, out: {|candidate|, |candidate ∩ active|, swapped (0/1), blocks copied
 *                  out, blocks copied in, error bits, slots released, 0}.  Error bits: 1 = a candidate outside
 *                  [0, n_blocks); 2 = a block to load is not in the CPU pool; 4 = more candidates than slots;
 *                  8 = the two maps are not inverse to each other.  With a non-zero error nothing is moved
 *                  and the maps are left as they were.
 *   workspace      >= slim_kv_swap_workspace_bytes(n_blocks, n_slots) bytes, device, 256-byte aligned
 * Which free slot an arriving block takes is the library's choice (ascending blocks into ascending
 * freed slots); callers read it from slot_of_block.  The host sees offloaded bytes after it has synchronised
 * with `stream`.  Errors (host side, nothing enqueued): INVALID_ARG (null, sizes < 1, gamma not in [0, 1]
 * or NaN), UNSUPPORTED (alignment, block_bytes % 16), WORKSPACE_TOO_SMALL.
 */
size_t slim_kv_swap_workspace_bytes(int n_blocks, int n_slots);
int slim_kv_swap(const int* candidate, int n_candidates, int n_blocks, double gamma, int* slot_of_block,
                 int* block_of_slot, int* in_memory, int n_slots, void* gpu_pool, void* host_pool,
                 size_t block_bytes, int* info, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Decode-step attention over the active blocks -- Section 4.1: only active blocks take part in attention and
 * have their KV in GPU memory; every response token is retained.  One new token:
 *   out[h, :] = sum_j softmax_j(scale * q[h, :] . k_j^{g}) v_j^{g},   g = h / (Hq/Hkv),
 * j over the prompt tokens of every block that sits in the slot pool (block_of_slot[s] >= 0; the last prompt
 * block may be short) and over the n_response response tokens.  The pool is read where the KV swap has put the
 * blocks, through block_of_slot; no gather, no host round trip.
 *   q, out         [Hq, 128] dtype
 *   gpu_pool       slot s at byte s*slot_bytes; inside it, at layer_offset, K[block, Hkv, 128] then
 *                  V[block, Hkv, 128] of the slot's block (dtype)
 *   block_of_slot  [n_slots] int32 device (as kept by slim_kv_swap)
 *   k_response, v_response  [n_response, Hkv, 128] dtype (NULL when n_response = 0)
 *   workspace      >= slim_decode_attn_workspace_bytes(...), 256-byte aligned: per-slot partial results
 * softmax_scale 0 => 1/sqrt(128).  At least one key must exist (an empty pool without response tokens gives NaN).
 * Errors: INVALID_ARG (nulls, sizes, Hq % Hkv, slot too small for the payload), UNSUPPORTED (head_dim != 128,
 * more than 8 query heads per kv head, alignment), WORKSPACE_TOO_SMALL.
 */
size_t slim_decode_attn_workspace_bytes(int n_slots, int n_response, int n_q_heads);
int slim_decode_attn(const void* q, const void* gpu_pool, size_t slot_bytes, size_t layer_offset,
                     const int* block_of_slot, int n_slots, int block, int n_prompt_tokens, const void* k_response,
                     const void* v_response, int n_response, int n_q_heads, int n_kv_heads, int head_dim,
                     float softmax_scale, int dtype, void* out, void* workspace, size_t workspace_bytes,
                     void* stream);

/* ------------------------------------------------------------------------------------------------
 * One layer for one newly decoded token -- the decoding phase of Fig. 2 with the KV cache of Section 4.3: "QKV
 * Generation" for the token, attention of its Query over the active blocks in the slot pool, the earlier response
 * tokens and itself, output projection, FFN.
 *   slim_gemv: the single-token projection, out[n] = s * (w[n, :] . x) + bias[n] + residual[n] (NULL = absent), or
 *              with w_up: silu(s * w . x) * (s * w_up . x);  s = *scale (device float, e.g. the token's 1/rms from
 *              slim_row_rstd for a folded gain) or 1 when scale is NULL.  Every weight is read once.  out may alias
 *              residual.  k_in % 8 == 0 (bf16) / % 4 (fp32), k_in <= 16376 (the token is staged in 64 KiB of LDS as floats,
 *              beside 16 bytes of partial sums; UNSUPPORTED beyond), 16-byte aligned w, w_up, x.
 *   slim_decode_layer:
 *     x_new [hidden], position = the token's position (for RoPE), x_out [hidden] (may not alias x_new)
 *     gpu_pool / slot_bytes / layer_offset / block_of_slot / n_slots / n_prompt_tokens: as slim_decode_attn
 *     k_response, v_response [>= n_response + 1, Hkv, 128]: rows 0..n_response-1 are the earlier response tokens;
 *                    the call WRITES the token's own Key (post-RoPE) and Value states into row n_response
 *     q_out [Hq, 128] or NULL: the token's Query states (post-RoPE), e.g. for the scoring window of the next steps
 *     workspace >= slim_decode_layer_workspace_bytes(...), 256-byte aligned
 *   Weights as slim_pruned_layer (NULL gains = folded).  head_dim 128, at most 8 query heads per kv head, hidden,
 *   ffn, Hq*128 <= 16376.  6 launches with folded gains (8 otherwise), no host synchronisation.  Errors as the stage
 *   calls.
 */
int slim_gemv(const void* w, const void* w_up, const void* x, const float* scale, const void* bias,
              const void* residual, int n_out, int k_in, int dtype, void* out, void* stream);
size_t slim_decode_layer_workspace_bytes(const slim_layer_shape* s, int n_slots, int n_response);
int slim_decode_layer(const slim_layer_shape* s, const slim_layer_weights* w, const void* x_new, int position,
                      const void* gpu_pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot,
                      int n_slots, int n_prompt_tokens, void* k_response, void* v_response, int n_response,
                      void* x_out, void* q_out, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIM_H */
