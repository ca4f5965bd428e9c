// C entry points of libslim: argument checks, workspace carving and the order of kernel launches of
// the pruned prefill layer.  No kernel lives here.
#include "slim_common.h"
#include <math.h>
#include <algorithm>
#include <mutex>
#include <string.h>

namespace slim {

// Scratch of the entry point that allocates nothing (slim_score_blocks_static): the head-group-summed window
// query that travels from the reduction kernel to the scoring kernel.  Each GPU holds its own copy of the array
// at its own address; host code uses the address hipGetSymbolAddress reports for the current device, never the
// array's name.
constexpr int kScratchFloats = 8192;                 // the largest Hkv * head_dim the scoring kernels take
constexpr int kScratchDevices = 64;
static __device__ __align__(256) float scratch[kScratchFloats];
static std::mutex g_scratch_mutex;
static float* g_scratch_ptr[kScratchDevices];        // per device, filled on the first call there

static int scratch_of_current_device(float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_hip_error(e);
    if (dev < 0 || dev >= kScratchDevices) return SLIM_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return set_hip_error(e);
        if (!p) return SLIM_HIP_ERROR;
        g_scratch_ptr[dev] = (float*)p;
    }
    *out = g_scratch_ptr[dev];
    return SLIM_OK;
}

static thread_local char g_hip_error[256] = "";

int set_hip_error(hipError_t e) {
    strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
    return SLIM_HIP_ERROR;
}

static bool dtype_ok(int dtype) { return dtype == SLIM_F32 || dtype == SLIM_BF16; }

static int forced_count(unsigned flags, int nb) {
    int c = ((flags & SLIM_FORCE_FIRST) ? 1 : 0) + ((flags & SLIM_FORCE_LAST) ? 1 : 0);
    return c > nb ? nb : c;
}

// Workspace layout of slim_pruned_layer (every region 256-byte aligned).
struct LayerPlan {
    size_t h, k_all, q_win, qt, scores, table, tscore, rstd, rstd2, kc, vc, qc, o, o_all, act, total;
    int nb, n_out;
    bool prune;
};

static LayerPlan plan_layer(const slim_layer_shape* s, int N, int n_keep) {
    LayerPlan p{};
    const size_t es = elem_size(s->dtype);
    p.nb = (N + s->block - 1) / s->block;
    p.prune = n_keep < p.nb;
    p.n_out = p.prune ? slim_kept_tokens(N, s->block, n_keep) : N;
    const size_t kv = (size_t)s->n_kv_heads * s->head_dim, qd = (size_t)s->n_q_heads * s->head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    p.h = take((size_t)N * s->hidden * es);              // RMSNorm output: all N rows, later n' rows
    p.k_all = take((size_t)N * kv * es);                 // Key states of all tokens
    // Query states of the window, or (window query taken straight from the hidden rows) its float partial sums
    p.q_win = take(std::max((size_t)s->window * qd * es,
                            slim_window_query_from_rows_workspace_bytes(std::min(s->window, kWindowRowsMax), s->n_q_heads)));
    p.qt = take(slim_score_blocks_workspace_bytes(s->n_kv_heads, s->head_dim));
    p.scores = take((size_t)p.nb * sizeof(float));
    p.table = take((size_t)N * s->head_dim * sizeof(float));            // cos | sin of every token's rotation angles
    p.tscore = take((size_t)N * s->n_kv_heads * sizeof(float));         // per-(token, kv head) score partials
    p.rstd = take((size_t)N * sizeof(float));                           // 1/rms of the incoming rows (folded gains)
    p.rstd2 = take((size_t)N * sizeof(float));                          // ... of the rows that continue
    const bool after = p.prune && s->placement == SLIM_PRUNE_AFTER_ATTENTION;
    const size_t n_att = after ? (size_t)N : (size_t)p.n_out;    // rows that go through attention
    p.kc = (p.prune && !after) ? take((size_t)p.n_out * kv * es) : p.k_all;   // compacted keys
    p.vc = take(n_att * kv * es);
    p.qc = take(n_att * qd * es);
    p.o_all = after ? take(n_att * qd * es) : 0;         // attention output of all N rows, compacted into o
    p.o = take((size_t)p.n_out * qd * es);
    p.act = take((size_t)p.n_out * s->ffn * es);
    p.total = off;
    return p;
}

static int check_shape(const slim_layer_shape* s) {
    if (!s) return SLIM_INVALID_ARG;
    if (s->hidden < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->head_dim < 1 || s->ffn < 1 || s->block < 1 ||
        s->unit < 1 || s->window < 1 || s->unit > s->block || s->n_q_heads % s->n_kv_heads != 0 ||
        !(s->rope_theta > 0.f) || !(s->rms_eps >= 0.f) || s->scoring < 0 || s->scoring > SLIM_POOL_MAX ||
        s->placement < 0 || s->placement > SLIM_PRUNE_AFTER_ATTENTION)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(s->dtype)) return SLIM_UNSUPPORTED;
    if (s->dtype == SLIM_BF16 && (s->head_dim != 128 || s->hidden % 8 != 0 || s->ffn % 8 != 0)) return SLIM_UNSUPPORTED;
    if (s->dtype == SLIM_F32 && (s->head_dim != 32 && s->head_dim != 64 && s->head_dim != 128)) return SLIM_UNSUPPORTED;
    return SLIM_OK;
}

}  // namespace slim

using namespace slim;

extern "C" {

const char* slim_status_string(int code) {
    switch (code) {
        case SLIM_OK: return "ok";
        case SLIM_INVALID_ARG: return "invalid argument";
        case SLIM_UNSUPPORTED: return "unsupported shape or dtype";
        case SLIM_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SLIM_HIP_ERROR: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* slim_last_hip_error(void) { return g_hip_error; }

size_t slim_score_blocks_workspace_bytes(int n_kv_heads, int head_dim) {
    if (n_kv_heads < 1 || head_dim < 1) return 0;
    return align_up((size_t)n_kv_heads * head_dim * sizeof(float), 256);
}

int slim_score_blocks(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads, int n_kv_heads,
                      int head_dim, int block, int unit, int dtype, float* scores, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (!q_win || !k || !scores || !workspace || n_tokens < 1 || window < 1 || n_q_heads < 1 || n_kv_heads < 1 ||
        head_dim < 1 || block < 1 || unit < 1 || unit > block || n_q_heads % n_kv_heads != 0)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const int E = n_kv_heads * head_dim;
    if (E % (dtype == SLIM_BF16 ? 8 : 4) != 0 || E > 8192 || !aligned16(k)) return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_score_blocks_workspace_bytes(n_kv_heads, head_dim)) return SLIM_WORKSPACE_TOO_SMALL;
    return launch_score(q_win, k, n_tokens, window, n_q_heads, n_kv_heads, head_dim, block, unit, 0, dtype, scores,
                        (float*)workspace, (hipStream_t)stream);
}

int slim_score_blocks_static(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads, int n_kv_heads,
                             int head_dim, int block, int unit, int dtype, float* scores, void* stream) {
    if (!q_win || !k || !scores || n_tokens < 1 || window < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 ||
        block < 1 || unit < 1 || unit > block || n_q_heads % n_kv_heads != 0)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const long long E = (long long)n_kv_heads * head_dim;
    if (E > kScratchFloats || E % (dtype == SLIM_BF16 ? 8 : 4) != 0 || !aligned16(k)) return SLIM_UNSUPPORTED;
    float* qt = nullptr;
    const int rc = scratch_of_current_device(&qt);
    if (rc != SLIM_OK) return rc;
    // Both kernels write every element of the scratch they read (qt[0 .. E)), so nothing needs clearing.
    return launch_score(q_win, k, n_tokens, window, n_q_heads, n_kv_heads, head_dim, block, unit, 0, dtype, scores, qt,
                        (hipStream_t)stream);
}

int slim_score_blocks_pooled(const void* q_win, const void* k, int n_tokens, int window, int n_q_heads,
                             int n_kv_heads, int head_dim, int block, int pooling, int dtype, float* scores,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!q_win || !k || !scores || !workspace || n_tokens < 1 || window < 1 || n_q_heads < 1 || n_kv_heads < 1 ||
        head_dim < 1 || block < 1 || n_q_heads % n_kv_heads != 0 || (pooling != SLIM_POOL_AVG && pooling != SLIM_POOL_MAX))
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const int E = n_kv_heads * head_dim;
    if (E % (dtype == SLIM_BF16 ? 8 : 4) != 0 || E > 8192 || !aligned16(k)) return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_score_blocks_workspace_bytes(n_kv_heads, head_dim)) return SLIM_WORKSPACE_TOO_SMALL;
    return launch_score(q_win, k, n_tokens, window, n_q_heads, n_kv_heads, head_dim, block, block, pooling, dtype,
                        scores, (float*)workspace, (hipStream_t)stream);
}

int slim_unit_keys(const void* k, int n_tokens, int n_kv_heads, int head_dim, int block, int unit, int dtype,
                   float* k_rep, void* stream) {
    if (!k || !k_rep || n_tokens < 1 || n_kv_heads < 1 || head_dim < 1 || block < 1 || unit < 1 || unit > block)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const int E = n_kv_heads * head_dim;
    if (E % (dtype == SLIM_BF16 ? 8 : 4) != 0 || E > 8192 || !aligned16(k) || !aligned16(k_rep)) return SLIM_UNSUPPORTED;
    return launch_unit_keys(k, n_tokens, E, block, unit, dtype, k_rep, (hipStream_t)stream);
}

int slim_score_blocks_from_unit_keys(const void* q_win, const float* k_rep, int n_tokens, int window, int n_q_heads,
                                     int n_kv_heads, int head_dim, int block, int unit, int dtype, float* scores,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    if (!q_win || !k_rep || !scores || !workspace || n_tokens < 1 || window < 1 || n_q_heads < 1 || n_kv_heads < 1 ||
        head_dim < 1 || block < 1 || unit < 1 || unit > block || n_q_heads % n_kv_heads != 0)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const int E = n_kv_heads * head_dim;
    if (E % (dtype == SLIM_BF16 ? 8 : 4) != 0 || E > 8192 || !aligned16(k_rep)) return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_score_blocks_workspace_bytes(n_kv_heads, head_dim)) return SLIM_WORKSPACE_TOO_SMALL;
    return launch_score_from_unit_keys(q_win, k_rep, n_tokens, window, n_q_heads, n_kv_heads, head_dim, block, unit,
                                       dtype, scores, (float*)workspace, (hipStream_t)stream);
}

size_t slim_decode_attn_workspace_bytes(int n_slots, int n_response, int n_q_heads) {
    if (n_slots < 0 || n_response < 0 || n_q_heads < 1 || n_slots + n_response < 1) return 0;
    return align_up(((size_t)n_slots + (size_t)(n_response + 63) / 64) * n_q_heads * 130 * sizeof(float), 256);
}

int slim_decode_attn(const void* q, const void* gpu_pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot,
                     int n_slots, int block, int n_prompt_tokens, const void* k_response, const void* v_response,
                     int n_response, int n_q_heads, int n_kv_heads, int head_dim, float softmax_scale, int dtype, void* out,
                     void* workspace, size_t workspace_bytes, void* stream) {
    if (!q || !out || !workspace || n_slots < 0 || n_response < 0 || n_slots + n_response < 1 || n_q_heads < 1 ||
        n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 || head_dim < 1 || (n_slots > 0 && (!gpu_pool || !block_of_slot ||
        block < 1 || n_prompt_tokens < 1)) || (n_response > 0 && (!k_response || !v_response)))
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const size_t kv_bytes = (size_t)n_kv_heads * head_dim * elem_size(dtype);
    if (n_slots > 0 && layer_offset + 2 * (size_t)block * kv_bytes > slot_bytes) return SLIM_INVALID_ARG;
    if (head_dim != 128 || n_q_heads / n_kv_heads > 8 || slot_bytes % 16 != 0 || layer_offset % 16 != 0 || !aligned16(q) ||
        (n_slots > 0 && !aligned16(gpu_pool)) || (n_response > 0 && (!aligned16(k_response) || !aligned16(v_response))) ||
        n_slots + (n_response + 63) / 64 > 65535 * 32)
        return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_decode_attn_workspace_bytes(n_slots, n_response, n_q_heads)) return SLIM_WORKSPACE_TOO_SMALL;
    if (softmax_scale == 0.f) softmax_scale = 1.0f / sqrtf((float)head_dim);
    return launch_decode_attn(q, gpu_pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt_tokens,
                              k_response, v_response, n_response, n_q_heads, n_kv_heads, softmax_scale, dtype, out,
                              (float*)workspace, (hipStream_t)stream);
}

int slim_gemv(const void* w, const void* w_up, const void* x, const float* scale, const void* bias, const void* residual,
              int n_out, int k_in, int dtype, void* out, void* stream) {
    if (!w || !x || !out || n_out < 1 || k_in < 1) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    if (k_in % (dtype == SLIM_BF16 ? 8 : 4) != 0 || k_in > 16376 || !aligned16(w) || !aligned16(x) || (w_up && !aligned16(w_up)))
        return SLIM_UNSUPPORTED;
    return launch_gemv(w, w_up, x, scale, -1.f, bias, residual, n_out, k_in, dtype, out, (hipStream_t)stream);
}

// Workspace of slim_decode_layer: h | rstd | q | o | act | attention partials
struct DecodePlan { size_t h, rstd, q, o, act, attn, total; };
static DecodePlan plan_decode(const slim_layer_shape* s, int n_slots, int n_response) {
    DecodePlan p{};
    const size_t es = elem_size(s->dtype), qd = (size_t)s->n_q_heads * s->head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    p.h = take((size_t)s->hidden * es);
    p.rstd = take(2 * sizeof(float));
    p.q = take(qd * es);
    p.o = take(qd * es);
    p.act = take((size_t)s->ffn * es);
    p.attn = take(slim_decode_attn_workspace_bytes(n_slots, n_response + 1, s->n_q_heads));
    p.total = off;
    return p;
}

size_t slim_decode_layer_workspace_bytes(const slim_layer_shape* s, int n_slots, int n_response) {
    if (check_shape(s) != SLIM_OK || n_slots < 0 || n_response < 0) return 0;
    return plan_decode(s, n_slots, n_response).total;
}

int slim_decode_layer(const slim_layer_shape* s, const slim_layer_weights* w, const void* x_new, int position,
                      const void* gpu_pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot, int n_slots,
                      int n_prompt_tokens, void* k_response, void* v_response, int n_response, void* x_out, void* q_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(s);
    if (rc) return rc;
    if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down || !x_new || !x_out ||
        !k_response || !v_response || !workspace || position < 0 || n_slots < 0 || n_response < 0 ||
        (n_slots > 0 && (!gpu_pool || !block_of_slot || n_prompt_tokens < 1)))
        return SLIM_INVALID_ARG;
    const int dt = s->dtype, Hd = s->hidden, Hq = s->n_q_heads, Hkv = s->n_kv_heads, d = s->head_dim;
    const int qd = Hq * d, kvd = Hkv * d, vec = dt == SLIM_BF16 ? 8 : 4;
    const size_t es = elem_size(dt);
    if (d != 128 || Hq / Hkv > 8 || Hd % vec != 0 || s->ffn % vec != 0 || Hd > 16376 || s->ffn > 16376 || qd > 16376 ||
        !aligned16(x_new) || !aligned16(x_out) || !aligned16(k_response) || !aligned16(v_response) ||
        ((uintptr_t)workspace & 255u) || slot_bytes % 16 != 0 || layer_offset % 16 != 0 || (n_slots > 0 && !aligned16(gpu_pool)) ||
        (q_out && !aligned16(q_out)))
        return SLIM_UNSUPPORTED;
    if (n_slots > 0 && layer_offset + 2 * (size_t)s->block * kvd * es > slot_bytes) return SLIM_INVALID_ARG;
    const DecodePlan p = plan_decode(s, n_slots, n_response);
    if (workspace_bytes < p.total) return SLIM_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    unsigned char* ws = (unsigned char*)workspace;
    void *h = ws + p.h, *q = q_out ? q_out : (void*)(ws + p.q), *o = ws + p.o, *act = ws + p.act;
    void* k_new = (unsigned char*)k_response + (size_t)n_response * kvd * es;
    void* v_new = (unsigned char*)v_response + (size_t)n_response * kvd * es;
#define SLIM_TRY(call) do { rc = (call); if (rc) return rc; } while (0)
    // QKV generation for the token in one launch: the norm (with a folded gain: a statistic that the kernel forms from
    // its own copy of the token; else a normalised copy first), the three projections with their biases, RoPE at the
    // token's position.  Its Key/Value states become row n_response of the response buffers.
    const void* a = x_new;
    float eps = s->rms_eps;
    if (w->g_attn) { SLIM_TRY(launch_rmsnorm(x_new, w->g_attn, 1, Hd, s->rms_eps, dt, h, st)); a = h; eps = -1.f; }
    SLIM_TRY(launch_gemv_qkv(w->wq, w->wk, w->wv, w->bq, w->bk, w->bv, a, eps, qd, kvd, Hd, position, s->rope_theta, dt, q,
                             k_new, v_new, st));
    // attention over the active blocks, the earlier response tokens and the token itself
    SLIM_TRY(launch_decode_attn(q, gpu_pool, slot_bytes, layer_offset, block_of_slot, n_slots, s->block, n_prompt_tokens,
                                k_response, v_response, n_response + 1, Hq, Hkv, 1.0f / sqrtf((float)d), dt, o,
                                (float*)(ws + p.attn), st));
    // output projection + residual, FFN + residual
    SLIM_TRY(launch_gemv(w->wo, nullptr, o, nullptr, -1.f, nullptr, x_new, Hd, qd, dt, x_out, st));
    a = x_out;
    eps = s->rms_eps;
    if (w->g_ffn) { SLIM_TRY(launch_rmsnorm(x_out, w->g_ffn, 1, Hd, s->rms_eps, dt, h, st)); a = h; eps = -1.f; }
    SLIM_TRY(launch_gemv(w->w_gate, w->w_up, a, nullptr, eps, nullptr, nullptr, s->ffn, Hd, dt, act, st));
    SLIM_TRY(launch_gemv(w->w_down, nullptr, act, nullptr, -1.f, nullptr, x_out, Hd, s->ffn, dt, x_out, st));
#undef SLIM_TRY
    return SLIM_OK;
}

int slim_rope_table(const int* pos, int n, int head_dim, float theta, float* table, void* stream) {
    if (!table || n < 1 || head_dim < 2 || head_dim % 2 != 0 || head_dim > 256 || !(theta > 0.f)) return SLIM_INVALID_ARG;
    return launch_rope_table(pos, 0, n, head_dim, theta, table, (hipStream_t)stream);
}

int slim_window_query(const void* q_win, int window, int n_q_heads, int n_kv_heads, int head_dim, int dtype, float* qt,
                      void* stream) {
    if (!q_win || !qt || window < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 || n_q_heads % n_kv_heads != 0)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    return launch_window_query(q_win, window, n_q_heads, n_kv_heads, head_dim, dtype, qt, (hipStream_t)stream);
}

size_t slim_window_query_from_rows_workspace_bytes(int window, int n_q_heads) {
    if (window < 1 || n_q_heads < 1) return 0;
    return align_up((size_t)kWindowSplitsMax * window * n_q_heads * 128 * sizeof(float), 256);
}

int slim_window_query_from_rows(const void* rows, int lda, const void* wq, const void* bias, const float* rstd,
                                const float* table, int window, int n_q_heads, int n_kv_heads, int k_in, float* qt,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (!rows || !wq || !table || !qt || !workspace || window < 1 || n_q_heads < 1 || n_kv_heads < 1 || k_in < 1 ||
        lda < k_in || n_q_heads % n_kv_heads != 0)
        return SLIM_INVALID_ARG;
    if (window > kWindowRowsMax || k_in % 64 != 0 || lda % 8 != 0 || !aligned16(rows) || !aligned16(wq) ||
        !aligned16(workspace))
        return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_window_query_from_rows_workspace_bytes(window, n_q_heads)) return SLIM_WORKSPACE_TOO_SMALL;
    return launch_window_query_rows(rows, lda, wq, bias, rstd, table, window, n_q_heads, n_kv_heads, k_in,
                                    (float*)workspace, qt, (hipStream_t)stream);
}

int slim_linear_rope(const void* a, int lda, const void* w, const void* bias, const float* table, int m, int n_heads,
                     int head_dim, int k_in, int ldo, int dtype, const float* rstd, void* out, const float* qt,
                     float* token_scores, void* stream) {
    if (!a || !w || !table || !out || m < 1 || n_heads < 1 || head_dim < 1 || k_in < 1 || lda < k_in ||
        ldo < n_heads * head_dim || (qt && !token_scores))
        return SLIM_INVALID_ARG;
    if (dtype != SLIM_BF16 || head_dim != 128 || k_in % 64 != 0 || lda % 8 != 0 || ldo % 8 != 0 || !aligned16(a) ||
        !aligned16(w) || !aligned16(table) || !aligned16(out) || (bias && !aligned16(bias)) || (qt && !aligned16(qt)))
        return SLIM_UNSUPPORTED;
    return launch_linear_rope(a, lda, w, bias, table, qt, qt ? token_scores : nullptr, rstd, m, n_heads, k_in, ldo, out,
                              (hipStream_t)stream);
}

int slim_linear_pair(const void* a, int lda, const void* w_1, const void* bias_1, int n_1, int ldo_1, void* out_1,
                     const void* w_2, const void* bias_2, int n_2, int ldo_2, void* out_2, const float* rstd, int m,
                     int k_in, int dtype, void* stream) {
    if (!a || !w_1 || !w_2 || !out_1 || !out_2 || m < 1 || n_1 < 1 || n_2 < 1 || k_in < 1 || lda < k_in || ldo_1 < n_1 ||
        ldo_2 < n_2 || !bias_1 != !bias_2)
        return SLIM_INVALID_ARG;
    if (dtype != SLIM_BF16 || k_in % 64 != 0 || lda % 8 != 0 || m <= 128 || !aligned16(a) || !aligned16(w_1) ||
        !aligned16(w_2) || (bias_1 && (!aligned16(bias_1) || !aligned16(bias_2))))
        return SLIM_UNSUPPORTED;
    return launch_linear_pair(a, lda, w_1, bias_1, n_1, ldo_1, out_1, w_2, bias_2, n_2, ldo_2, out_2, rstd, m, k_in,
                              (hipStream_t)stream);
}

int slim_row_rstd(const void* x, int n, int hidden, float eps, int dtype, float* rstd, void* stream) {
    if (!x || !rstd || n < 1 || hidden < 1 || !(eps >= 0.f)) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    return launch_row_rstd(x, n, hidden, eps, dtype, rstd, (hipStream_t)stream);
}

static int check_norm_linear(const void* a, int lda, const void* w, const void* bias, const float* rstd, int m, int n_out,
                             int k_in, int ldo, int dtype, const void* out) {
    if (!a || !w || !rstd || !out || m < 1 || n_out < 1 || k_in < 1 || lda < k_in || ldo < n_out) return SLIM_INVALID_ARG;
    if (dtype != SLIM_BF16 || k_in % 64 != 0 || lda % 8 != 0 || !aligned16(a) || !aligned16(w) || (bias && !aligned16(bias)))
        return SLIM_UNSUPPORTED;
    return SLIM_OK;
}

int slim_rmsnorm_linear(const void* a, int lda, const void* w, const void* bias, const float* rstd, int m, int n_out,
                        int k_in, int ldo, int dtype, void* out, void* stream) {
    int rc = check_norm_linear(a, lda, w, bias, rstd, m, n_out, k_in, ldo, dtype, out);
    if (rc) return rc;
    return launch_linear_scaled(a, lda, w, nullptr, bias, rstd, m, n_out, k_in, ldo, out, (hipStream_t)stream);
}

int slim_rmsnorm_swiglu_linear(const void* a, int lda, const void* w_gate, const void* w_up, const float* rstd, int m,
                               int n_out, int k_in, int ldo, int dtype, void* out, void* stream) {
    if (!w_up) return SLIM_INVALID_ARG;
    int rc = check_norm_linear(a, lda, w_gate, nullptr, rstd, m, n_out, k_in, ldo, dtype, out);
    if (rc) return rc;
    if (!aligned16(w_up)) return SLIM_UNSUPPORTED;
    return launch_linear_scaled(a, lda, w_gate, w_up, nullptr, rstd, m, n_out, k_in, ldo, out, (hipStream_t)stream);
}

int slim_fold_gain(const void* w, const void* gain, int n_out, int k_in, int dtype, void* out, void* stream) {
    if (!w || !gain || !out || n_out < 1 || k_in < 1) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    return launch_fold_gain(w, gain, n_out, k_in, dtype, out, (hipStream_t)stream);
}

int slim_score_blocks_from_token_scores(const float* token_scores, int n_tokens, int n_kv_heads, int block, int unit,
                                        float* scores, void* stream) {
    if (!token_scores || !scores || n_tokens < 1 || n_kv_heads < 1 || block < 1 || unit < 1 || unit > block)
        return SLIM_INVALID_ARG;
    return launch_token_score_blocks(token_scores, n_tokens, n_kv_heads, block, unit, scores, (hipStream_t)stream);
}

size_t slim_kv_swap_workspace_bytes(int n_blocks, int n_slots) {
    if (n_blocks < 1 || n_slots < 1) return 0;
    return align_up(((size_t)n_blocks + 4 * (size_t)n_slots + 1) * sizeof(int), 256);
}

int slim_kv_swap(const int* candidate, int n_candidates, int n_blocks, double gamma, int* slot_of_block,
                 int* block_of_slot, int* in_memory, int n_slots, void* gpu_pool, void* host_pool, size_t block_bytes,
                 int* info, void* workspace, size_t workspace_bytes, void* stream) {
    if (!candidate || !slot_of_block || !block_of_slot || !in_memory || !gpu_pool || !host_pool || !info || !workspace ||
        n_candidates < 1 || n_blocks < 1 || n_slots < 1 || block_bytes < 1 || !(gamma >= 0.0 && gamma <= 1.0))
        return SLIM_INVALID_ARG;
    if (block_bytes % 16 != 0 || !aligned16(gpu_pool) || !aligned16(host_pool)) return SLIM_UNSUPPORTED;
    if (workspace_bytes < slim_kv_swap_workspace_bytes(n_blocks, n_slots)) return SLIM_WORKSPACE_TOO_SMALL;
    return launch_kv_swap(candidate, n_candidates, n_blocks, gamma, slot_of_block, block_of_slot, in_memory, n_slots,
                          gpu_pool, host_pool, block_bytes, info, (int*)workspace, (hipStream_t)stream);
}

int slim_select_topk_blocks(const float* scores, int n_blocks, int n_keep, unsigned force_flags, int* kept_blocks,
                            void* stream) {
    if (!scores || !kept_blocks || n_blocks < 1 || n_keep < 1) return SLIM_INVALID_ARG;
    if (n_keep < n_blocks && n_keep < forced_count(force_flags, n_blocks)) return SLIM_INVALID_ARG;
    return launch_select(scores, n_blocks, n_keep, force_flags, kept_blocks, (hipStream_t)stream);
}

int slim_compact_tokens(const void* src, const int* pos_in, const int* kept_blocks, int n_keep, int block,
                        int n_tokens, int row_elems, int dtype, void* dst, int* pos_out, void* stream) {
    if (!src || !dst || !kept_blocks || n_keep < 1 || block < 1 || n_tokens < 1 || row_elems < 1) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    const int nb = (n_tokens + block - 1) / block;
    if (n_keep > nb || n_keep > 65535) return n_keep > nb ? SLIM_INVALID_ARG : SLIM_UNSUPPORTED;
    return launch_compact(src, pos_in, kept_blocks, n_keep, block, n_tokens, row_elems, dtype, dst, pos_out,
                          (hipStream_t)stream);
}

int slim_prefill_attn(const void* q, const void* k, const void* v, int n, int n_q_heads, int n_kv_heads,
                      int head_dim, float softmax_scale, int dtype, void* out, void* stream) {
    if (!q || !k || !v || !out || n < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1 ||
        n_q_heads % n_kv_heads != 0 || softmax_scale < 0.f)
        return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    if (dtype == SLIM_BF16 && (head_dim != 128 || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)))
        return SLIM_UNSUPPORTED;
    if (dtype == SLIM_F32 && head_dim != 32 && head_dim != 64 && head_dim != 128) return SLIM_UNSUPPORTED;
    if (dtype == SLIM_F32 && n_q_heads > 65535) return SLIM_UNSUPPORTED;
    return launch_attn(q, k, v, n, n_q_heads, n_kv_heads, head_dim, softmax_scale, dtype, out, (hipStream_t)stream);
}

int slim_rmsnorm(const void* x, const void* gain, int n, int hidden, float eps, int dtype, void* out, void* stream) {
    if (!x || !gain || !out || n < 1 || hidden < 1 || !(eps >= 0.f)) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    return launch_rmsnorm(x, gain, n, hidden, eps, dtype, out, (hipStream_t)stream);
}

int slim_rope(void* x, const int* pos, int n, int n_heads, int head_dim, float theta, int dtype, void* stream) {
    if (!x || n < 1 || n_heads < 1 || head_dim < 1 || !(theta > 0.f)) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype) || head_dim % 4 != 0 || head_dim > 256) return SLIM_UNSUPPORTED;
    return launch_rope(x, pos, 0, n, n_heads, head_dim, theta, dtype, (hipStream_t)stream);
}

static int linear_checks(const void* a, int lda, const void* w, int m, int n_out, int k_in, int ldo, int dtype,
                         const void* out) {
    if (!a || !w || !out || m < 1 || n_out < 1 || k_in < 1 || lda < k_in || ldo < n_out) return SLIM_INVALID_ARG;
    if (!dtype_ok(dtype)) return SLIM_UNSUPPORTED;
    if (dtype == SLIM_BF16 && (k_in % 8 != 0 || lda % 8 != 0 || !aligned16(a) || !aligned16(w))) return SLIM_UNSUPPORTED;
    return SLIM_OK;
}

int slim_linear(const void* a, int lda, const void* w, const void* residual, int m, int n_out, int k_in, int ldo,
                int dtype, void* out, void* stream) {
    int rc = linear_checks(a, lda, w, m, n_out, k_in, ldo, dtype, out);
    if (rc) return rc;
    return launch_linear(a, lda, w, nullptr, residual, nullptr, m, n_out, k_in, ldo, dtype, out, (hipStream_t)stream);
}

int slim_linear_bias(const void* a, int lda, const void* w, const void* bias, int m, int n_out, int k_in, int ldo,
                     int dtype, void* out, void* stream) {
    int rc = linear_checks(a, lda, w, m, n_out, k_in, ldo, dtype, out);
    if (rc) return rc;
    if (!bias) return SLIM_INVALID_ARG;
    if (!aligned16(bias)) return SLIM_UNSUPPORTED;
    return launch_linear(a, lda, w, nullptr, nullptr, bias, m, n_out, k_in, ldo, dtype, out, (hipStream_t)stream);
}

int slim_swiglu_linear(const void* a, int lda, const void* w_gate, const void* w_up, int m, int n_out, int k_in,
                       int ldo, int dtype, void* out, void* stream) {
    if (!w_up) return SLIM_INVALID_ARG;
    int rc = linear_checks(a, lda, w_gate, m, n_out, k_in, ldo, dtype, out);
    if (rc) return rc;
    if (dtype == SLIM_BF16 && !aligned16(w_up)) return SLIM_UNSUPPORTED;
    return launch_linear(a, lda, w_gate, w_up, nullptr, nullptr, m, n_out, k_in, ldo, dtype, out, (hipStream_t)stream);
}

int slim_kept_tokens(int n_tokens, int block, int n_keep) {
    if (n_tokens < 1 || block < 1 || n_keep < 1) return 0;
    const int nb = (n_tokens + block - 1) / block;
    if (n_keep >= nb) return n_tokens;
    return (n_keep - 1) * block + (n_tokens - (nb - 1) * block);
}

size_t slim_pruned_layer_workspace_bytes(const slim_layer_shape* s, int n_tokens, int n_keep) {
    if (check_shape(s) != SLIM_OK || n_tokens < 1 || n_keep < 1) return 0;
    return plan_layer(s, n_tokens, n_keep).total;
}

int slim_pruned_layer(const slim_layer_shape* s, const slim_layer_weights* w, const void* x_in, const int* pos_in,
                      int n_tokens, int n_keep, void* x_out, int* pos_out, int* kept_blocks_out, float* scores_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(s);
    if (rc) return rc;
    if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down || !x_in || !x_out ||
        !workspace || n_tokens < 1 || n_keep < 1)
        return SLIM_INVALID_ARG;
    // A NULL gain means the gain is already folded into the projections that follow the norm (slim_fold_gain);
    // the norm then runs inside those projections, which the kernels cover for bf16 and hidden % 64 == 0.
    if ((!w->g_attn || !w->g_ffn) && (s->dtype != SLIM_BF16 || s->hidden % 64 != 0)) return SLIM_UNSUPPORTED;
    const int N = n_tokens;
    const LayerPlan p = plan_layer(s, N, n_keep);
    if (p.prune) {
        if (!kept_blocks_out || !pos_out) return SLIM_INVALID_ARG;
        if (n_keep < forced_count(s->flags, p.nb)) return SLIM_INVALID_ARG;
        if (!(s->flags & SLIM_FORCE_LAST) && N % s->block != 0) return SLIM_INVALID_ARG;
        if (n_keep > 65535) return SLIM_UNSUPPORTED;
    }
    if (workspace_bytes < p.total) return SLIM_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255u) || !aligned16(x_in) || !aligned16(x_out)) return SLIM_UNSUPPORTED;
    if ((w->bq && !aligned16(w->bq)) || (w->bk && !aligned16(w->bk)) || (w->bv && !aligned16(w->bv))) return SLIM_UNSUPPORTED;

    hipStream_t st = (hipStream_t)stream;
    unsigned char* ws = (unsigned char*)workspace;
    const int dt = s->dtype, Hd = s->hidden, Hq = s->n_q_heads, Hkv = s->n_kv_heads, d = s->head_dim;
    const int qd = Hq * d, kvd = Hkv * d;
    const size_t es = elem_size(dt);
    void *h = ws + p.h, *k_all = ws + p.k_all, *q_win = ws + p.q_win, *kc = ws + p.kc, *vc = ws + p.vc,
         *qc = ws + p.qc, *o = ws + p.o, *act = ws + p.act;
    float* qt = (float*)(ws + p.qt);
#define SLIM_TRY(call) do { rc = (call); if (rc) return rc; } while (0)

    // Query/Key projection + RoPE at the given positions.  Keys of bf16 heads of 128: one kernel, the rotation (and, in
    // a pruning layer with TokenUnit scoring, the per-token dot with the window query) in the GEMM epilogue, so the
    // Key states are written once and not re-read for scoring.  Queries: projection, then the RoPE kernel (measured:
    // the rotation in the epilogue gains nothing for the wider Query projection once its cos/sin table is paid for).
    // With a folded gain (NULL g_attn / g_ffn) the projections read the residual stream itself and normalise it on
    // the fly, and no normalised copy is written; otherwise `h` holds RMSNorm(rows) and the projections read that.
    float* table = (float*)(ws + p.table);
    float* tscore = (float*)(ws + p.tscore);
    const bool fused = dt == SLIM_BF16 && d == 128 && Hd % 64 == 0;
    const bool fused_score = fused && p.prune && s->scoring == 0;
    const bool fold_attn = !w->g_attn, fold_ffn = !w->g_ffn;
    float* rstd_in = (float*)(ws + p.rstd);      // 1/rms of the incoming rows, and of the rows that continue
    float* rstd_kept = (float*)(ws + p.rstd2);
    // `sc`: the 1/rms of the rows of `a` when they are raw residual rows (folded gain), null when they are normalised.
    auto project = [&](const void* a, const float* sc, const void* wmat, const void* bias, int m, int n_feat, void* out) -> int {
        if (sc) return launch_linear_scaled(a, Hd, wmat, nullptr, bias, sc, m, n_feat, Hd, n_feat, out, st);
        return launch_linear(a, Hd, wmat, nullptr, nullptr, bias, m, n_feat, Hd, n_feat, dt, out, st);
    };
    auto project_rope = [&](const void* a, const float* sc, const void* wmat, const void* bias, const int* pos_, int pos0,
                            int m, int heads, void* out, const float* tab, const float* qt_, float* ts) -> int {
        if (tab) return launch_linear_rope(a, Hd, wmat, bias, tab, qt_, ts, sc, m, heads, Hd, heads * d, out, st);
        int r = project(a, sc, wmat, bias, m, heads * d, out);
        return r ? r : launch_rope(out, pos_, pos0, m, heads, d, s->rope_theta, dt, st);
    };
    // Query (+ RoPE) and Value states of m rows.  One launch for both projections where the kernel covers it.
    auto project_qv = [&](const void* a, const float* sc, const int* pos_, int m, void* q_out, void* v_out) -> int {
        int r;
        if (dt == SLIM_BF16 && Hd % 64 == 0 && m > 128 && !w->bq == !w->bv)
            r = launch_linear_pair(a, Hd, w->wq, w->bq, qd, qd, q_out, w->wv, w->bv, kvd, kvd, v_out, sc, m, Hd, st);
        else {
            r = project(a, sc, w->wq, w->bq, m, qd, q_out);
            if (!r) r = project(a, sc, w->wv, w->bv, m, kvd, v_out);
        }
        return r ? r : launch_rope(q_out, pos_, 0, m, Hq, d, s->rope_theta, dt, st);
    };
    auto block_scores = [&](const void* q_window, int w_eff, float* scores) -> int {
        if (fused_score) return launch_token_score_blocks(tscore, N, Hkv, s->block, s->unit, scores, st);
        return launch_score(q_window, k_all, N, w_eff, Hq, Hkv, d, s->block, s->unit, s->scoring, dt, scores, qt, st);
    };

    const void* rows_in = x_in;        // what the projections of the incoming tokens read
    const float* sc_in = nullptr;
    if (fold_attn) {
        // (the same pass over the rows leaves the cos / sin table of their positions for the Key projection)
        SLIM_TRY(launch_row_rstd(x_in, N, Hd, s->rms_eps, dt, rstd_in, st, pos_in, d, s->rope_theta, fused ? table : nullptr));
        sc_in = rstd_in;
    } else {
        SLIM_TRY(launch_rmsnorm(x_in, w->g_attn, N, Hd, s->rms_eps, dt, h, st));
        rows_in = h;
    }
    if (fused && !fold_attn) SLIM_TRY(launch_rope_table(pos_in, 0, N, d, s->rope_theta, table, st));
    const float* ktab = fused ? table : nullptr;   // cos/sin rows of the incoming tokens, for the Key projection

    const void* resid = x_in;          // residual stream entering the attention branch
    const int* pos = pos_in;           // positions of the rows that continue
    const int n = p.n_out;
    const int w_eff = s->window < N ? s->window : N;
    const bool after = p.prune && s->placement == SLIM_PRUNE_AFTER_ATTENTION;
    // The window query: with the scores riding on the Key projection it is all that is needed of the window's Query
    // states, and it is taken straight from the window's hidden rows (skinny split projection, rotation and means in
    // float); both placements use the same kernels, so they select from identical scores.
    const bool win_direct = fused_score && w_eff <= kWindowRowsMax;
    auto window_query_direct = [&]() -> int {
        const unsigned char* r_win = (const unsigned char*)rows_in + (size_t)(N - w_eff) * Hd * es;
        return launch_window_query_rows(r_win, Hd, w->wq, w->bq, sc_in ? sc_in + (N - w_eff) : nullptr,
                                        table + (size_t)(N - w_eff) * d, w_eff, Hq, Hkv, Hd, (float*)q_win, qt, st);
    };
    if (after) {
        // Attention first, over all N tokens; its last w_eff Query rows are the local window.
        void* o_all = ws + p.o_all;
        SLIM_TRY(project_qv(rows_in, sc_in, pos_in, N, qc, vc));
        const unsigned char* q_last = (const unsigned char*)qc + (size_t)(N - w_eff) * qd * es;
        if (win_direct) SLIM_TRY(window_query_direct());
        else if (fused_score) SLIM_TRY(launch_window_query(q_last, w_eff, Hq, Hkv, d, dt, qt, st));
        SLIM_TRY(project_rope(rows_in, sc_in, w->wk, w->bk, pos_in, 0, N, Hkv, k_all, ktab, fused_score ? qt : nullptr, tscore));
        SLIM_TRY(launch_attn(qc, k_all, vc, N, Hq, Hkv, d, 0.f, dt, o_all, st));
        float* scores = scores_out ? scores_out : (float*)(ws + p.scores);
        SLIM_TRY(block_scores(q_last, w_eff, scores));
        SLIM_TRY(launch_select(scores, p.nb, n_keep, s->flags, kept_blocks_out, st));
        // Residual rows + positions into x_out / pos_out, attention output rows into o.
        SLIM_TRY(launch_compact(x_in, pos_in, kept_blocks_out, n_keep, s->block, N, Hd, dt, x_out, pos_out, st));
        SLIM_TRY(launch_compact(o_all, nullptr, kept_blocks_out, n_keep, s->block, N, qd, dt, o, nullptr, st));
        resid = x_out;
    } else {
    if (p.prune && win_direct) {
        SLIM_TRY(window_query_direct());
    } else if (p.prune) {
        // Query states of the local window (last w_eff rows) and their head-group-summed mean.
        const unsigned char* r_win = (const unsigned char*)rows_in + (size_t)(N - w_eff) * Hd * es;
        SLIM_TRY(project_rope(r_win, sc_in ? sc_in + (N - w_eff) : nullptr, w->wq, w->bq,
                              pos_in ? pos_in + (N - w_eff) : nullptr, N - w_eff, w_eff, Hq, q_win, nullptr, nullptr, nullptr));
        if (fused_score) SLIM_TRY(launch_window_query(q_win, w_eff, Hq, Hkv, d, dt, qt, st));
    }
    // Key states of every incoming token.
    SLIM_TRY(project_rope(rows_in, sc_in, w->wk, w->bk, pos_in, 0, N, Hkv, k_all, ktab, fused_score ? qt : nullptr, tscore));
    const void* rows = rows_in;        // what the Q/V projections of the continuing tokens read
    const float* sc = sc_in;
    if (p.prune) {
        float* scores = scores_out ? scores_out : (float*)(ws + p.scores);
        SLIM_TRY(block_scores(q_win, w_eff, scores));
        SLIM_TRY(launch_select(scores, p.nb, n_keep, s->flags, kept_blocks_out, st));
        // Hidden rows + positions into x_out / pos_out, keys into kc, and with folded gains the rows' statistics
        // (those of the kept rows are the compacted ones): one launch.
        {
            const void* srcs[3] = {x_in, k_all, rstd_in};
            void* dsts[3] = {x_out, kc, rstd_kept};
            const size_t rb[3] = {(size_t)Hd * es, (size_t)kvd * es, sizeof(float)};
            if ((Hd * es) % 4 == 0 && (kvd * es) % 4 == 0)
                SLIM_TRY(launch_compact_multi(fold_attn ? 3 : 2, srcs, dsts, rb, pos_in, pos_out, kept_blocks_out, n_keep,
                                              s->block, N, st));
            else {
                SLIM_TRY(launch_compact(x_in, pos_in, kept_blocks_out, n_keep, s->block, N, Hd, dt, x_out, pos_out, st));
                SLIM_TRY(launch_compact(k_all, nullptr, kept_blocks_out, n_keep, s->block, N, kvd, dt, kc, nullptr, st));
                if (fold_attn)
                    SLIM_TRY(launch_compact(rstd_in, nullptr, kept_blocks_out, n_keep, s->block, N, 1, SLIM_F32, rstd_kept,
                                            nullptr, st));
            }
        }
        rows = x_out;
        if (fold_attn) {
            sc = rstd_kept;
        } else {
            SLIM_TRY(launch_rmsnorm(x_out, w->g_attn, n, Hd, s->rms_eps, dt, h, st));
            rows = h;
        }
        resid = x_out;
        pos = pos_out;
    } else {
        if (kept_blocks_out) SLIM_TRY(launch_select(nullptr, p.nb, p.nb, 0, kept_blocks_out, st));
        if (pos_out) SLIM_TRY(launch_positions(pos_in, pos_out, N, st));
    }

    // Q, V of the rows that continue; RoPE on Q at the original positions.
    SLIM_TRY(project_qv(rows, sc, pos, n, qc, vc));
    SLIM_TRY(launch_attn(qc, kc, vc, n, Hq, Hkv, d, 0.f, dt, o, st));
    }
    // y = resid + Wo o  (into x_out);  z = y + Wdown(silu(Wgate r) * Wup r), r = RMSNorm(y)  (in place)
    SLIM_TRY(launch_linear(o, qd, w->wo, nullptr, resid, nullptr, n, Hd, qd, Hd, dt, x_out, st));
    if (fold_ffn) {
        SLIM_TRY(launch_row_rstd(x_out, n, Hd, s->rms_eps, dt, rstd_kept, st));
        SLIM_TRY(launch_linear_scaled(x_out, Hd, w->w_gate, w->w_up, nullptr, rstd_kept, n, s->ffn, Hd, s->ffn, act, st));
    } else {
        SLIM_TRY(launch_rmsnorm(x_out, w->g_ffn, n, Hd, s->rms_eps, dt, h, st));
        SLIM_TRY(launch_linear(h, Hd, w->w_gate, w->w_up, nullptr, nullptr, n, s->ffn, Hd, s->ffn, dt, act, st));
    }
    SLIM_TRY(launch_linear(act, s->ffn, w->w_down, nullptr, x_out, nullptr, n, Hd, s->ffn, Hd, dt, x_out, st));
#undef SLIM_TRY
    return SLIM_OK;
}

// Walks the schedule on the host: tokens entering each layer, the largest layer workspace, and the
// number of kept-block indices the pruning layers emit.  Returns the final token count, 0 on bad input.
static int walk_schedule(const slim_layer_shape* s, int n_layers, const int* n_keep, int n_tokens,
                         size_t* max_layer_ws, size_t* kept_total) {
    if (check_shape(s) != SLIM_OK || n_layers < 1 || !n_keep || n_tokens < 1) return 0;
    int n = n_tokens;
    size_t ws = 0, kept = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int nb = (n + s->block - 1) / s->block;
        const bool prune = n_keep[l] > 0 && n_keep[l] < nb;
        const int keep = prune ? n_keep[l] : nb;
        if (prune && (keep < forced_count(s->flags, nb) || (!(s->flags & SLIM_FORCE_LAST) && n % s->block != 0)))
            return 0;
        const size_t need = plan_layer(s, n, keep).total;
        if (need > ws) ws = need;
        if (prune) { kept += (size_t)keep; n = slim_kept_tokens(n, s->block, keep); }
    }
    if (max_layer_ws) *max_layer_ws = ws;
    if (kept_total) *kept_total = kept;
    return n;
}

int slim_prefill_model_tokens(const slim_layer_shape* s, int n_layers, const int* n_keep, int n_tokens) {
    return walk_schedule(s, n_layers, n_keep, n_tokens, nullptr, nullptr);
}

// Workspace: [layer workspace | hidden A | hidden B | pos A | pos B | kept scratch]
size_t slim_prefill_model_workspace_bytes(const slim_layer_shape* s, int n_layers, const int* n_keep, int n_tokens) {
    size_t lw = 0;
    if (!walk_schedule(s, n_layers, n_keep, n_tokens, &lw, nullptr)) return 0;
    const size_t hid = align_up((size_t)n_tokens * s->hidden * elem_size(s->dtype), 256);
    const size_t ints = align_up((size_t)n_tokens * sizeof(int), 256);
    return align_up(lw, 256) + 2 * hid + 3 * ints;
}

int slim_prefill_model(const slim_layer_shape* s, const slim_layer_weights* layers, int n_layers, const int* n_keep,
                       const void* x_in, const int* pos_in, int n_tokens, void* x_out, int* pos_out,
                       int* kept_blocks_out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(s);
    if (rc) return rc;
    if (!layers || !n_keep || !x_in || !x_out || !workspace || n_layers < 1 || n_tokens < 1) return SLIM_INVALID_ARG;
    size_t lw = 0;
    if (!walk_schedule(s, n_layers, n_keep, n_tokens, &lw, nullptr)) return SLIM_INVALID_ARG;
    if (workspace_bytes < slim_prefill_model_workspace_bytes(s, n_layers, n_keep, n_tokens)) return SLIM_WORKSPACE_TOO_SMALL;
    if ((uintptr_t)workspace & 255u) return SLIM_UNSUPPORTED;
    lw = align_up(lw, 256);
    const size_t hid = align_up((size_t)n_tokens * s->hidden * elem_size(s->dtype), 256);
    const size_t ints = align_up((size_t)n_tokens * sizeof(int), 256);
    unsigned char* ws = (unsigned char*)workspace;
    void* hbuf[2] = {ws + lw, ws + lw + hid};
    int* pbuf[2] = {(int*)(ws + lw + 2 * hid), (int*)(ws + lw + 2 * hid + ints)};
    int* kept_scratch = (int*)(ws + lw + 2 * hid + 2 * ints);

    const void* x = x_in;
    const int* pos = pos_in;
    int n = n_tokens, hsel = 0, psel = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int nb = (n + s->block - 1) / s->block;
        const bool prune = n_keep[l] > 0 && n_keep[l] < nb;
        const int keep = prune ? n_keep[l] : nb;
        void* y = (l == n_layers - 1) ? x_out : hbuf[hsel];
        int* kept = kept_blocks_out ? kept_blocks_out : kept_scratch;
        rc = slim_pruned_layer(s, &layers[l], x, pos, n, keep, y, prune ? pbuf[psel] : nullptr, prune ? kept : nullptr,
                               nullptr, workspace, lw, stream);
        if (rc) return rc;
        if (prune) {
            if (kept_blocks_out) kept_blocks_out += keep;
            pos = pbuf[psel];
            psel ^= 1;
            n = slim_kept_tokens(n, s->block, keep);
        }
        x = y;
        hsel ^= 1;
    }
    if (pos_out) return launch_positions(pos, pos_out, n, (hipStream_t)stream);
    return SLIM_OK;
}

}  // extern "C"
