// Decode-step attention over the active blocks (Section 4.1: only active blocks take part in attention and have
// their KV in GPU memory; every response token is retained).  One new token's Query states attend to the prompt
// tokens of the blocks that currently sit in the GPU slot pool -- read through block_of_slot, wherever the KV swap
// (Algorithm 1) has put them -- and to all response tokens.  HBM-bound: every resident key and value is read once.
//
// Split over the keys: one workgroup per (slot or 64-token chunk of the response, kv head) leaves a partial
// (max, sum, weighted values) for the query heads of that kv head; a second kernel merges the partials.  Softmax
// is order-independent, so the slot order does not matter.
#include "slim_common.h"

namespace slim {

constexpr int DD = 128;          // head_dim
constexpr int DCH = 64;          // keys per chunk
constexpr int DGMAX = 8;         // query heads per kv head
constexpr int DPART = DD + 2;    // floats of a partial: values, max (base-2 domain), sum

// A wave owns 16 keys of a 64-key chunk and keeps its own running (max, sum, values): no workgroup barrier until
// the four waves' states are merged at the end.  Scores: 4 lanes per key, 32 dims each (16-byte loads), reduced
// with two shuffles.  Values: a lane owns dims 2 l, 2 l + 1 of all 16 keys (4-byte loads, a row is read by the
// whole wave), the probabilities go through a wave-private LDS strip.
template <typename T, int G>
__global__ void __launch_bounds__(256) decode_attn_partial_kernel(
    const T* __restrict__ q, const unsigned char* __restrict__ pool, size_t slot_bytes, size_t layer_offset,
    const int* __restrict__ block_of_slot, int n_slots, int block, int n_prompt, const T* __restrict__ k_resp,
    const T* __restrict__ v_resp, int n_resp, int Hq, int Hkv, float scale_log2e, float* __restrict__ part) {
    constexpr int V = Elem<T>::kVec;
    // Query heads of this kv head: floats times scale * log2(e) (fp32 path), or the bf16 pairs as they are, for
    // v_dot2_f32_bf16 (half the registers; the scale is then applied to the dot products).
    __shared__ float qs[G][sizeof(T) == 2 ? DD / 2 : DD];
    __shared__ float ps[4][16][G];                   // per wave: probabilities of its 16 keys
    __shared__ float ws_m[4][G], ws_l[4][G];     // per wave: running max and sum
    __shared__ float red[4][G][DD];                  // per wave: weighted values
    const int item = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;   // G = Hq / Hkv query heads per kv head
    const int wave = tid >> 6, lane = tid & 63;
    const size_t row_stride = (size_t)Hkv * DD;
    const int nb = (n_prompt + block - 1) / block;

    const T *kp, *vp;
    int rows;
    if (item < n_slots) {
        const int b = block_of_slot[item];
        rows = (b < 0 || b >= nb) ? 0 : min(block, n_prompt - b * block);
        kp = reinterpret_cast<const T*>(pool + (size_t)item * slot_bytes + layer_offset);
        vp = kp + (size_t)block * row_stride;
    } else {
        const int j = item - n_slots;
        rows = min(DCH, n_resp - j * DCH);
        kp = k_resp + (size_t)j * DCH * row_stride;
        vp = v_resp + (size_t)j * DCH * row_stride;
    }
    if constexpr (sizeof(T) == 2) {
        for (int i = tid; i < G * DD / 2; i += 256)
            qs[i / (DD / 2)][i % (DD / 2)] = __builtin_bit_cast(float, reinterpret_cast<const uint32_t*>(q + (size_t)g * G * DD)[i]);
    } else {
        for (int i = tid; i < G * DD; i += 256) qs[i / DD][i % DD] = Elem<T>::ld(q + (size_t)(g * G + i / DD) * DD + i % DD) * scale_log2e;
    }
    __syncthreads();

    float m_run[G], l_run[G], oacc[G][2];
#pragma unroll
    for (int h = 0; h < G; ++h) { m_run[h] = -INFINITY; l_run[h] = 0.f; oacc[h][0] = oacc[h][1] = 0.f; }
    const int kl = lane >> 2, prt = lane & 3;            // scores: key kl of the wave's 16, dims 32 prt ..
    for (int c0 = wave * 16; c0 < rows; c0 += DCH) {     // this wave's keys c0 .. c0 + 15 (wave-uniform bounds)
        const int cr = min(16, rows - c0);
        float dot[G];
#pragma unroll
        for (int h = 0; h < G; ++h) dot[h] = 0.f;
        // rows past the end are clamped to the last one (their logit is masked below), so no load is conditional;
        // all loads of the chunk are requested before any arithmetic
        uint4 raw[32 / V];
        {
            const T* kr = kp + (size_t)(c0 + min(kl, cr - 1)) * row_stride + (size_t)g * DD + prt * 32;
#pragma unroll
            for (int c = 0; c < 32 / V; ++c) raw[c] = *reinterpret_cast<const uint4*>(kr + c * V);
        }
        float v0[16], v1[16];
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            {   // clamped like the keys: a row past the end gets probability 0
                const T* vr = vp + (size_t)(c0 + min(kk, cr - 1)) * row_stride + (size_t)g * DD + 2 * lane;
                if constexpr (sizeof(T) == 2) {          // one 4-byte load for the bf16 pair
                    const uint32_t pr = *reinterpret_cast<const uint32_t*>(vr);
                    v0[kk] = lo_bf16(pr);
                    v1[kk] = hi_bf16(pr);
                } else {
                    v0[kk] = Elem<T>::ld(vr);
                    v1[kk] = Elem<T>::ld(vr + 1);
                }
            }
        }
        if constexpr (sizeof(T) == 2) {
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t kw[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
#pragma unroll
                for (int h = 0; h < G; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        dot[h] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw[i]),
                                                                 __builtin_bit_cast(bf16x2, qs[h][prt * 16 + c * 4 + i]), dot[h], false);
            }
#pragma unroll
            for (int h = 0; h < G; ++h) dot[h] *= scale_log2e;
        } else {
#pragma unroll
            for (int c = 0; c < 32 / V; ++c) {
                float f[V];
                Elem<T>::unpack(raw[c], f);
#pragma unroll
                for (int h = 0; h < G; ++h) {
#pragma unroll
                    for (int i = 0; i < V; ++i) dot[h] += f[i] * qs[h][prt * 32 + c * V + i];
                }
            }
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float sc = dot[h] + __shfl_xor(dot[h], 1, 64);
            sc += __shfl_xor(sc, 2, 64);
            sc = kl < cr ? sc : -INFINITY;
            float cm = sc;                               // maximum over the 16 keys (lanes 4 apart)
#pragma unroll
            for (int o = 4; o < 64; o <<= 1) cm = fmaxf(cm, __shfl_xor(cm, o, 64));
            const float mn = fmaxf(m_run[h], cm);        // finite: the wave has at least one key here
            const float al = __builtin_amdgcn_exp2f(m_run[h] - mn);
            const float p = __builtin_amdgcn_exp2f(sc - mn);
            float sum = p;
#pragma unroll
            for (int o = 4; o < 64; o <<= 1) sum += __shfl_xor(sum, o, 64);
            m_run[h] = mn;
            l_run[h] = l_run[h] * al + sum;
            oacc[h][0] *= al;
            oacc[h][1] *= al;
            if (prt == 0) ps[wave][kl][h] = p;
        }
        __builtin_amdgcn_wave_barrier();                 // the strip is written and read by this wave only
#pragma unroll
        for (int kk = 0; kk < 16; ++kk)
#pragma unroll
            for (int h = 0; h < G; ++h)
                {
                    const float p = ps[wave][kk][h];
                    oacc[h][0] += p * v0[kk];
                    oacc[h][1] += p * v1[kk];
                }
        __builtin_amdgcn_wave_barrier();
    }
    // ---- the four waves' states are merged, and the partial is written
#pragma unroll
    for (int h = 0; h < G; ++h)
        {
            red[wave][h][2 * lane] = oacc[h][0];
            red[wave][h][2 * lane + 1] = oacc[h][1];
            if (lane == 0) { ws_m[wave][h] = m_run[h]; ws_l[wave][h] = l_run[h]; }
        }
    __syncthreads();
    for (int i = tid; i < G * DD; i += 256) {
        const int h = i / DD, dd = i - h * DD;
        const float M = fmaxf(fmaxf(ws_m[0][h], ws_m[1][h]), fmaxf(ws_m[2][h], ws_m[3][h]));
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = ws_l[w][h] > 0.f ? __builtin_amdgcn_exp2f(ws_m[w][h] - M) : 0.f;
            o += sc * red[w][h][dd];
            l += sc * ws_l[w][h];
        }
        float* dst = part + ((size_t)item * Hq + g * G + h) * DPART;
        dst[dd] = o;
        if (dd == 0) { dst[DD] = M; dst[DD + 1] = l; }
    }
}

// One workgroup per query head: out = sum_i 2^(m_i - M) o_i / sum_i 2^(m_i - M) l_i over the partials.  1024
// threads = 8 groups of 128 dims; the weights of up to 1024 partials at a time are formed in parallel and kept in
// LDS, then group j takes the partials j, j + 8, ... so that the loads of a thread do not depend on each other.
// A partial without keys has sum 0 and zero values, and gets weight 0.
constexpr int DMT = 1024;
template <typename T>
__global__ void __launch_bounds__(DMT) decode_attn_merge_kernel(const float* __restrict__ part, int n_items, int Hq,
                                                                T* __restrict__ out) {
    __shared__ float wts[DMT];
    __shared__ float wred[DMT / 64];
    __shared__ float accs[DMT / DD][DD];
    const int h = blockIdx.x, tid = threadIdx.x, grp = tid >> 7, dd = tid & (DD - 1);
    auto item = [&](int i) { return part + ((size_t)i * Hq + h) * DPART; };
    float m = -INFINITY;
    for (int i = tid; i < n_items; i += DMT) m = fmaxf(m, item(i)[DD]);
    m = wave_max(m);
    if ((tid & 63) == 0) wred[tid >> 6] = m;
    __syncthreads();
    float M = wred[0];
#pragma unroll
    for (int i = 1; i < DMT / 64; ++i) M = fmaxf(M, wred[i]);
    __syncthreads();
    float lsum = 0.f, acc = 0.f;
    for (int base = 0; base < n_items; base += DMT) {
        const int i = base + tid;
        float w = 0.f;
        if (i < n_items) {
            const float* p = item(i);
            if (p[DD + 1] > 0.f) {
                w = __builtin_amdgcn_exp2f(p[DD] - M);
                lsum += w * p[DD + 1];
            }
        }
        wts[tid] = w;
        __syncthreads();
        const int cnt = min(DMT, n_items - base);
#pragma unroll 4
        for (int j = grp; j < cnt; j += DMT / DD) acc += wts[j] * item(base + j)[dd];
        __syncthreads();
    }
    lsum = wave_sum(lsum);
    if ((tid & 63) == 0) wred[tid >> 6] = lsum;
    accs[grp][dd] = acc;
    __syncthreads();
    if (grp == 0) {
        float L = 0.f, a = 0.f;
#pragma unroll
        for (int i = 0; i < DMT / 64; ++i) L += wred[i];
#pragma unroll
        for (int i = 0; i < DMT / DD; ++i) a += accs[i][dd];
        Elem<T>::st(out + (size_t)h * DD + dd, a / L);
    }
}

template <typename T, int G>
static void launch_decode_partial(const void* q, const void* pool, size_t slot_bytes, size_t layer_offset,
                                  const int* block_of_slot, int n_slots, int block, int n_prompt, const void* k_resp,
                                  const void* v_resp, int n_resp, int Hq, int Hkv, float sl, float* part, int n_items,
                                  hipStream_t st) {
    hipLaunchKernelGGL((decode_attn_partial_kernel<T, G>), dim3(n_items, Hkv), dim3(256), 0, st, (const T*)q,
                       (const unsigned char*)pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt,
                       (const T*)k_resp, (const T*)v_resp, n_resp, Hq, Hkv, sl, part);
}

template <typename T>
static int launch_decode_attn_t(const void* q, const void* pool, size_t slot_bytes, size_t layer_offset,
                                const int* block_of_slot, int n_slots, int block, int n_prompt, const void* k_resp,
                                const void* v_resp, int n_resp, int Hq, int Hkv, float sl, void* out, float* part,
                                hipStream_t st) {
    const int n_items = n_slots + (n_resp + DCH - 1) / DCH;
#define SLIM_DEC(GG) case GG: launch_decode_partial<T, GG>(q, pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, \
                                                            n_prompt, k_resp, v_resp, n_resp, Hq, Hkv, sl, part, n_items, st); break
    switch (Hq / Hkv) {
        SLIM_DEC(1); SLIM_DEC(2); SLIM_DEC(3); SLIM_DEC(4); SLIM_DEC(5); SLIM_DEC(6); SLIM_DEC(7); SLIM_DEC(8);
        default: return SLIM_UNSUPPORTED;
    }
#undef SLIM_DEC
    hipLaunchKernelGGL(decode_attn_merge_kernel<T>, dim3(Hq), dim3(DMT), 0, st, part, n_items, Hq, (T*)out);
    return check_launch();
}

int launch_decode_attn(const void* q, const void* pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot,
                       int n_slots, int block, int n_prompt, const void* k_resp, const void* v_resp, int n_resp, int Hq,
                       int Hkv, float scale, int dtype, void* out, float* part, hipStream_t st) {
    const float sl = scale * 1.4426950408889634f;
    if (dtype == SLIM_BF16)
        return launch_decode_attn_t<bf16_t>(q, pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt, k_resp,
                                            v_resp, n_resp, Hq, Hkv, sl, out, part, st);
    return launch_decode_attn_t<float>(q, pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt, k_resp,
                                       v_resp, n_resp, Hq, Hkv, sl, out, part, st);
}

}  // namespace slim
