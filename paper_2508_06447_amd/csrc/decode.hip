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

template <typename T>
__global__ void __launch_bounds__(256) decode_attn_partial_kernel(
    const T* __restrict__ q, const unsigned char* __restrict__ pool, size_t slot_bytes, size_t layer_offset,
    const int* __restrict__ block_of_slot, int n_slots, int block, int n_prompt, const T* __restrict__ k_resp,
    const T* __restrict__ v_resp, int n_resp, int Hq, int Hkv, float scale_log2e, float* __restrict__ part) {
    constexpr int V = Elem<T>::kVec;
    __shared__ float qs[DGMAX][DD];                      // query heads of this kv head, times scale * log2(e)
    __shared__ float ss[DCH][DGMAX];                     // logits, then probabilities, of the chunk
    __shared__ float m_run[DGMAX], l_run[DGMAX], alpha[DGMAX];
    __shared__ float red[4][DGMAX][DD];
    const int item = blockIdx.x, g = blockIdx.y, G = Hq / Hkv, tid = threadIdx.x;
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
    for (int i = tid; i < G * DD; i += 256) qs[i / DD][i % DD] = Elem<T>::ld(q + (size_t)(g * G + i / DD) * DD + i % DD) * scale_log2e;
    if (tid < DGMAX) { m_run[tid] = -INFINITY; l_run[tid] = 0.f; }
    float oacc[DGMAX][2];
#pragma unroll
    for (int h = 0; h < DGMAX; ++h) oacc[h][0] = oacc[h][1] = 0.f;
    __syncthreads();

    const int key = tid >> 2, prt = tid & 3;             // scores: 4 threads per key, 32 dims each
    const int dp = tid & 63, kq = tid >> 6;              // values: thread owns dims 2 dp, 2 dp + 1 of 16 keys
    for (int c0 = 0; c0 < rows; c0 += DCH) {
        const int cr = min(DCH, rows - c0);
        // ---- logits of the chunk
        float dot[DGMAX];
#pragma unroll
        for (int h = 0; h < DGMAX; ++h) dot[h] = 0.f;
        if (key < cr) {
            const T* kr = kp + (size_t)(c0 + key) * row_stride + (size_t)g * DD + prt * 32;
#pragma unroll
            for (int c = 0; c < 32 / V; ++c) {
                float f[V];
                Elem<T>::unpack(*reinterpret_cast<const uint4*>(kr + c * V), f);
#pragma unroll
                for (int h = 0; h < DGMAX; ++h)
                    if (h < G) {
#pragma unroll
                        for (int i = 0; i < V; ++i) dot[h] += f[i] * qs[h][prt * 32 + c * V + i];
                    }
            }
        }
#pragma unroll
        for (int h = 0; h < DGMAX; ++h) {
            dot[h] += __shfl_xor(dot[h], 1, 64);
            dot[h] += __shfl_xor(dot[h], 2, 64);
        }
        if (prt == 0) {
#pragma unroll
            for (int h = 0; h < DGMAX; ++h) ss[key][h] = key < cr ? dot[h] : -INFINITY;
        }
        __syncthreads();
        // ---- running maximum and rescale factor per head (wave 0: lane = key)
        if (tid < 64) {
            for (int h = 0; h < G; ++h) {
                const float cm = wave_max(ss[tid][h]);
                if (tid == 0) {
                    const float mn = fmaxf(m_run[h], cm);                // finite: the chunk has at least one key
                    alpha[h] = __builtin_amdgcn_exp2f(m_run[h] - mn);    // exp2(-inf) = 0 for the first chunk
                    m_run[h] = mn;
                }
            }
        }
        __syncthreads();
        for (int i = tid; i < DCH * G; i += 256) {
            const int kk = i / G, h = i - kk * G;
            ss[kk][h] = __builtin_amdgcn_exp2f(ss[kk][h] - m_run[h]);
        }
        __syncthreads();
        if (tid < 64) {
            for (int h = 0; h < G; ++h) {
                const float sum = wave_sum(ss[tid][h]);
                if (tid == 0) l_run[h] = l_run[h] * alpha[h] + sum;
            }
        }
        // ---- values: this thread's 16 keys of the chunk
#pragma unroll
        for (int h = 0; h < DGMAX; ++h) { oacc[h][0] *= alpha[h < G ? h : 0]; oacc[h][1] *= alpha[h < G ? h : 0]; }
        for (int kk = kq * 16; kk < min(kq * 16 + 16, cr); ++kk) {
            const T* vr = vp + (size_t)(c0 + kk) * row_stride + (size_t)g * DD + 2 * dp;
            float v0, v1;
            if constexpr (sizeof(T) == 2) {              // one 4-byte load for the bf16 pair
                const uint32_t pr = *reinterpret_cast<const uint32_t*>(vr);
                v0 = lo_bf16(pr);
                v1 = hi_bf16(pr);
            } else {
                v0 = Elem<T>::ld(vr);
                v1 = Elem<T>::ld(vr + 1);
            }
#pragma unroll
            for (int h = 0; h < DGMAX; ++h)
                if (h < G) { oacc[h][0] += ss[kk][h] * v0; oacc[h][1] += ss[kk][h] * v1; }
        }
        __syncthreads();                                 // ss and alpha are rewritten by the next chunk
    }
    // ---- the four key quarters are summed, and the partial is written
#pragma unroll
    for (int h = 0; h < DGMAX; ++h)
        if (h < G) { red[kq][h][2 * dp] = oacc[h][0]; red[kq][h][2 * dp + 1] = oacc[h][1]; }
    __syncthreads();
    for (int i = tid; i < G * DD; i += 256) {
        const int h = i / DD, dd = i - h * DD;
        float* dst = part + ((size_t)item * Hq + g * G + h) * DPART;
        dst[dd] = red[0][h][dd] + red[1][h][dd] + red[2][h][dd] + red[3][h][dd];
        if (dd == 0) { dst[DD] = m_run[h]; dst[DD + 1] = l_run[h]; }
    }
}

// One workgroup per query head: out = sum_i 2^(m_i - M) o_i / sum_i 2^(m_i - M) l_i over the partials with keys.
template <typename T>
__global__ void __launch_bounds__(DD) decode_attn_merge_kernel(const float* __restrict__ part, int n_items, int Hq,
                                                               T* __restrict__ out) {
    const int h = blockIdx.x, dd = threadIdx.x;
    float M = -INFINITY;
    for (int i = 0; i < n_items; ++i) M = fmaxf(M, part[((size_t)i * Hq + h) * DPART + DD]);
    float acc = 0.f, l = 0.f;
    for (int i = 0; i < n_items; ++i) {
        const float* p = part + ((size_t)i * Hq + h) * DPART;
        if (p[DD + 1] > 0.f) {
            const float w = __builtin_amdgcn_exp2f(p[DD] - M);
            acc += w * p[dd];
            l += w * p[DD + 1];
        }
    }
    Elem<T>::st(out + (size_t)h * DD + dd, acc / l);
}

int launch_decode_attn(const void* q, const void* pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot,
                       int n_slots, int block, int n_prompt, const void* k_resp, const void* v_resp, int n_resp, int Hq,
                       int Hkv, float scale, int dtype, void* out, float* part, hipStream_t st) {
    const int n_items = n_slots + (n_resp + DCH - 1) / DCH;
    const float sl = scale * 1.4426950408889634f;
    if (dtype == SLIM_BF16) {
        hipLaunchKernelGGL(decode_attn_partial_kernel<bf16_t>, dim3(n_items, Hkv), dim3(256), 0, st, (const bf16_t*)q,
                           (const unsigned char*)pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt,
                           (const bf16_t*)k_resp, (const bf16_t*)v_resp, n_resp, Hq, Hkv, sl, part);
        hipLaunchKernelGGL(decode_attn_merge_kernel<bf16_t>, dim3(Hq), dim3(DD), 0, st, part, n_items, Hq, (bf16_t*)out);
    } else {
        hipLaunchKernelGGL(decode_attn_partial_kernel<float>, dim3(n_items, Hkv), dim3(256), 0, st, (const float*)q,
                           (const unsigned char*)pool, slot_bytes, layer_offset, block_of_slot, n_slots, block, n_prompt,
                           (const float*)k_resp, (const float*)v_resp, n_resp, Hq, Hkv, sl, part);
        hipLaunchKernelGGL(decode_attn_merge_kernel<float>, dim3(Hq), dim3(DD), 0, st, part, n_items, Hq, (float*)out);
    }
    return check_launch();
}

}  // namespace slim
