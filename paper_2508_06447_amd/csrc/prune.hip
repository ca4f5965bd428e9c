// Block-wise prompt token pruning (Section 4.2): block scores (Eq. 1-2), block selection,
// hidden-state compaction.  All three are HBM-/latency-bound; none uses matrix cores.
#include "slim_common.h"

namespace slim {

// -------------------------------------------------------------------------------------------------
// Scores.  By linearity of Eq. (2),
//   (1/Hq) sum_h q_l^h . k_rep^{g(h)}(j,m) = k_rep(j,m) . qt,   qt[g,:] = (1/Hq) sum_{h in group g} q_l^h,
// so the window query is reduced once to qt[Hkv*d] and each unit needs one dot product of length
// Hkv*d with its mean key.
// -------------------------------------------------------------------------------------------------
// 64 elements of qt per workgroup, 16 slices of the window per element (slice s takes tokens s, s+16, ..);
// the slices are summed in a fixed order through LDS, so the result is deterministic.
template <typename T>
__global__ void __launch_bounds__(1024) window_query_kernel(const T* __restrict__ q_win, int w, int Hq, int Hkv,
                                                            int d, float* __restrict__ qt) {
    __shared__ float part[16][64];
    const int le = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + le;                  // element of [Hkv, d]
    float acc = 0.f;
    if (e < Hkv * d) {
        const int g = e / d, c = e - g * d, G = Hq / Hkv;
        for (int t = slice; t < w; t += 16)
            for (int h = g * G; h < (g + 1) * G; ++h) acc += Elem<T>::ld(q_win + ((size_t)t * Hq + h) * d + c);
    }
    part[slice][le] = acc;
    __syncthreads();
    if (slice == 0 && e < Hkv * d) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += part[i][le];
        qt[e] = s / ((float)w * (float)Hq);              // mean over the window, then mean over heads
    }
}

// One workgroup per block j, one wave per TokenUnit (waves stride over the units).  A wave reads its
// unit's rows in 16-byte chunks, accumulates sum_t k[t,:] . qt, divides by the unit's token count
// (Eq. 1 then the dot of Eq. 2) and the workgroup takes the max over units.
template <typename T>
__global__ void __launch_bounds__(1024) block_score_kernel(const T* __restrict__ k, const float* __restrict__ qt,
                                                            int N, int E /*Hkv*d*/, int block, int unit,
                                                            float* __restrict__ scores) {
    constexpr int V = Elem<T>::kVec;
    extern __shared__ float smem[];                      // qt copy [E] + per-wave maxima [16]
    float* qs = smem;
    float* wmax = smem + E;
    const int j = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int e = threadIdx.x; e < E; e += blockDim.x) qs[e] = qt[e];
    __syncthreads();
    const int b0 = j * block, b1 = min(b0 + block, N);
    const int nchunk = E / V;
    float best = -INFINITY;
    for (int u0 = b0 + wave * unit; u0 < b1; u0 += nw * unit) {
        const int u1 = min(u0 + unit, b1);
        float acc = 0.f;
        for (int c = lane; c < nchunk; c += 64) {
            float ksum[V];
#pragma unroll
            for (int i = 0; i < V; ++i) ksum[i] = 0.f;
#pragma unroll 8
            for (int t = u0; t < u1; ++t) {
                uint4 raw = *reinterpret_cast<const uint4*>(k + (size_t)t * E + (size_t)c * V);
                float f[V];
                Elem<T>::unpack(raw, f);
#pragma unroll
                for (int i = 0; i < V; ++i) ksum[i] += f[i];
            }
#pragma unroll
            for (int i = 0; i < V; ++i) acc += ksum[i] * qs[c * V + i];
        }
        acc = wave_sum(acc) / (float)(u1 - u0);
        best = fmaxf(best, acc);
    }
    if (lane == 0) wmax[wave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = wmax[0];
        for (int i = 1; i < nw; ++i) m = fmaxf(m, wmax[i]);
        scores[j] = m;
    }
}

// Pooled scoring, the two baselines of the scoring ablation (Table 3): one representative key per block,
// the average or the element-wise maximum of its token keys, then the same dot with qt.  One workgroup
// of 512 threads per block: thread = (token slice s, 16-byte chunk c); slices are combined through LDS in
// a fixed order, then the chunks' partial dots are summed over the workgroup.
template <typename T, bool MAXPOOL>
__global__ void __launch_bounds__(512) block_pool_score_kernel(const T* __restrict__ k, const float* __restrict__ qt,
                                                               int N, int E /*Hkv*d*/, int block,
                                                               float* __restrict__ scores) {
    constexpr int V = Elem<T>::kVec;
    extern __shared__ float smem[];                      // qt copy [E] + slice partials [512*V] + wave sums [8]
    float* qs = smem;
    float* part = smem + E;
    float* wsum = part + 512 * V;
    const int j = blockIdx.x, tid = threadIdx.x;
    for (int e = tid; e < E; e += 512) qs[e] = qt[e];
    const int b0 = j * block, b1 = min(b0 + block, N);
    const int nchunk = E / V;
    int C = 512;
    while (C > nchunk) C >>= 1;                          // chunks handled side by side: power of two <= nchunk
    const int S = 512 / C, c0 = tid % C, sl = tid / C;   // S token slices: slice sl takes tokens sl, sl+S, ..
    float dot = 0.f;
    __syncthreads();
    for (int base = 0; base < nchunk; base += C) {
        const int c = base + c0;
        float p[V];
#pragma unroll
        for (int i = 0; i < V; ++i) p[i] = MAXPOOL ? -INFINITY : 0.f;
        if (c < nchunk) {
            for (int t = b0 + sl; t < b1; t += S) {
                uint4 raw = *reinterpret_cast<const uint4*>(k + (size_t)t * E + (size_t)c * V);
                float f[V];
                Elem<T>::unpack(raw, f);
#pragma unroll
                for (int i = 0; i < V; ++i) p[i] = MAXPOOL ? fmaxf(p[i], f[i]) : p[i] + f[i];
            }
        }
        if (S > 1) {
#pragma unroll
            for (int i = 0; i < V; ++i) part[(sl * C + c0) * V + i] = p[i];
            __syncthreads();
            if (sl == 0) {
                for (int o = 1; o < S; ++o)
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        const float x = part[(o * C + c0) * V + i];
                        p[i] = MAXPOOL ? fmaxf(p[i], x) : p[i] + x;
                    }
            }
            __syncthreads();
        }
        if (sl == 0 && c < nchunk) {
#pragma unroll
            for (int i = 0; i < V; ++i) dot += p[i] * qs[c * V + i];
        }
    }
    dot = wave_sum(dot);
    if ((tid & 63) == 0) wsum[tid >> 6] = dot;
    __syncthreads();
    if (tid == 0) {
        float m = 0.f;
        for (int i = 0; i < 8; ++i) m += wsum[i];
        scores[j] = MAXPOOL ? m : m / (float)(b1 - b0);
    }
}

// pooling: 0 = TokenUnits (Eq. 1-2), 1 = average pooling, 2 = max pooling
int launch_score(const void* q_win, const void* k, int N, int w, int Hq, int Hkv, int d, int block, int unit,
                 int pooling, int dtype, float* scores, float* qtilde, hipStream_t st) {
    const int E = Hkv * d, nb = (N + block - 1) / block;
    const int M = (block + unit - 1) / unit;
    const int waves = M < 1 ? 1 : (M > 16 ? 16 : M);
    const size_t smem = (size_t)(E + 16) * sizeof(float);
    dim3 g1((E + 63) / 64);
    if (dtype == SLIM_BF16) {
        hipLaunchKernelGGL(window_query_kernel<bf16_t>, g1, dim3(1024), 0, st, (const bf16_t*)q_win, w, Hq, Hkv, d, qtilde);
        const size_t smem_p = (size_t)(E + 512 * Elem<bf16_t>::kVec + 8) * sizeof(float);
        if (pooling == 1)
            hipLaunchKernelGGL((block_pool_score_kernel<bf16_t, false>), dim3(nb), dim3(512), smem_p, st, (const bf16_t*)k,
                               qtilde, N, E, block, scores);
        else if (pooling == 2)
            hipLaunchKernelGGL((block_pool_score_kernel<bf16_t, true>), dim3(nb), dim3(512), smem_p, st, (const bf16_t*)k,
                               qtilde, N, E, block, scores);
        else
            hipLaunchKernelGGL(block_score_kernel<bf16_t>, dim3(nb), dim3(64 * waves), smem, st, (const bf16_t*)k,
                               qtilde, N, E, block, unit, scores);
    } else {
        hipLaunchKernelGGL(window_query_kernel<float>, g1, dim3(1024), 0, st, (const float*)q_win, w, Hq, Hkv, d, qtilde);
        const size_t smem_p = (size_t)(E + 512 * Elem<float>::kVec + 8) * sizeof(float);
        if (pooling == 1)
            hipLaunchKernelGGL((block_pool_score_kernel<float, false>), dim3(nb), dim3(512), smem_p, st, (const float*)k,
                               qtilde, N, E, block, scores);
        else if (pooling == 2)
            hipLaunchKernelGGL((block_pool_score_kernel<float, true>), dim3(nb), dim3(512), smem_p, st, (const float*)k,
                               qtilde, N, E, block, scores);
        else
            hipLaunchKernelGGL(block_score_kernel<float>, dim3(nb), dim3(64 * waves), smem, st, (const float*)k, qtilde,
                               N, E, block, unit, scores);
    }
    return check_launch();
}

// -------------------------------------------------------------------------------------------------
// Decode-time form of the scores (Section 4.2: during decoding the window is the most recent tokens and
// the prompt's Key states may sit in CPU memory).  Eq. (1) is evaluated once, when the keys are produced,
// and kept as k_rep[nb, M, E] in float; Eq. (2) then reads 1/unit of the bytes of the keys.
// -------------------------------------------------------------------------------------------------
// One wave per TokenUnit, 4 units per workgroup.  Units past the end of the prompt are written as zeros.
template <typename T>
__global__ void __launch_bounds__(256) unit_keys_kernel(const T* __restrict__ k, int N, int E, int block, int unit,
                                                         int M, int n_units, float* __restrict__ k_rep) {
    constexpr int V = Elem<T>::kVec;
    const int lane = threadIdx.x & 63;
    const int u = blockIdx.x * 4 + (threadIdx.x >> 6);   // unit index = j*M + m
    if (u >= n_units) return;
    const int j = u / M, m = u - j * M;
    const int b1 = min((j + 1) * block, N);
    const int u0 = j * block + m * unit, u1 = min(u0 + unit, b1);   // u1 <= u0: the unit does not exist
    const float inv = u1 > u0 ? 1.f / (float)(u1 - u0) : 0.f;
    for (int c = lane; c < E / V; c += 64) {
        float ksum[V];
#pragma unroll
        for (int i = 0; i < V; ++i) ksum[i] = 0.f;
#pragma unroll 8
        for (int t = u0; t < u1; ++t) {
            uint4 raw = *reinterpret_cast<const uint4*>(k + (size_t)t * E + (size_t)c * V);
            float f[V];
            Elem<T>::unpack(raw, f);
#pragma unroll
            for (int i = 0; i < V; ++i) ksum[i] += f[i];
        }
        float* dst = k_rep + (size_t)u * E + (size_t)c * V;
#pragma unroll
        for (int q = 0; q < V / 4; ++q)
            *reinterpret_cast<float4*>(dst + 4 * q) = make_float4(ksum[4 * q] * inv, ksum[4 * q + 1] * inv,
                                                                  ksum[4 * q + 2] * inv, ksum[4 * q + 3] * inv);
    }
}

// One workgroup per block, one wave per stored unit key: dot with qt, max over the units the block has.
__global__ void __launch_bounds__(1024) unit_score_kernel(const float* __restrict__ k_rep,
                                                           const float* __restrict__ qt, int N, int E, int block,
                                                           int unit, int M, float* __restrict__ scores) {
    extern __shared__ float smem[];                      // qt copy [E] + per-wave maxima [16]
    float* qs = smem;
    float* wmax = smem + E;
    const int j = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int e = threadIdx.x; e < E; e += blockDim.x) qs[e] = qt[e];
    __syncthreads();
    const int rows = min(block, N - j * block);
    const int m_have = (rows + unit - 1) / unit;         // units this block really has
    float best = -INFINITY;
    for (int m = wave; m < m_have; m += nw) {
        const float* kr = k_rep + ((size_t)j * M + m) * E;
        float acc = 0.f;
        for (int c = lane; c < E / 4; c += 64) {
            const float4 a = *reinterpret_cast<const float4*>(kr + 4 * c);
            acc += a.x * qs[4 * c] + a.y * qs[4 * c + 1] + a.z * qs[4 * c + 2] + a.w * qs[4 * c + 3];
        }
        best = fmaxf(best, wave_sum(acc));
    }
    if (lane == 0) wmax[wave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        float mx = wmax[0];
        for (int i = 1; i < nw; ++i) mx = fmaxf(mx, wmax[i]);
        scores[j] = mx;
    }
}

// Block scores from per-token partial scores (the K projection's RoPE epilogue leaves, for every token and kv
// head, the dot of the token's key with that head's part of the window query).  Summing the heads gives
// k_t . qt; by linearity the mean of those over a TokenUnit is Eq. (1) dotted as in Eq. (2), and the block takes
// the maximum over its units.  One workgroup per block, one thread per unit (strided), fixed summation order.
__global__ void __launch_bounds__(256) token_score_blocks_kernel(const float* __restrict__ ts, int N, int H, int block,
                                                                 int unit, float* __restrict__ scores) {
    __shared__ float wmax[4];
    const int j = blockIdx.x, b0 = j * block, b1 = min(b0 + block, N);
    float best = -INFINITY;
    for (int u0 = b0 + threadIdx.x * unit; u0 < b1; u0 += 256 * unit) {
        const int u1 = min(min(u0 + unit, b0 + block), b1);
        float acc = 0.f;
        for (int t = u0; t < u1; ++t) {
            float s = 0.f;
            for (int h = 0; h < H; ++h) s += ts[(size_t)t * H + h];
            acc += s;
        }
        best = fmaxf(best, acc / (float)(u1 - u0));
    }
    best = wave_max(best);
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) scores[j] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}

int launch_token_score_blocks(const float* token_scores, int N, int H, int block, int unit, float* scores, hipStream_t st) {
    const int nb = (N + block - 1) / block;
    hipLaunchKernelGGL(token_score_blocks_kernel, dim3(nb), dim3(256), 0, st, token_scores, N, H, block, unit, scores);
    return check_launch();
}

int launch_window_query(const void* q_win, int w, int Hq, int Hkv, int d, int dtype, float* qtilde, hipStream_t st) {
    dim3 g1((Hkv * d + 63) / 64);
    if (dtype == SLIM_BF16)
        hipLaunchKernelGGL(window_query_kernel<bf16_t>, g1, dim3(1024), 0, st, (const bf16_t*)q_win, w, Hq, Hkv, d, qtilde);
    else
        hipLaunchKernelGGL(window_query_kernel<float>, g1, dim3(1024), 0, st, (const float*)q_win, w, Hq, Hkv, d, qtilde);
    return check_launch();
}

int launch_unit_keys(const void* k, int N, int E, int block, int unit, int dtype, float* k_rep, hipStream_t st) {
    const int nb = (N + block - 1) / block, M = (block + unit - 1) / unit, n_units = nb * M;
    dim3 grid((n_units + 3) / 4);
    if (dtype == SLIM_BF16)
        hipLaunchKernelGGL(unit_keys_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)k, N, E, block, unit, M,
                           n_units, k_rep);
    else
        hipLaunchKernelGGL(unit_keys_kernel<float>, grid, dim3(256), 0, st, (const float*)k, N, E, block, unit, M,
                           n_units, k_rep);
    return check_launch();
}

int launch_score_from_unit_keys(const void* q_win, const float* k_rep, int N, int w, int Hq, int Hkv, int d,
                                int block, int unit, int dtype, float* scores, float* qtilde, hipStream_t st) {
    const int E = Hkv * d, nb = (N + block - 1) / block, M = (block + unit - 1) / unit;
    const int waves = M > 16 ? 16 : M;
    dim3 g1((E + 63) / 64);
    if (dtype == SLIM_BF16)
        hipLaunchKernelGGL(window_query_kernel<bf16_t>, g1, dim3(1024), 0, st, (const bf16_t*)q_win, w, Hq, Hkv, d, qtilde);
    else
        hipLaunchKernelGGL(window_query_kernel<float>, g1, dim3(1024), 0, st, (const float*)q_win, w, Hq, Hkv, d, qtilde);
    hipLaunchKernelGGL(unit_score_kernel, dim3(nb), dim3(64 * waves), (size_t)(E + 16) * sizeof(float), st, k_rep, qtilde,
                       N, E, block, unit, M, scores);
    return check_launch();
}

// -------------------------------------------------------------------------------------------------
// Selection: one workgroup.  An 8-bit-digit radix select over order-preserving integer keys finds
// the score of the last block to take; equal scores are taken in ascending index order; the kept
// set is written ascending through a prefix sum of the keep flags.  Integer work only, so the
// result does not depend on the order in which threads run.
// -------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t b = __builtin_bit_cast(uint32_t, s);
    if ((b << 1) == 0) b = 0;                            // -0.0 == +0.0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);   // ascending in the float order
}

constexpr int kSelThreads = 1024;

// Exclusive prefix sum of one int per thread across the workgroup; returns the total in `total`.
__device__ int block_exclusive_scan(int v, int* wsum /*[16]*/, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();                                     // wsum free from the previous use
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < kSelThreads / 64; ++i) {
        int s = wsum[i];
        if (i < wave) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

__global__ void __launch_bounds__(kSelThreads) select_blocks_kernel(const float* __restrict__ scores, int nb,
                                                                     int n_keep, unsigned flags,
                                                                     int* __restrict__ kept) {
    __shared__ int hist[256];
    __shared__ int wsum[kSelThreads / 64];
    __shared__ uint32_t s_prefix;
    __shared__ int s_remaining;
    const int tid = threadIdx.x;
    const bool f_first = flags & SLIM_FORCE_FIRST, f_last = flags & SLIM_FORCE_LAST;
    auto forced = [&](int j) { return (f_first && j == 0) || (f_last && j == nb - 1); };
    const int n_forced = (f_first ? 1 : 0) + ((f_last && !(f_first && nb == 1)) ? 1 : 0);
    const int take = n_keep - n_forced;                  // > 0 slots for the non-forced blocks, < nb - n_forced

    uint32_t thr = 0;                                    // key of the last block taken
    int n_eq = 0;                                        // how many blocks with that exact key to take
    if (take > 0) {
        if (tid == 0) { s_prefix = 0; s_remaining = take; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            for (int j = tid; j < nb; j += kSelThreads) {
                if (forced(j)) continue;
                uint32_t key = score_key(scores[j]);
                if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
            }
            __syncthreads();
            if (tid < 64) {
                // Find the digit that holds the rem-th largest candidate: lane l owns the digits
                // 255-4l .. 252-4l (descending); a wave scan gives the count of larger digits.
                const int rem = s_remaining;
                int c[4], tot = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) { c[k] = hist[255 - (4 * tid + k)]; tot += c[k]; }
                int inc = tot;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const int t = __shfl_up(inc, o, 64);
                    if (tid >= o) inc += t;
                }
                int above = inc - tot;                   // candidates with a larger digit than this lane's first
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (above < rem && rem <= above + c[k]) {          // true for exactly one (lane, k)
                        s_prefix = prefix | ((uint32_t)(255 - (4 * tid + k)) << shift);
                        s_remaining = rem - above;
                    }
                    above += c[k];
                }
            }
            __syncthreads();
        }
        thr = s_prefix;
        n_eq = s_remaining;
    }

    int eq_seen = 0, out_base = 0;
    for (int base = 0; base < nb; base += kSelThreads) {
        const int j = base + tid;
        bool in = j < nb, fz = in && forced(j);
        uint32_t key = (in && !fz && take > 0) ? score_key(scores[j]) : 0;
        int is_eq = (in && !fz && take > 0 && key == thr) ? 1 : 0;
        int tot_eq;
        int eq_rank = block_exclusive_scan(is_eq, wsum, tot_eq) + eq_seen;
        int keep = fz || (in && !fz && take > 0 && (key > thr || (is_eq && eq_rank < n_eq)));
        int tot_keep;
        int slot = block_exclusive_scan(keep, wsum, tot_keep) + out_base;
        if (keep) kept[slot] = j;
        eq_seen += tot_eq;
        out_base += tot_keep;
    }
}

__global__ void iota_kernel(int* out, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = i;
}

__global__ void positions_kernel(const int* __restrict__ pos_in, int* __restrict__ pos_out, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) pos_out[i] = pos_in ? pos_in[i] : i;
}

int launch_positions(const int* pos_in, int* pos_out, int n, hipStream_t st) {
    hipLaunchKernelGGL(positions_kernel, dim3((n + 255) / 256), dim3(256), 0, st, pos_in, pos_out, n);
    return check_launch();
}

int launch_select(const float* scores, int nb, int n_keep, unsigned flags, int* kept, hipStream_t st) {
    if (n_keep >= nb) {
        hipLaunchKernelGGL(iota_kernel, dim3((nb + 255) / 256), dim3(256), 0, st, kept, nb);
    } else {
        hipLaunchKernelGGL(select_blocks_kernel, dim3(1), dim3(kSelThreads), 0, st, scores, nb, n_keep, flags, kept);
    }
    return check_launch();
}

// -------------------------------------------------------------------------------------------------
// Compaction: a kept block is one contiguous run of block*row bytes in src and in dst, so the gather
// is a segmented copy.  grid = (chunks per block, kept blocks); each thread moves kCopyVecs 16-byte
// vectors, loads first, then stores.
// -------------------------------------------------------------------------------------------------
constexpr int kCopyThreads = 256;
constexpr int kCopyVecs = 4;

template <typename V>
__global__ void __launch_bounds__(kCopyThreads) compact_kernel(const V* __restrict__ src, V* __restrict__ dst,
                                                               const int* __restrict__ kept, int block, int N,
                                                               int nb, size_t row_vecs,
                                                               const int* __restrict__ pos_in,
                                                               int* __restrict__ pos_out) {
    const int i = blockIdx.y;
    const int kb = kept[i];
    if ((unsigned)kb >= (unsigned)nb) return;
    const int rows = min(block, N - kb * block);
    const size_t seg = (size_t)rows * row_vecs;
    const V* s = src + (size_t)kb * block * row_vecs;
    V* d = dst + (size_t)i * block * row_vecs;
    const size_t base = (size_t)blockIdx.x * (kCopyThreads * kCopyVecs) + threadIdx.x;
    V tmp[kCopyVecs];
#pragma unroll
    for (int u = 0; u < kCopyVecs; ++u) {
        size_t o = base + (size_t)u * kCopyThreads;
        if (o < seg) tmp[u] = __builtin_nontemporal_load(s + o);
    }
#pragma unroll
    for (int u = 0; u < kCopyVecs; ++u) {
        size_t o = base + (size_t)u * kCopyThreads;
        if (o < seg) __builtin_nontemporal_store(tmp[u], d + o);
    }
    if (blockIdx.x == 0 && pos_out) {
        for (int r = threadIdx.x; r < rows; r += kCopyThreads) {
            int t = kb * block + r;
            pos_out[(size_t)i * block + r] = pos_in ? pos_in[t] : t;
        }
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

int launch_compact(const void* src, const int* pos_in, const int* kept, int n_keep, int block, int N,
                   int row_elems, int dtype, void* dst, int* pos_out, hipStream_t st) {
    const size_t row_bytes = (size_t)row_elems * elem_size(dtype);
    const int nb = (N + block - 1) / block;
    const size_t per = (size_t)kCopyThreads * kCopyVecs;
    if (row_bytes % 16 == 0 && aligned16(src) && aligned16(dst)) {
        size_t rv = row_bytes / 16, chunks = ((size_t)block * rv + per - 1) / per;
        hipLaunchKernelGGL(compact_kernel<u32x4>, dim3((unsigned)chunks, n_keep), dim3(kCopyThreads), 0, st,
                           (const u32x4*)src, (u32x4*)dst, kept, block, N, nb, rv, pos_in, pos_out);
    } else if (row_bytes % 4 == 0) {
        size_t rv = row_bytes / 4, chunks = ((size_t)block * rv + per - 1) / per;
        hipLaunchKernelGGL(compact_kernel<uint32_t>, dim3((unsigned)chunks, n_keep), dim3(kCopyThreads), 0, st,
                           (const uint32_t*)src, (uint32_t*)dst, kept, block, N, nb, rv, pos_in, pos_out);
    } else {
        size_t rv = row_bytes / 2, chunks = ((size_t)block * rv + per - 1) / per;
        hipLaunchKernelGGL(compact_kernel<uint16_t>, dim3((unsigned)chunks, n_keep), dim3(kCopyThreads), 0, st,
                           (const uint16_t*)src, (uint16_t*)dst, kept, block, N, nb, rv, pos_in, pos_out);
    }
    return check_launch();
}

// Several arrays compacted by the same kept set in one launch (hidden rows + positions, keys, row statistics):
// grid = (chunks of the widest array's block run, kept blocks, arrays).  Rows are multiples of 4 bytes; a run is
// moved in 16-byte vectors when it allows, else in words.
struct CompactSegs {
    const unsigned char* src[4];
    unsigned char* dst[4];
    unsigned long long row_bytes[4];
    int n;
};

__global__ void __launch_bounds__(kCopyThreads) compact_multi_kernel(CompactSegs segs, const int* __restrict__ kept,
                                                                     int block, int N, int nb,
                                                                     const int* __restrict__ pos_in,
                                                                     int* __restrict__ pos_out) {
    const int i = blockIdx.y, a = blockIdx.z;
    const int kb = kept[i];
    if ((unsigned)kb >= (unsigned)nb) return;
    const int rows = min(block, N - kb * block);
    const size_t rb = segs.row_bytes[a];
    const size_t run = (size_t)rows * rb;
    const unsigned char* s = segs.src[a] + (size_t)kb * block * rb;
    unsigned char* d = segs.dst[a] + (size_t)i * block * rb;
    if (((rb * block) % 16 == 0) && (run % 16 == 0) && ((((uintptr_t)segs.src[a]) | ((uintptr_t)segs.dst[a])) & 15) == 0) {
        const u32x4* sv = reinterpret_cast<const u32x4*>(s);
        u32x4* dv = reinterpret_cast<u32x4*>(d);
        const size_t seg = run / 16;
        const size_t base = (size_t)blockIdx.x * (kCopyThreads * kCopyVecs) + threadIdx.x;
        u32x4 tmp[kCopyVecs];
#pragma unroll
        for (int u = 0; u < kCopyVecs; ++u) {
            const size_t o = base + (size_t)u * kCopyThreads;
            if (o < seg) tmp[u] = __builtin_nontemporal_load(sv + o);
        }
#pragma unroll
        for (int u = 0; u < kCopyVecs; ++u) {
            const size_t o = base + (size_t)u * kCopyThreads;
            if (o < seg) __builtin_nontemporal_store(tmp[u], dv + o);
        }
    } else {
        const uint32_t* sw = reinterpret_cast<const uint32_t*>(s);
        uint32_t* dw = reinterpret_cast<uint32_t*>(d);
        const size_t seg = run / 4;
        for (size_t o = (size_t)blockIdx.x * kCopyThreads + threadIdx.x; o < seg; o += (size_t)gridDim.x * kCopyThreads)
            dw[o] = sw[o];
    }
    if (a == 0 && blockIdx.x == 0 && pos_out) {
        for (int r = threadIdx.x; r < rows; r += kCopyThreads) {
            const int t = kb * block + r;
            pos_out[(size_t)i * block + r] = pos_in ? pos_in[t] : t;
        }
    }
}

// Up to 4 arrays [N, row_bytes[a]] -> [n', row_bytes[a]]; positions ride with array 0.  row_bytes % 4 == 0.
int launch_compact_multi(int n_arrays, const void* const* src, void* const* dst, const size_t* row_bytes, const int* pos_in,
                         int* pos_out, const int* kept, int n_keep, int block, int N, hipStream_t st) {
    CompactSegs segs;
    size_t widest = 0;
    segs.n = n_arrays;
    for (int a = 0; a < 4; ++a) {
        const bool on = a < n_arrays;
        segs.src[a] = on ? (const unsigned char*)src[a] : nullptr;
        segs.dst[a] = on ? (unsigned char*)dst[a] : nullptr;
        segs.row_bytes[a] = on ? row_bytes[a] : 0;
        if (on && row_bytes[a] > widest) widest = row_bytes[a];
    }
    const size_t per = (size_t)kCopyThreads * kCopyVecs * 16;
    const size_t chunks = ((size_t)block * widest + per - 1) / per;
    const int nb = (N + block - 1) / block;
    hipLaunchKernelGGL(compact_multi_kernel, dim3((unsigned)chunks, n_keep, n_arrays), dim3(kCopyThreads), 0, st, segs, kept,
                       block, N, nb, pos_in, pos_out);
    return check_launch();
}

}  // namespace slim
