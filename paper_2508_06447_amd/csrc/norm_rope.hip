// RMSNorm and rotary position embedding: the per-token, HBM-bound parts of "QKV Generation" (Fig. 2).
#include "slim_common.h"
#include <math.h>

namespace slim {

// One workgroup per token row.  Pass 1 sums squares (fp32), pass 2 re-reads the row (L2-resident)
// and writes gain * x * rsqrt(mean + eps).
template <typename T, bool VEC>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                      int hidden, float eps, T* __restrict__ out) {
    constexpr int V = Elem<T>::kVec;
    __shared__ float part[4];
    const T* row = x + (size_t)blockIdx.x * hidden;
    T* orow = out + (size_t)blockIdx.x * hidden;
    float ss = 0.f;
    if (VEC) {
        for (int c = threadIdx.x; c < hidden / V; c += 256) {
            float f[V];
            Elem<T>::unpack(*reinterpret_cast<const uint4*>(row + (size_t)c * V), f);
#pragma unroll
            for (int i = 0; i < V; ++i) ss += f[i] * f[i];
        }
    } else {
        for (int c = threadIdx.x; c < hidden; c += 256) { float v = Elem<T>::ld(row + c); ss += v * v; }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float inv = 1.0f / sqrtf(tot / (float)hidden + eps);
    if (VEC) {
        for (int c = threadIdx.x; c < hidden / V; c += 256) {
            float f[V], g[V];
            Elem<T>::unpack(*reinterpret_cast<const uint4*>(row + (size_t)c * V), f);
            Elem<T>::unpack(*reinterpret_cast<const uint4*>(gain + (size_t)c * V), g);
#pragma unroll
            for (int i = 0; i < V; ++i) f[i] = g[i] * (f[i] * inv);
            *reinterpret_cast<uint4*>(orow + (size_t)c * V) = Elem<T>::pack(f);
        }
    } else {
        for (int c = threadIdx.x; c < hidden; c += 256)
            Elem<T>::st(orow + c, Elem<T>::ld(gain + c) * (Elem<T>::ld(row + c) * inv));
    }
}

int launch_rmsnorm(const void* x, const void* gain, int n, int hidden, float eps, int dtype, void* out, hipStream_t st) {
    const size_t es = elem_size(dtype);
    const bool vec = ((size_t)hidden * es) % 16 == 0 && aligned16(x) && aligned16(out) && aligned16(gain);
#define SLIM_RMS(T, VEC) hipLaunchKernelGGL((rmsnorm_kernel<T, VEC>), dim3(n), dim3(256), 0, st, (const T*)x, \
                                            (const T*)gain, hidden, eps, (T*)out)
    if (dtype == SLIM_BF16) { if (vec) SLIM_RMS(bf16_t, true); else SLIM_RMS(bf16_t, false); }
    else                    { if (vec) SLIM_RMS(float, true);  else SLIM_RMS(float, false); }
#undef SLIM_RMS
    return check_launch();
}

// RoPE in place on x[n, H, d].  A thread owns two adjacent rotation indices (2p, 2p+1) of one token
// and walks over the heads, so each angle is formed once per token: angle = pos * inv_freq[i] in
// double, sincos in double, rounded to float.  inv_freq comes from the host (theta^(-2i/d) in double).
struct RopeFreq { double inv_freq[128]; };               // head_dim <= 256

template <typename T>
__global__ void __launch_bounds__(256) rope_kernel(T* __restrict__ x, const int* __restrict__ pos, int pos0, int n,
                                                   int H, int d, RopeFreq fr) {
    const int per_tok = d / 4;                           // threads per token
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int t = idx / per_tok, p = idx - t * per_tok;
    if (t >= n) return;
    const double ps = (double)(pos ? pos[t] : pos0 + t);
    double s0, c0, s1, c1;
    sincos(ps * fr.inv_freq[2 * p], &s0, &c0);
    sincos(ps * fr.inv_freq[2 * p + 1], &s1, &c1);
    const float cf0 = (float)c0, sf0 = (float)s0, cf1 = (float)c1, sf1 = (float)s1;
    const int half = d / 2;
    T* base = x + (size_t)t * H * d + 2 * p;
    for (int h = 0; h < H; ++h) {
        T* a = base + (size_t)h * d;
        T* b = a + half;
        float a0 = Elem<T>::ld(a), a1 = Elem<T>::ld(a + 1), b0 = Elem<T>::ld(b), b1 = Elem<T>::ld(b + 1);
        Elem<T>::st(a, a0 * cf0 - b0 * sf0);
        Elem<T>::st(a + 1, a1 * cf1 - b1 * sf1);
        Elem<T>::st(b, b0 * cf0 + a0 * sf0);
        Elem<T>::st(b + 1, b1 * cf1 + a1 * sf1);
    }
}

int launch_rope(void* x, const int* pos, int pos0, int n, int H, int d, float theta, int dtype, hipStream_t st) {
    RopeFreq fr;
    for (int i = 0; i < d / 2; ++i) fr.inv_freq[i] = pow((double)theta, -2.0 * (double)i / (double)d);
    const long long threads = (long long)n * (d / 4);
    dim3 grid((unsigned)((threads + 255) / 256));
    if (dtype == SLIM_BF16) hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, dim3(256), 0, st, (bf16_t*)x, pos, pos0, n, H, d, fr);
    else hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, st, (float*)x, pos, pos0, n, H, d, fr);
    return check_launch();
}

// out[n, k] = w[n, k] * gain[k]: folds an RMSNorm gain into the weights of the projection that follows it.
template <typename T>
__global__ void __launch_bounds__(256) fold_gain_kernel(const T* __restrict__ w, const T* __restrict__ gain, size_t total,
                                                        int k_in, T* __restrict__ out) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256)
        Elem<T>::st(out + i, Elem<T>::ld(w + i) * Elem<T>::ld(gain + (i % k_in)));
}

int launch_fold_gain(const void* w, const void* gain, int n_out, int k_in, int dtype, void* out, hipStream_t st) {
    const size_t total = (size_t)n_out * k_in;
    const unsigned grid = (unsigned)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    if (dtype == SLIM_BF16)
        hipLaunchKernelGGL(fold_gain_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)w, (const bf16_t*)gain, total,
                           k_in, (bf16_t*)out);
    else
        hipLaunchKernelGGL(fold_gain_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)w, (const float*)gain, total, k_in,
                           (float*)out);
    return check_launch();
}

// One rotation angle's cos / sin: the angle is formed in double and reduced to [-pi, pi] in double (two-term
// 2*pi), then evaluated in float: within 3e-7 of the double result, four orders below a bf16 rounding, at a
// fraction of the cost of a double sincos.
__device__ __forceinline__ void rope_cos_sin(double pos, double inv_freq, float& cs, float& sn) {
    const double a = pos * inv_freq;
    const double k = rint(a * 0.15915494309189535);                      // a / (2 pi)
    const double r = fma(-k, 2.4492935982947064e-16, fma(-k, 6.283185307179586, a));
    sincosf((float)r, &sn, &cs);
}

// rstd[t] = 1 / sqrt(mean(x[t, :]^2) + eps): the row statistic of RMSNorm alone, for projections that apply it to
// their accumulators instead of reading a normalised copy.  One wave per row, 4 rows per workgroup.  With a table
// pointer the wave also writes the row's cos / sin table entry (see rope_table_kernel): lane i takes angle i, and
// the arithmetic hides under the row's memory traffic.
template <typename T>
__global__ void __launch_bounds__(256) row_rstd_kernel(const T* __restrict__ x, int n, int hidden, float eps,
                                                       float* __restrict__ rstd, const int* __restrict__ pos, int half,
                                                       RopeFreq fr, float* __restrict__ table) {
    constexpr int V = Elem<T>::kVec;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= n) return;
    const T* row = x + (size_t)t * hidden;
    float ss = 0.f;
    if (hidden % V == 0 && (((uintptr_t)row) & 15) == 0) {
        for (int c = lane; c < hidden / V; c += 64) {
            float f[V];
            Elem<T>::unpack(*reinterpret_cast<const uint4*>(row + (size_t)c * V), f);
#pragma unroll
            for (int i = 0; i < V; ++i) ss += f[i] * f[i];
        }
    } else {
        for (int c = lane; c < hidden; c += 64) { const float v = Elem<T>::ld(row + c); ss += v * v; }
    }
    if (table) {
        const double ps = (double)(pos ? pos[t] : t);
        for (int i = lane; i < half; i += 64) {
            float cs, sn;
            rope_cos_sin(ps, fr.inv_freq[i], cs, sn);
            table[(size_t)t * 2 * half + i] = cs;
            table[(size_t)t * 2 * half + half + i] = sn;
        }
    }
    ss = wave_sum(ss);
    if (lane == 0) rstd[t] = 1.0f / sqrtf(ss / (float)hidden + eps);
}

static RopeFreq rope_freq(int d, float theta) {
    RopeFreq fr;
    for (int i = 0; i < d / 2; ++i) fr.inv_freq[i] = pow((double)theta, -2.0 * (double)i / (double)d);
    return fr;
}

// table != null: also the cos / sin table of the rows' positions (pos null = 0..n-1) for head_dim d.
int launch_row_rstd(const void* x, int n, int hidden, float eps, int dtype, float* rstd, hipStream_t st,
                    const int* pos, int d, float theta, float* table) {
    const RopeFreq fr = table ? rope_freq(d, theta) : RopeFreq();
    if (dtype == SLIM_BF16)
        hipLaunchKernelGGL(row_rstd_kernel<bf16_t>, dim3((n + 3) / 4), dim3(256), 0, st, (const bf16_t*)x, n, hidden, eps, rstd,
                           pos, d / 2, fr, table);
    else
        hipLaunchKernelGGL(row_rstd_kernel<float>, dim3((n + 3) / 4), dim3(256), 0, st, (const float*)x, n, hidden, eps, rstd,
                           pos, d / 2, fr, table);
    return check_launch();
}

// cos / sin table for the RoPE epilogue of the projections: table[t][0..half) = cos(pos[t] * inv_freq[i]),
// table[t][half..2*half) = sin.
__global__ void __launch_bounds__(256) rope_table_kernel(const int* __restrict__ pos, int pos0, int n, int half,
                                                         RopeFreq fr, float* __restrict__ table) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int t = idx / half, i = idx - t * half;
    if (t >= n) return;
    float cs, sn;
    rope_cos_sin((double)(pos ? pos[t] : pos0 + t), fr.inv_freq[i], cs, sn);
    table[(size_t)t * 2 * half + i] = cs;
    table[(size_t)t * 2 * half + half + i] = sn;
}

int launch_rope_table(const int* pos, int pos0, int n, int d, float theta, float* table, hipStream_t st) {
    const RopeFreq fr = rope_freq(d, theta);
    const long long threads = (long long)n * (d / 2);
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, pos, pos0, n, d / 2, fr,
                       table);
    return check_launch();
}

}  // namespace slim
