// Projections of ONE token (decoding phase of Fig. 2: "QKV Generation" and "FFN" for the newly decoded token):
//   out[n] = s * (w[n, :] . x) (+ bias[n]) (+ residual[n]),   or   silu(s * w0[n, :] . x) * (s * w1[n, :] . x),
// s = the token's 1/rms (fused RMSNorm with a folded gain: formed by every workgroup from its own LDS copy of the
// token, or read from *scale) or 1.  HBM-bound: every weight is read once.  The token is staged in LDS as floats; a
// wave owns 4 output features and walks their rows in 16-byte chunks, 64 chunks per step; sums by wave reduction, one
// rounding.  Up to three weight matrices with their own bias and output share one launch (the Query, Key and Value
// projections), and a segment can ask for RoPE at the token's position: its waves then own the features
// {i, i+1, i+64, i+65} of a 128-wide head, so that the rotate-half partners meet in one wave.
#include "slim_common.h"

namespace slim {

struct GemvSeg {
    const void* w;
    const void* bias;        // null: none
    void* out;
    int n;                   // output features (a multiple of 4 except in the last segment; of 128 with rope)
    int rope;                // != 0: rotate heads of 128 features
};
struct GemvArgs {
    GemvSeg seg[3];
    int n_seg;
    const void* w_up;        // SwiGLU: second matrix of segment 0 (n_seg == 1)
    const void* x;
    const float* scale;      // null: 1 (or the in-kernel statistic when norm_eps >= 0)
    float norm_eps;          // >= 0: s = 1 / sqrt(mean(x^2) + norm_eps) computed here
    const void* residual;    // segment 0 only
    int k;
    int position;            // RoPE position of the token
    float theta;
};

template <typename T, bool SWIGLU>
__global__ void __launch_bounds__(256) gemv_kernel(GemvArgs a) {
    constexpr int V = Elem<T>::kVec, R = 4, NM = SWIGLU ? 2 : 1;
    extern __shared__ float xs[];
    __shared__ float part[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, K = a.k;
    const T* x = (const T*)a.x;
    float ss = 0.f;
    for (int c = tid; c < K / V; c += 256) {
        float f[V];
        Elem<T>::unpack(*reinterpret_cast<const uint4*>(x + (size_t)c * V), f);
#pragma unroll
        for (int i = 0; i < V; ++i) { xs[c * V + i] = f[i]; ss += f[i] * f[i]; }
    }
    ss = wave_sum(ss);
    if (lane == 0) part[wave] = ss;
    __syncthreads();
    float sc = a.scale ? *a.scale : 1.0f;
    if (a.norm_eps >= 0.f) sc = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)K + a.norm_eps);

    // this wave's segment and rows
    int j = blockIdx.x * 4 + wave, s = 0;
    while (s < a.n_seg - 1 && j >= (a.seg[s].n + R - 1) / R) { j -= (a.seg[s].n + R - 1) / R; ++s; }
    const GemvSeg sg = a.seg[s];
    const int N = sg.n;
    if (j * R >= N) return;
    int rown[R];                                         // output feature of each of the wave's rows
    if (sg.rope) {
        const int head = j >> 5, i0 = (j & 31) * 2;
#pragma unroll
        for (int r = 0; r < R; ++r) rown[r] = head * 128 + i0 + (r & 1) + (r >> 1) * 64;
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) rown[r] = min(j * R + r, N - 1);   // rows past the end repeat the last one
    }
    const T* rows[NM][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        rows[0][r] = (const T*)sg.w + (size_t)rown[r] * K;
        if (SWIGLU) rows[NM - 1][r] = (const T*)a.w_up + (size_t)rown[r] * K;
    }
    float acc[NM][R];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[m][r] = 0.f;
    const int nchunk = K / V;
#pragma unroll 2
    for (int c = lane; c < nchunk; c += 64) {
        uint4 raw[NM][R];
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int r = 0; r < R; ++r) raw[m][r] = *reinterpret_cast<const uint4*>(rows[m][r] + (size_t)c * V);
        float xf[V];
#pragma unroll
        for (int i = 0; i < V; ++i) xf[i] = xs[c * V + i];
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float f[V];
                Elem<T>::unpack(raw[m][r], f);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[m][r] += f[i] * xf[i];
            }
    }
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[m][r] = wave_sum(acc[m][r]);
    if (lane < R) {
        auto pick = [&](const float (&v)[R], int r) { return r == 0 ? v[0] : r == 1 ? v[1] : r == 2 ? v[2] : v[3]; };
        const int n = sg.rope ? (j >> 5) * 128 + (j & 31) * 2 + (lane & 1) + (lane >> 1) * 64 : j * R + lane;
        if (n < N) {
            float val = pick(acc[0], lane) * sc;
            if (SWIGLU) {
                const float u = pick(acc[NM - 1], lane) * sc;
                val = val / (1.0f + __expf(-val)) * u;
            }
            const T* bias = (const T*)sg.bias;
            if (bias) val += Elem<T>::ld(bias + n);
            if (sg.rope) {
                // partner = the row 64 features away, held by lane ^ 2; both with scale and bias applied
                const int np = n ^ 64;                   // (n % 128) +- 64 inside the head
                float other = pick(acc[0], lane ^ 2) * sc;
                if (bias) other += Elem<T>::ld(bias + np);
                const int i = n & 63;
                const double inv_freq = pow((double)a.theta, -2.0 * (double)i / 128.0);
                const double ang = (double)a.position * inv_freq;
                const double kk = rint(ang * 0.15915494309189535);
                const double red = fma(-kk, 2.4492935982947064e-16, fma(-kk, 6.283185307179586, ang));
                float sn, cs;
                sincosf((float)red, &sn, &cs);
                val = (n & 64) ? val * cs + other * sn : val * cs - other * sn;
            }
            if (s == 0 && a.residual) val += Elem<T>::ld((const T*)a.residual + n);
            Elem<T>::st((T*)sg.out + n, val);
        }
    }
}

static int launch_gemv_args(const GemvArgs& a, int dtype, hipStream_t st) {
    int waves = 0;
    for (int s = 0; s < a.n_seg; ++s) waves += (a.seg[s].n + 3) / 4;
    const dim3 grid((waves + 3) / 4);
    const size_t smem = (size_t)a.k * sizeof(float);
#define SLIM_GEMV(T, S) hipLaunchKernelGGL((gemv_kernel<T, S>), grid, dim3(256), smem, st, a)
    if (dtype == SLIM_BF16) { if (a.w_up) SLIM_GEMV(bf16_t, true); else SLIM_GEMV(bf16_t, false); }
    else                    { if (a.w_up) SLIM_GEMV(float, true);  else SLIM_GEMV(float, false); }
#undef SLIM_GEMV
    return check_launch();
}

// One matrix (or gate/up pair).  k_in a multiple of 8 (bf16) or 4 (fp32), x and the weights 16-byte aligned,
// k_in * 4 bytes of LDS (checked by the caller).  norm_eps >= 0 computes the scale from x itself.
int launch_gemv(const void* w0, const void* w1, const void* x, const float* scale, float norm_eps, const void* bias,
                const void* residual, int n_out, int k_in, int dtype, void* out, hipStream_t st) {
    GemvArgs a{};
    a.seg[0] = GemvSeg{w0, bias, out, n_out, 0};
    a.n_seg = 1;
    a.w_up = w1;
    a.x = x;
    a.scale = scale;
    a.norm_eps = norm_eps;
    a.residual = residual;
    a.k = k_in;
    return launch_gemv_args(a, dtype, st);
}

// Query, Key and Value projections of one token in one launch: RMSNorm statistic in the kernel when norm_eps >= 0
// (x = the raw residual row), biases or null, RoPE on q and k at `position` (heads of 128).
int launch_gemv_qkv(const void* wq, const void* wk, const void* wv, const void* bq, const void* bk, const void* bv,
                    const void* x, float norm_eps, int n_q, int n_kv, int k_in, int position, float theta, int dtype,
                    void* q, void* k, void* v, hipStream_t st) {
    GemvArgs a{};
    a.seg[0] = GemvSeg{wq, bq, q, n_q, 1};
    a.seg[1] = GemvSeg{wk, bk, k, n_kv, 1};
    a.seg[2] = GemvSeg{wv, bv, v, n_kv, 0};
    a.n_seg = 3;
    a.x = x;
    a.norm_eps = norm_eps;
    a.k = k_in;
    a.position = position;
    a.theta = theta;
    return launch_gemv_args(a, dtype, st);
}

}  // namespace slim
