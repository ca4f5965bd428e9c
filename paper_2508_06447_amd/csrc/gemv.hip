// Projections of ONE token (decoding phase of Fig. 2: "QKV Generation" and "FFN" for the newly decoded token):
//   out[n] = s * (w[n, :] . x) (+ bias[n]) (+ residual[n]),   or   silu(s * w0[n, :] . x) * (s * w1[n, :] . x),
// s = *scale (the token's 1/rms for a fused RMSNorm with folded gain) or 1.  HBM-bound: every weight is read once.
// The token is staged in LDS as floats; a wave owns 4 consecutive output features and walks their rows in 16-byte
// chunks, 64 chunks per step, so that a step reads 4 contiguous KiB; sums by wave reduction, one rounding.
#include "slim_common.h"

namespace slim {

template <typename T, bool SWIGLU>
__global__ void __launch_bounds__(256) gemv_kernel(const T* __restrict__ w0, const T* __restrict__ w1,
                                                   const T* __restrict__ x, const float* __restrict__ scale,
                                                   const T* __restrict__ bias, const T* residual, T* out, int N, int K) {
    constexpr int V = Elem<T>::kVec, R = 4, NM = SWIGLU ? 2 : 1;
    extern __shared__ float xs[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int c = tid; c < K / V; c += 256) {
        float f[V];
        Elem<T>::unpack(*reinterpret_cast<const uint4*>(x + (size_t)c * V), f);
#pragma unroll
        for (int i = 0; i < V; ++i) xs[c * V + i] = f[i];
    }
    __syncthreads();
    const int r0 = (blockIdx.x * 4 + wave) * R;
    if (r0 >= N) return;
    float acc[NM][R];
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[m][r] = 0.f;
    const T* rows[NM][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const size_t ro = (size_t)min(r0 + r, N - 1) * K;    // rows past the end repeat the last one (not stored)
        rows[0][r] = w0 + ro;
        if (SWIGLU) rows[NM - 1][r] = w1 + ro;
    }
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
    if (lane < R && r0 + lane < N) {
        const float sc = scale ? *scale : 1.0f;
        float a = lane == 0 ? acc[0][0] : lane == 1 ? acc[0][1] : lane == 2 ? acc[0][2] : acc[0][3];
        a *= sc;
        const int n = r0 + lane;
        if (SWIGLU) {
            float u = lane == 0 ? acc[NM - 1][0] : lane == 1 ? acc[NM - 1][1] : lane == 2 ? acc[NM - 1][2] : acc[NM - 1][3];
            u *= sc;
            a = a / (1.0f + __expf(-a)) * u;
        }
        if (bias) a += Elem<T>::ld(bias + n);
        if (residual) a += Elem<T>::ld(residual + n);
        Elem<T>::st(out + n, a);
    }
}

// At most one of w1 (SwiGLU) and bias/residual combinations as in the matrix versions; k_in a multiple of 8 (bf16)
// or 4 (fp32), x and the weights 16-byte aligned, k_in * 4 bytes of LDS (checked by the caller).
int launch_gemv(const void* w0, const void* w1, const void* x, const float* scale, const void* bias, const void* residual,
                int n_out, int k_in, int dtype, void* out, hipStream_t st) {
    const dim3 grid((n_out + 15) / 16);
    const size_t smem = (size_t)k_in * sizeof(float);
#define SLIM_GEMV(T, S) hipLaunchKernelGGL((gemv_kernel<T, S>), grid, dim3(256), smem, st, (const T*)w0, (const T*)w1, \
        (const T*)x, scale, (const T*)bias, (const T*)residual, (T*)out, n_out, k_in)
    if (dtype == SLIM_BF16) { if (w1) SLIM_GEMV(bf16_t, true); else SLIM_GEMV(bf16_t, false); }
    else                    { if (w1) SLIM_GEMV(float, true);  else SLIM_GEMV(float, false); }
#undef SLIM_GEMV
    return check_launch();
}

}  // namespace slim
