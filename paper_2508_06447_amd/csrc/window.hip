// The window query of Eq. (2) straight from the hidden rows of the local window, without materialised Query
// states: qt[g, :] = (1 / (w * Hq)) * sum over the window rows t and the query heads h of group g of
// RoPE_t(Wq_h x_t * rstd_t + bq_h).  The projection of so few rows (w <= 256, typically 64) is a skinny GEMM whose
// only cost is reading Wq once; a tile-per-workgroup GEMM has too few tiles to pull it through the chip, so here
// the reduction dimension is split over workgroups and waves, the partial sums (float) go to a small buffer, and a
// second kernel adds them in a fixed order, applies the row scale, bias and rotation in float, and takes the means.
// bf16 inputs, head_dim 128.
#include "slim_common.h"

namespace slim {

constexpr int kWqFeat = 32;                          // features (Wq rows) per workgroup: two MFMA row tiles
constexpr int kWqTok = 64;                           // window rows per workgroup: four MFMA column tiles
constexpr int kWqChunk = 64;                         // reduction elements per wave and loop step

// grid (n_feat / 32, splits, ceil(w / 64)), 256 threads.  The k_in / 64 chunks of the reduction dimension are dealt
// evenly to the splits * 4 waves.  16x16x32 MFMAs: lane (r, q) = (lane % 16, lane / 16) supplies 8 elements of row r,
// and which 8 is free as long as both operands agree, so in step j of a chunk it reads the 16 bytes at
// j * 64 + q * 16 of its row: every load instruction covers 64 contiguous bytes of each of 16 rows.
// partial[split][t][f] float, t < w.
__global__ void __launch_bounds__(256) window_proj_kernel(const bf16_t* __restrict__ x, int lda, int w,
                                                          const bf16_t* __restrict__ wq, int k_in, int n_feat,
                                                          float* __restrict__ partial) {
    __shared__ f32x4 red[4][8][64];                     // [wave][feature tile * 4 + row tile][lane], 32 KB
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, q = lane >> 4;
    const int f0 = blockIdx.x * kWqFeat, split = blockIdx.y, t0 = blockIdx.z * kWqTok;
    const int n_chunks = k_in / kWqChunk, parts = gridDim.y * 4, me = split * 4 + wave;
    const int c_lo = (int)((long long)n_chunks * me / parts), c_hi = (int)((long long)n_chunks * (me + 1) / parts);
    const bf16_t* pa[2];
    const bf16_t* pb[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) pa[i] = wq + (size_t)(f0 + i * 16 + l16) * k_in + q * 8;
    // Rows past the window repeat its last row: they are computed and never stored.
#pragma unroll
    for (int i = 0; i < 4; ++i) pb[i] = x + (size_t)min(t0 + i * 16 + l16, w - 1) * lda + q * 8;
    f32x4 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a[2][2], b[2][4];                             // [step of the chunk][tile]
    auto load = [&](int c) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = c * kWqChunk + j * 32;
#pragma unroll
            for (int i = 0; i < 2; ++i) a[j][i] = *reinterpret_cast<const bf16x8*>(pa[i] + k);
#pragma unroll
            for (int i = 0; i < 4; ++i) b[j][i] = *reinterpret_cast<const bf16x8*>(pb[i] + k);
        }
    };
    if (c_lo < c_hi) load(c_lo);
    for (int c = c_lo; c < c_hi; ++c) {
        bf16x8 ca[2][2], cb[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int i = 0; i < 2; ++i) ca[j][i] = a[j][i];
#pragma unroll
            for (int i = 0; i < 4; ++i) cb[j][i] = b[j][i];
        }
        if (c + 1 < c_hi) load(c + 1);                   // the next chunk's loads fly under this chunk's MFMAs
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    acc[i][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ca[j][i], cb[j][m], acc[i][m], 0, 0, 0);
    }
    // Accumulator element e of lane (l16, q) in tile (i, m): feature f0 + i * 16 + q * 4 + e, row t0 + m * 16 + l16.
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int m = 0; m < 4; ++m) red[wave][i * 4 + m][lane] = acc[i][m];
    __syncthreads();
    // Wave v adds tiles 2v and 2v + 1 of the four waves, in wave order; a lane stores 4 consecutive features of a row.
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int tile = wave * 2 + u, i = tile >> 2, m = tile & 3;
        const int t = t0 + m * 16 + l16;
        f32x4 s = red[0][tile][lane];
#pragma unroll
        for (int v = 1; v < 4; ++v) s += red[v][tile][lane];
        if (t < w)
            *reinterpret_cast<f32x4*>(partial + ((size_t)split * w + t) * n_feat + f0 + i * 16 + q * 4) = s;
    }
}

// grid (Hkv, 4), 1024 threads: thread (slice, cc) takes rotation pair (c, c + 64), c = blockIdx.y * 16 + cc, of every
// head of the group for the window rows slice, slice + 64, ..; the 64 slices are added in slice order through LDS.
__global__ void __launch_bounds__(1024) window_query_finish_kernel(const float* __restrict__ partial, int splits, int w,
                                                                   int n_feat, const float* __restrict__ rstd,
                                                                   const bf16_t* __restrict__ bias,
                                                                   const float* __restrict__ table, int Hq, int Hkv,
                                                                   float* __restrict__ qt) {
    __shared__ float part[64][32];
    const int cc = threadIdx.x & 15, slice = threadIdx.x >> 4, g = blockIdx.x, G = Hq / Hkv;
    const int c = blockIdx.y * 16 + cc;
    float lo_sum = 0.f, hi_sum = 0.f;
    for (int t = slice; t < w; t += 64) {
        const float cs = table[(size_t)t * 128 + c], sn = table[(size_t)t * 128 + 64 + c];
        const float sc = rstd ? rstd[t] : 1.f;
        for (int j = 0; j < G; ++j) {
            const int f = (g * G + j) * 128 + c;
            float lo = 0.f, hi = 0.f;
            for (int s = 0; s < splits; ++s) {
                const float* row = partial + ((size_t)s * w + t) * n_feat + f;
                lo += row[0];
                hi += row[64];
            }
            lo *= sc;
            hi *= sc;
            if (bias) { lo += bf16_to_f32(bias[f]); hi += bf16_to_f32(bias[f + 64]); }
            lo_sum += lo * cs - hi * sn;
            hi_sum += hi * cs + lo * sn;
        }
    }
    part[slice][cc] = lo_sum;
    part[slice][16 + cc] = hi_sum;
    __syncthreads();
    if (threadIdx.x < 32) {
        float s = 0.f;
#pragma unroll 8
        for (int i = 0; i < 64; ++i) s += part[i][threadIdx.x];
        const int e = (threadIdx.x < 16 ? c : 64 + blockIdx.y * 16 + (threadIdx.x - 16));
        qt[g * 128 + e] = s / ((float)w * (float)Hq);
    }
}

// How many ways the workgroups split the reduction dimension: enough for one workgroup per CU or more, at least
// one 64-element chunk per wave.
static int window_splits(int n_feat, int k_in) {
    int s = 1;
    while (s < kWindowSplitsMax && (n_feat / kWqFeat) * s < 512 && k_in / kWqChunk >= 8 * s) s *= 2;
    return s;
}

// x: the w window rows (bf16, row stride lda), wq [Hq*128, k_in] bf16, rstd [w] or null, bias [Hq*128] bf16 or null,
// table [w, 128] cos | sin of the window rows, partial: kWindowSplitsMax * w * Hq*128 floats.  k_in % 64 == 0,
// 16-byte aligned rows (checked by the caller).
int launch_window_query_rows(const void* x, int lda, const void* wq, const void* bias, const float* rstd,
                             const float* table, int w, int Hq, int Hkv, int k_in, float* partial, float* qt,
                             hipStream_t st) {
    const int n_feat = Hq * 128, splits = window_splits(n_feat, k_in);
    hipLaunchKernelGGL(window_proj_kernel, dim3(n_feat / kWqFeat, splits, (w + kWqTok - 1) / kWqTok), dim3(256), 0, st,
                       (const bf16_t*)x, lda, w, (const bf16_t*)wq, k_in, n_feat, partial);
    int rc = check_launch();
    if (rc) return rc;
    hipLaunchKernelGGL(window_query_finish_kernel, dim3(Hkv, 4), dim3(1024), 0, st, (const float*)partial, splits, w, n_feat,
                       rstd, (const bf16_t*)bias, table, Hq, Hkv, qt);
    return check_launch();
}

}  // namespace slim
