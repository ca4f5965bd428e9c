// Dense projections of the layer ("QKV Generation", output projection and FFN of Fig. 2):
//   out[m, n] = sum_k a[m, k] * w[n, k]            (both operands contiguous along k)
// with three epilogues: plain, + residual, and SwiGLU (two weight matrices, silu(gate) * up).
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The weight tile is the MFMA "A" operand
// and the activation tile the "B" operand, so a lane ends up with 4 consecutive output features of
// one token and stores them as one 8-byte vector.
#include "slim_common.h"

namespace slim {

enum { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2 };

constexpr int BK = 64;                                   // k-depth of an LDS tile (8 chunks of 16 bytes)

// LDS tile: rows of 64 bf16 = 8 chunks of 16 B; chunk c of row r lives at chunk slot c ^ swz(r),
// so that the 16 lanes served together by a 128-bit LDS read hit distinct banks.
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }
__device__ __forceinline__ int lds_off(int r, int c) { return (r * 8 + (c ^ swz(r))) * 16; }   // bytes

// TW x TA: number of 32-row MFMA tiles per wave along the weight (n) and activation (m) directions.
// Workgroup = 4 waves arranged WGN x WGM.  SwiGLU uses two weight tiles per n (gate, up).
template <int TW, int TA, int WGN, int WGM, int EPI>
__global__ void __launch_bounds__(256) gemm_bf16_kernel(const bf16_t* __restrict__ A, int lda,
                                                        const bf16_t* __restrict__ W0,
                                                        const bf16_t* __restrict__ W1,
                                                        const bf16_t* R, bf16_t* C, int ldo, int M, int N, int K,
                                                        int tiles_m, int tiles_n) {
    static_assert(WGN * WGM == 4, "4 waves");
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;        // weight matrices
    constexpr int BN = 32 * TW * WGN;                    // output features per workgroup (per matrix)
    constexpr int BM = 32 * TA * WGM;                    // tokens per workgroup
    constexpr int WROWS = BN * NW;                       // weight rows staged per k-tile
    constexpr int STAGE = (WROWS + BM) * BK * 2;         // bytes per LDS stage
    extern __shared__ __align__(16) unsigned char lds[];

    // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so give each XCD a
    // contiguous run of logical tiles; inside the run walk bands of GM token-tiles, feature-tile by
    // feature-tile, so the workgroups resident on one XCD share few distinct operand tiles in its L2.
    int L = blockIdx.x;
    const int total = tiles_m * tiles_n;
    if (total % 8 == 0) L = (L & 7) * (total >> 3) + (L >> 3);
    constexpr int GM = 8;
    const int band_sz = GM * tiles_n;
    const int band = L / band_sz;
    const int gm = min(GM, tiles_m - band * GM);
    const int rem = L - band * band_sz;
    const int tm = band * GM + rem % gm, tn = rem / gm;
    const int n0 = tn * BN, m0 = tm * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WGN, wm = wave / WGN;
    const int l32 = lane & 31, hh = lane >> 5;

    // global -> register staging: thread owns chunk column (tid & 7) of rows (tid >> 3) + 32*i
    constexpr int WLD = WROWS / 32, ALD = BM / 32;
    uint4 wreg[WLD], areg[ALD];
    const int lc = tid & 7, lr = tid >> 3;
    auto load_tiles = [&](int k0) {
        const int kk = k0 + lc * 8;
        const bool kin = kk < K;
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const int r = lr + 32 * i;
            const int mat = NW == 2 ? r / BN : 0;
            const int n = min(n0 + (NW == 2 ? r - mat * BN : r), N - 1);
            const bf16_t* src = (mat ? W1 : W0) + (size_t)n * K + kk;
            wreg[i] = kin ? *reinterpret_cast<const uint4*>(src) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < ALD; ++i) {
            const int m = min(m0 + lr + 32 * i, M - 1);
            areg[i] = kin ? *reinterpret_cast<const uint4*>(A + (size_t)m * lda + kk) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tiles = [&](int stage) {
        unsigned char* ws = lds + stage * STAGE;
        unsigned char* as = ws + WROWS * BK * 2;
#pragma unroll
        for (int i = 0; i < WLD; ++i) *reinterpret_cast<uint4*>(ws + lds_off(lr + 32 * i, lc)) = wreg[i];
#pragma unroll
        for (int i = 0; i < ALD; ++i) *reinterpret_cast<uint4*>(as + lds_off(lr + 32 * i, lc)) = areg[i];
    };

    f32x16 acc[NW][TW][TA];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
            for (int j = 0; j < TA; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[w][i][j][v] = 0.f;

    const int KT = (K + BK - 1) / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_tiles((kt + 1) * BK);
        const unsigned char* ws = lds + (kt & 1) * STAGE;
        const unsigned char* as = ws + WROWS * BK * 2;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[TA], wf[NW][TW];
#pragma unroll
            for (int j = 0; j < TA; ++j)
                af[j] = *reinterpret_cast<const bf16x8*>(as + lds_off((wm * TA + j) * 32 + l32, ks * 2 + hh));
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < TW; ++i)
                    wf[w][i] = *reinterpret_cast<const bf16x8*>(
                        ws + lds_off(w * BN + (wn * TW + i) * 32 + l32, ks * 2 + hh));
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < TW; ++i)
#pragma unroll
                    for (int j = 0; j < TA; ++j)
                        acc[w][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[w][i], af[j], acc[w][i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_tiles((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: acc[..][i][j][v] is out[token m][feature n] with
    //   m = m0 + (wm*TA + j)*32 + l32,   n = n0 + (wn*TW + i)*32 + 8*(v/4) + 4*hh + (v%4)
    const bool vec_ok = (N % 4 == 0) && (ldo % 4 == 0);
#pragma unroll
    for (int j = 0; j < TA; ++j) {
        const int m = m0 + (wm * TA + j) * 32 + l32;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < TW; ++i) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int n = n0 + (wn * TW + i) * 32 + 8 * vg + 4 * hh;
                if (n >= N) continue;
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (EPI == EPI_SWIGLU) {
                        const float g = acc[0][i][j][vg * 4 + e], u = acc[NW - 1][i][j][vg * 4 + e];
                        o[e] = g / (1.0f + __expf(-g)) * u;
                    } else {
                        o[e] = acc[0][i][j][vg * 4 + e];
                    }
                }
                bf16_t* dst = C + (size_t)m * ldo + n;
                if (vec_ok) {
                    if (EPI == EPI_RESIDUAL) {
                        const uint2 r = *reinterpret_cast<const uint2*>(R + (size_t)m * ldo + n);
                        o[0] += lo_bf16(r.x); o[1] += hi_bf16(r.x); o[2] += lo_bf16(r.y); o[3] += hi_bf16(r.y);
                    }
                    *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (n + e < N) {
                            float val = o[e];
                            if (EPI == EPI_RESIDUAL) val += bf16_to_f32(R[(size_t)m * ldo + n + e]);
                            dst[e] = f32_to_bf16(val);
                        }
                    }
                }
            }
        }
    }
}

template <int TW, int TA, int WGN, int WGM, int EPI>
static int launch_bf16(const bf16_t* A, int lda, const bf16_t* W0, const bf16_t* W1, const bf16_t* R, bf16_t* C,
                       int ldo, int M, int N, int K, hipStream_t st) {
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int BN = 32 * TW * WGN, BM = 32 * TA * WGM;
    constexpr size_t smem = 2 * (size_t)(BN * NW + BM) * BK * 2;
    auto kern = gemm_bf16_kernel<TW, TA, WGN, WGM, EPI>;
    static bool attr_done = false;                       // raising the LDS limit is per function, once
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_hip_error(e);
        attr_done = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, st, A, lda, W0, W1, R, C, ldo, M, N, K,
                       tiles_m, tiles_n);
    return check_launch();
}

// fp32 path (small fp32 workloads only): 64x64 output tile, 16-deep k-tiles in LDS, 4x4 per thread.
template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, int lda,
                                                       const float* __restrict__ W0, const float* __restrict__ W1,
                                                       const float* R, float* C, int ldo, int M, int N, int K) {
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    __shared__ float as[16][65];
    __shared__ float ws[NW][16][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[NW][4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            const int r = i >> 4, c = i & 15, k = k0 + c;
            const int m = m0 + r, n = n0 + r;
            as[c][r] = (m < M && k < K) ? A[(size_t)m * lda + k] : 0.f;
            ws[0][c][r] = (n < N && k < K) ? W0[(size_t)n * K + k] : 0.f;
            if (NW == 2) ws[NW - 1][c][r] = (n < N && k < K) ? W1[(size_t)n * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            float a[4], w[NW][4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = as[c][ty * 4 + i];
#pragma unroll
            for (int q = 0; q < NW; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) w[q][j] = ws[q][c][tx * 4 + j];
#pragma unroll
            for (int q = 0; q < NW; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[q][i][j] += a[i] * w[q][j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float o = acc[0][i][j];
            if (EPI == EPI_SWIGLU) { const float g = o; o = g / (1.0f + expf(-g)) * acc[NW - 1][i][j]; }
            if (EPI == EPI_RESIDUAL) o += R[(size_t)m * ldo + n];
            C[(size_t)m * ldo + n] = o;
        }
    }
}

int launch_linear(const void* a, int lda, const void* w0, const void* w1, const void* residual, int m,
                  int n_out, int k_in, int ldo, int dtype, void* out, hipStream_t st) {
    if (dtype == SLIM_F32) {
        dim3 grid((n_out + 63) / 64, (m + 63) / 64);
#define SLIM_F32_GEMM(E) hipLaunchKernelGGL(gemm_f32_kernel<E>, grid, dim3(256), 0, st, (const float*)a, lda, \
        (const float*)w0, (const float*)w1, (const float*)residual, (float*)out, ldo, m, n_out, k_in)
        if (w1) SLIM_F32_GEMM(EPI_SWIGLU); else if (residual) SLIM_F32_GEMM(EPI_RESIDUAL); else SLIM_F32_GEMM(EPI_PLAIN);
#undef SLIM_F32_GEMM
        return check_launch();
    }
    const bf16_t *A = (const bf16_t*)a, *W0 = (const bf16_t*)w0, *W1 = (const bf16_t*)w1, *R = (const bf16_t*)residual;
    bf16_t* C = (bf16_t*)out;
    if (w1) return launch_bf16<2, 4, 2, 2, EPI_SWIGLU>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
    if (m <= 128) {
        if (residual) return launch_bf16<2, 2, 2, 2, EPI_RESIDUAL>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
        return launch_bf16<2, 2, 2, 2, EPI_PLAIN>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
    }
    if (residual) return launch_bf16<4, 4, 2, 2, EPI_RESIDUAL>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
    return launch_bf16<4, 4, 2, 2, EPI_PLAIN>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
}

}  // namespace slim
