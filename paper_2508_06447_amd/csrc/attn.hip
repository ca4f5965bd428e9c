// Causal grouped-query prefill attention ("Attention" stage of Fig. 2) over the compacted sequence.
//
// bf16 path (head_dim 128): flash-style single pass with online softmax, v_mfma_f32_32x32x16_bf16.
// A workgroup of 4 waves owns 128 queries of one head, each wave 32 of them; K/V tiles of 64 keys
// are staged in LDS (K row-major, V transposed) and double-buffered.
//
// Both products are computed transposed so that no register shuffle is needed between them:
//   S^T[key, query] = K . Q^T      (A operand = K rows from LDS, B operand = Q rows held in VGPRs)
//   O^T[d,   query] = V^T . P^T    (A operand = V^T rows from LDS, B operand = P^T from the S^T
//                                   accumulators, converted to bf16 in place)
// In the 32x32 accumulator layout a lane owns one query column, so the softmax statistics of a query
// live in two lanes (l and l^32) and need a single cross-lane exchange per tile.  The accumulator's
// row order (rows 8*(v/4) + 4*(lane/32) + v%4) is a permutation of the keys; the V^T fragments are
// read in the same permuted order, which leaves the contraction unchanged.
#include "slim_common.h"

namespace slim {

constexpr int AD = 128;          // head_dim of the MFMA path
constexpr int BQ = 128;          // queries per workgroup
constexpr int BKV = 64;          // keys per tile
constexpr int K_TILE_BYTES = BKV * AD * 2;
constexpr int KV_STAGE_BYTES = 2 * K_TILE_BYTES;

// K tile: row = key, 16 chunks of 16 B per row; chunk c of row r stored at slot c ^ (r & 15).
__device__ __forceinline__ int k_off(int r, int c) { return (r * 16 + (c ^ (r & 15))) * 16; }
// V^T tile: row = d index, 16 units of 8 B (4 keys) per row; unit u of row r at slot u ^ ((r >> 1) & 15).
__device__ __forceinline__ int vt_off(int r, int u) { return (r * 16 + (u ^ ((r >> 1) & 15))) * 8; }

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) attn_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kg,
                                                        const bf16_t* __restrict__ Vg, bf16_t* __restrict__ O,
                                                        int n, int Hq, int Hkv, float scale_log2e, int n_qt) {
    extern __shared__ __align__(16) unsigned char lds[];
    // Workgroup -> (head, query tile).  Ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous range of heads so the query heads sharing a kv head meet in one L2, and start the
    // query tiles with the most keys first.
    int L = blockIdx.x;
    const int total = n_qt * Hq;
    if (total % 8 == 0) L = (L & 7) * (total >> 3) + (L >> 3);
    const int h = L / n_qt, qt = n_qt - 1 - (L - h * n_qt);
    const int g = h / (Hq / Hkv);
    const int q0 = qt * BQ;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int qw0 = q0 + wave * 32;                       // first query of this wave
    const int qi = qw0 + l32;                             // this lane's query
    const size_t qstride = (size_t)Hq * AD, kvstride = (size_t)Hkv * AD;

    // Q fragments (B operand): 8 k-steps x 8 bf16 of row qi, d = ks*16 + hh*8 ..
    bf16x8 qf[8];
    {
        const bf16_t* qrow = Q + (size_t)min(qi, n - 1) * qstride + (size_t)h * AD + hh * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
    }

    // staging registers for the next K/V tile
    uint4 kreg[4];
    uint2 vreg[2][4];
    const bf16_t* kbase = Kg + (size_t)g * AD;
    const bf16_t* vbase = Vg + (size_t)g * AD;
    // K: thread owns chunk (tid & 15) of rows (tid >> 4) + 16*i.
    // V: thread owns d-group dg = tid & 31 (d = 4*dg..+3) and key-groups kg = (tid >> 5) + 8*i (keys 4*kg..+3).
    auto load_kv = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = min(k0 + (tid >> 4) + 16 * i, n - 1);
            kreg[i] = *reinterpret_cast<const uint4*>(kbase + (size_t)r * kvstride + (tid & 15) * 8);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int r = min(k0 + 4 * ((tid >> 5) + 8 * i) + kk, n - 1);
                vreg[i][kk] = *reinterpret_cast<const uint2*>(vbase + (size_t)r * kvstride + (tid & 31) * 4);
            }
    };
    auto store_kv = [&](int stage) {
        unsigned char* ks = lds + stage * KV_STAGE_BYTES;
        unsigned char* vs = ks + K_TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(ks + k_off((tid >> 4) + 16 * i, tid & 15)) = kreg[i];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kg = (tid >> 5) + 8 * i, dg = tid & 31;
            // 4 keys x 4 d  ->  4 d-rows x 4 keys
            const uint32_t a0 = vreg[i][0].x, a1 = vreg[i][0].y, b0 = vreg[i][1].x, b1 = vreg[i][1].y;
            const uint32_t c0 = vreg[i][2].x, c1 = vreg[i][2].y, e0 = vreg[i][3].x, e1 = vreg[i][3].y;
            uint2 r0 = make_uint2((a0 & 0xffffu) | (b0 << 16), (c0 & 0xffffu) | (e0 << 16));          // d + 0
            uint2 r1 = make_uint2((a0 >> 16) | (b0 & 0xffff0000u), (c0 >> 16) | (e0 & 0xffff0000u));  // d + 1
            uint2 r2 = make_uint2((a1 & 0xffffu) | (b1 << 16), (c1 & 0xffffu) | (e1 << 16));          // d + 2
            uint2 r3 = make_uint2((a1 >> 16) | (b1 & 0xffff0000u), (c1 >> 16) | (e1 & 0xffff0000u));  // d + 3
            *reinterpret_cast<uint2*>(vs + vt_off(4 * dg + 0, kg)) = r0;
            *reinterpret_cast<uint2*>(vs + vt_off(4 * dg + 1, kg)) = r1;
            *reinterpret_cast<uint2*>(vs + vt_off(4 * dg + 2, kg)) = r2;
            *reinterpret_cast<uint2*>(vs + vt_off(4 * dg + 3, kg)) = r3;
        }
    };

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int last_q = min(q0 + BQ, n) - 1;
    const int n_kt = last_q / BKV + 1;                    // causal: tiles up to the last query's diagonal
    load_kv(0);
    store_kv(0);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const int k0 = kt * BKV;
        if (kt + 1 < n_kt) load_kv(k0 + BKV);
        if (k0 <= qw0 + 31) {                             // some key of the tile is visible to this wave
            const unsigned char* ks = lds + (kt & 1) * KV_STAGE_BYTES;
            const unsigned char* vs = ks + K_TILE_BYTES;
            // ---- S^T = K Q^T : two 32-key sub-tiles
            f32x16 s[2];
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) s[jt][v] = 0.f;
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + k_off(jt * 32 + l32, st * 2 + hh));
                    s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[jt], 0, 0, 0);
                }
            }
            // ---- mask + running max (log2 domain)
            const bool need_mask = (k0 + BKV - 1 > qw0) || (k0 + BKV > n);
            float tmax = -INFINITY;
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = s[jt][v] * scale_log2e;
                    if (need_mask) {
                        const int key = k0 + jt * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
                        if (key > qi || key >= n) x = -INFINITY;
                    }
                    s[jt][v] = x;
                    tmax = fmaxf(tmax, x);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m_run, tmax);       // finite: key 0 is visible to every query
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
            uint32_t pb[2][8];                            // P^T as bf16 pairs: [sub-tile][v/2]
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s[jt][v] - m_new);
                    const float p1 = __builtin_amdgcn_exp2f(s[jt][v + 1] - m_new);
                    psum += p0 + p1;
                    pb[jt][v >> 1] = pack_bf16x2(p0, p1);
                }
            l_run = l_run * alpha + psum;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
            // ---- O^T += V^T P^T : 4 k-steps of 16 keys; step (jt, half) uses accumulator values
            //      v = half*8 .. half*8+7 of sub-tile jt, i.e. keys jt*32 + half*16 + {4*hh+0..3, 8+4*hh+0..3}
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const uint4 pw = make_uint4(pb[jt][half * 4 + 0], pb[jt][half * 4 + 1], pb[jt][half * 4 + 2],
                                                pb[jt][half * 4 + 3]);
                    const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
                    const int u0 = jt * 8 + half * 4 + hh;       // 4-key unit of keys 4*hh.. ; second unit is +2
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        const int r = dt * 32 + l32;
                        const uint2 lo = *reinterpret_cast<const uint2*>(vs + vt_off(r, u0));
                        const uint2 hi = *reinterpret_cast<const uint2*>(vs + vt_off(r, u0 + 2));
                        const bf16x8 vf = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[dt], 0, 0, 0);
                    }
                }
        }
        if (kt + 1 < n_kt) store_kv((kt + 1) & 1);
        __syncthreads();
    }

    // ---- normalise and store: lane holds O[qi][h][dt*32 + 8*(v/4) + 4*hh + v%4]
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (qi < n) {
        bf16_t* orow = O + (size_t)qi * qstride + (size_t)h * AD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int d = dt * 32 + 8 * vg + 4 * hh;
                *reinterpret_cast<uint2*>(orow + d) =
                    make_uint2(pack_bf16x2(oacc[dt][vg * 4 + 0] * inv, oacc[dt][vg * 4 + 1] * inv),
                               pack_bf16x2(oacc[dt][vg * 4 + 2] * inv, oacc[dt][vg * 4 + 3] * inv));
            }
    }
}

// fp32 path (small fp32 workloads): one wave per (query, head).  Lanes split the keys, each keeps
// its own online-softmax state over its keys, and the 64 partial states are merged at the end.
template <int D>
__global__ void __launch_bounds__(64) attn_f32_kernel(const float* __restrict__ Q, const float* __restrict__ Kg,
                                                      const float* __restrict__ Vg, float* __restrict__ O, int n,
                                                      int Hq, int Hkv, float scale) {
    const int i = blockIdx.x, h = blockIdx.y, g = h / (Hq / Hkv), lane = threadIdx.x;
    __shared__ float qs[D];
    for (int c = lane; c < D; c += 64) qs[c] = Q[((size_t)i * Hq + h) * D + c];
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc[D];
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] = 0.f;
    for (int j = lane; j <= i; j += 64) {
        const float* kr = Kg + ((size_t)j * Hkv + g) * D;
        const float* vr = Vg + ((size_t)j * Hkv + g) * D;
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) s += qs[c] * kr[c];
        s *= scale;
        const float mn = fmaxf(m, s), a = expf(m - mn), p = expf(s - mn);
        l = l * a + p;
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] = acc[c] * a + p * vr[c];
        m = mn;
    }
    const float mall = wave_max(m);
    const float w = (m == -INFINITY) ? 0.f : expf(m - mall);
    const float lall = wave_sum(l * w);
#pragma unroll
    for (int c = 0; c < D; ++c) {
        const float t = wave_sum(acc[c] * w);
        if (lane == 0) O[((size_t)i * Hq + h) * D + c] = t / lall;
    }
}

int launch_attn(const void* q, const void* k, const void* v, int n, int Hq, int Hkv, int d, float scale,
                int dtype, void* out, hipStream_t st) {
    if (scale == 0.f) scale = 1.0f / sqrtf((float)d);
    if (dtype == SLIM_BF16) {
        static bool attr_done = false;
        const int smem = 2 * KV_STAGE_BYTES;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return set_hip_error(e);
            attr_done = true;
        }
        const int n_qt = (n + BQ - 1) / BQ;
        hipLaunchKernelGGL(attn_bf16_kernel, dim3(n_qt * Hq), dim3(256), smem, st, (const bf16_t*)q, (const bf16_t*)k,
                           (const bf16_t*)v, (bf16_t*)out, n, Hq, Hkv, scale * 1.4426950408889634f, n_qt);
        return check_launch();
    }
    dim3 grid(n, Hq);
#define SLIM_ATTN_F32(D) hipLaunchKernelGGL(attn_f32_kernel<D>, grid, dim3(64), 0, st, (const float*)q, \
        (const float*)k, (const float*)v, (float*)out, n, Hq, Hkv, scale)
    switch (d) {
        case 32: SLIM_ATTN_F32(32); break;
        case 64: SLIM_ATTN_F32(64); break;
        case 128: SLIM_ATTN_F32(128); break;
        default: return SLIM_UNSUPPORTED;
    }
#undef SLIM_ATTN_F32
    return check_launch();
}

}  // namespace slim
