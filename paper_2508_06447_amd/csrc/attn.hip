// Causal grouped-query prefill attention ("Attention" stage of Fig. 2) over the compacted sequence.
//
// bf16 path (head_dim 128): flash-style single pass with online softmax, v_mfma_f32_32x32x16_bf16.
// A workgroup of 8 waves (two per SIMD) owns 256 queries of one head, each wave 32 of them.  K/V tiles
// of 128 keys go from global memory straight into LDS (global_load_lds_dwordx4), both row-major, double-
// buffered (2 x 64 KB); V fragments are read with the transposing LDS read (ds_read_b64_tr_b16).
//
// Both products are computed transposed so that no register shuffle is needed between them:
//   S^T[key, query] = K . Q^T      (A operand = K rows from LDS, B operand = Q rows held in VGPRs)
//   O^T[d,   query] = V^T . P^T    (A operand = V^T from LDS, B operand = P^T from the S^T
//                                   accumulators, converted to bf16 in place)
// In the 32x32 accumulator layout a lane owns one query column, so the softmax statistics of a query
// live in two lanes (l and l^32) and need a single cross-lane exchange per tile.  The accumulator's
// row order (rows 8*(v/4) + 4*(lane/32) + v%4) is a permutation of the keys; the V^T fragments are
// read in the same permuted order, which leaves the contraction unchanged.
#include "slim_common.h"

namespace slim {

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
#define SLIM_LDS_PTR(T, addr) ((__attribute__((address_space(3))) T*)(uintptr_t)(addr))

constexpr int AD = 128;          // head_dim of the MFMA path
constexpr int ANW = 8;           // waves per workgroup
constexpr int BQ = 32 * ANW;     // queries per workgroup
constexpr int BKV = 128;         // keys per tile
constexpr int NJ = BKV / 32;      // 32-key sub-tiles per tile
constexpr int NSTAGE = 2;        // K/V tiles resident in LDS
constexpr int TILE_BYTES = BKV * AD * 2;
constexpr int STAGE_BYTES = 2 * TILE_BYTES;             // K tile, then V tile

// Both tiles: row = key, 256 B = 16 chunks of 16 B.  K: chunk c of row r sits at slot c ^ (r & 15), so
// the 128-bit fragment reads (32 rows, one chunk column) are conflict-free.  V: slot c ^ (4 * (r & 3)),
// which spreads the 4 key rows x 4 chunks that one transposing read touches over all banks.
__device__ __forceinline__ int k_off(int r, int c) { return (r * 16 + (c ^ (r & 15))) * 16; }
__device__ __forceinline__ int v_off(int r, int c) { return (r * 16 + (c ^ ((r & 3) << 2))) * 16; }

__global__ void __launch_bounds__(64 * ANW) attn_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kg,
                                                             const bf16_t* __restrict__ Vg, bf16_t* __restrict__ O,
                                                             int n, int Hq, int Hkv, float scale_log2e, int n_qt) {
    extern __shared__ __align__(16) unsigned char lds[];
    // Workgroup -> (head, query tile).  Ids are dealt round-robin to the 8 XCDs and each XCD hands its
    // workgroups to its CUs in id order.  Give each XCD a contiguous range of heads, so the query heads
    // sharing a kv head meet in one L2, and walk that range's query tiles from the one with the most keys
    // down, all heads of the range at each size: longest-first order per XCD keeps its CUs evenly loaded.
    int h, qt_idx;
    if (Hq % 8 == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, hpx = Hq >> 3;
        h = xcd * hpx + j % hpx;
        qt_idx = n_qt - 1 - j / hpx;
    } else {
        h = blockIdx.x % Hq;
        qt_idx = n_qt - 1 - blockIdx.x / Hq;
    }
    const int g = h / (Hq / Hkv);
    const int q0 = qt_idx * BQ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hh = lane >> 5;
    const int qw0 = q0 + wave * 32;                       // first query of this wave
    const int qi = qw0 + l32;                             // this lane's query
    const size_t qstride = (size_t)Hq * AD, kvstride = (size_t)Hkv * AD;
    const unsigned lds_base = (unsigned)(uintptr_t)lds;

    // Q fragments (B operand): 8 k-steps x 8 bf16 of row qi, d = ks*16 + hh*8 .., multiplied by
    // softmax_scale * log2(e) once (rounded to bf16 again), so the MFMA result is the logit in the
    // base-2 domain and the softmax needs no multiply per element.
    bf16x8 qf[8];
    {
        const bf16_t* qrow = Q + (size_t)min(qi, n - 1) * qstride + (size_t)h * AD + hh * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            bf16x8 raw = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) raw[e] = (__bf16)((float)raw[e] * scale_log2e);
            qf[ks] = raw;
        }
    }

    // Tile t -> stage t % NSTAGE.  A wave-load moves 4 key rows x 256 B; each tile is BKV/4 wave-loads for
    // K and as many for V, spread evenly over the waves.  Lane l lands at LDS slot l%16 of row l/16, so it
    // fetches the global chunk that the swizzle assigns to that slot.  A load's address is a wave-uniform
    // base (first row of the tile, scalar registers) plus a loop-invariant per-lane byte offset; only the
    // last, ragged tile recomputes the offsets with its rows clamped to n-1.  Tiles past the end re-read
    // the last tile into a stage nobody reads, which keeps the count of loads in flight the same in
    // every iteration.
    const bf16_t* kbase = Kg + (size_t)g * AD;
    const bf16_t* vbase = Vg + (size_t)g * AD;
    const int n_kt_all = (n + BKV - 1) / BKV;
    constexpr int NLD = BKV / 4 / ANW;                    // wave-loads per wave per tile and operand
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    unsigned kofs[NLD], vofs[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int r = (i * ANW + uwave) * 4 + (lane >> 4), slot = lane & 15;
        kofs[i] = (unsigned)(((size_t)r * kvstride + (slot ^ (r & 15)) * 8) * 2);
        vofs[i] = (unsigned)(((size_t)r * kvstride + (slot ^ ((r & 3) << 2)) * 8) * 2);
    }
    auto issue_tile = [&](int t) {
        const int k0 = min(t, n_kt_all - 1) * BKV;
        const unsigned stage = lds_base + (t % NSTAGE) * STAGE_BYTES + uwave * 1024;
        const bf16_t* kt0 = kbase + (size_t)k0 * kvstride;
        const bf16_t* vt0 = vbase + (size_t)k0 * kvstride;
        if (k0 + BKV <= n) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                load_global_to_lds16(kt0, kofs[i], stage + i * ANW * 1024);
                load_global_to_lds16(vt0, vofs[i], stage + TILE_BYTES + i * ANW * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int r = (i * ANW + uwave) * 4 + (lane >> 4), slot = lane & 15;
                const size_t row = (size_t)(min(k0 + r, n - 1) - k0) * kvstride;
                load_global_to_lds16(kt0, (unsigned)((row + (slot ^ (r & 15)) * 8) * 2), stage + i * ANW * 1024);
                load_global_to_lds16(vt0, (unsigned)((row + (slot ^ ((r & 3) << 2)) * 8) * 2),
                                     stage + TILE_BYTES + i * ANW * 1024);
            }
        }
    };

    // Per-lane LDS byte offsets inside a stage (loop-invariant); tile rows are added as immediates.
    unsigned koff[8], voff[4];
#pragma unroll
    for (int st = 0; st < 8; ++st) koff[st] = k_off(l32, st * 2 + hh);
    {
        // Transposing read: in each group of 16 lanes, lane s supplies the address of 4 consecutive d of
        // key (s/4) and receives, for d = D0 + s, the 4 consecutive keys.  Lane groups 0/1 cover d 0-15 /
        // 16-31 of the fragment, groups 2/3 the keys 4-7 (the accumulator rows owned by lanes 32-63).
        const int G = lane >> 4, sl = lane & 15;
        const int key_lane = 4 * (G >> 1) + (sl >> 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            voff[dt] = TILE_BYTES + v_off(key_lane, dt * 4 + 2 * (G & 1) + ((sl & 3) >> 1)) + (sl & 1) * 8;
    }

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    // Softmax state.  Logits are kept relative to a reference r per query: the S^T accumulators start
    // from -r (negr, one value splat over the tile), so the MFMAs deliver s - r and P = exp2(s - r)
    // needs no subtraction.  r is the row maximum of the first tile and moves only when a later logit
    // exceeds it by more than REF_SLACK (then O and l are rescaled), so P <= 2^REF_SLACK; the final
    // O / l does not depend on r.
    constexpr float REF_SLACK = 8.0f;
    float ref = 0.f, l_run = 0.f;
    f32x16 negr;
#pragma unroll
    for (int v = 0; v < 16; ++v) negr[v] = 0.f;

    const int last_q = min(q0 + BQ, n) - 1;
    const int n_kt = last_q / BKV + 1;                    // causal: tiles up to the last query's diagonal
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t) issue_tile(t);
    __builtin_amdgcn_s_waitcnt(0x0070);                   // vmcnt(0) lgkmcnt(0)
    workgroup_barrier();

    for (int kt = 0; kt < n_kt; ++kt) {
        const int k0 = kt * BKV;
        issue_tile(kt + NSTAGE - 1);                      // its stage held tile kt-1, which every wave has left
        if (k0 <= qw0 + 31) {                             // some key of the tile is visible to this wave
            const unsigned sb = lds_base + (kt % NSTAGE) * STAGE_BYTES;
            // ---- S^T - r = K Q^T - r : NJ 32-key sub-tiles.  Fragment f = (k-step st, sub-tile jt) is
            //      read KAHEAD MFMAs before its use (the compiler, left alone, reads each fragment right
            //      before its MFMA and waits for it); consecutive MFMAs go to different accumulators.
            f32x16 s[NJ];
            {
                constexpr int NF = 8 * NJ, KAHEAD = 3;
                bf16x8 kf[KAHEAD + 1];
                auto ldk = [&](int f) {
                    return *(SLIM_LDS_PTR(const bf16x8, sb + koff[f / NJ]) + (f % NJ) * (32 * 256 / 16));
                };
#pragma unroll
                for (int f = 0; f < KAHEAD; ++f) kf[f] = ldk(f);
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    const int st = f / NJ, jt = f % NJ;
                    if (f + KAHEAD < NF) kf[(f + KAHEAD) % (KAHEAD + 1)] = ldk(f + KAHEAD);
                    __builtin_amdgcn_sched_barrier(0);
                    s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[f % (KAHEAD + 1)], qf[st], st == 0 ? negr : s[jt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // ---- causal / ragged mask (selects only; the branch is wave-uniform)
            if ((k0 + BKV - 1 > qw0) || (k0 + BKV > n)) {
                const int lim = min(qi, n - 1) - k0 - 4 * hh;     // visible: key offset in the tile <= lim
#pragma unroll
                for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        s[jt][v] = (jt * 32 + 8 * (v >> 2) + (v & 3)) > lim ? -INFINITY : s[jt][v];
            }
            // ---- row maximum relative to the reference; move the reference if it is exceeded by too much
            float tmax = -INFINITY;
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int v = 0; v < 16; v += 2) tmax = fmaxf(fmaxf(tmax, s[jt][v]), s[jt][v + 1]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const bool first = kt == 0;                   // every wave computes tile 0, where key 0 is visible
            if (first || __any(tmax > REF_SLACK)) {
                const float delta = first ? tmax : fmaxf(tmax, 0.f);
                ref += delta;
#pragma unroll
                for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) s[jt][v] -= delta;
#pragma unroll
                for (int v = 0; v < 16; ++v) negr[v] = -ref;
                if (!first) {
                    const float alpha = __builtin_amdgcn_exp2f(-delta);
                    l_run *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
                }
            }
            // ---- P = exp2(s - r), rounded to bf16 for the MFMA; the row sum adds the rounded values
            uint32_t pb[NJ][8];
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const f32x2 p = {__builtin_amdgcn_exp2f(s[jt][v]), __builtin_amdgcn_exp2f(s[jt][v + 1])};
                    const bf16x2 p2 = __builtin_convertvector(p, bf16x2);
                    l_run = __builtin_amdgcn_fdot2_f32_bf16(p2, ones, l_run, false);
                    pb[jt][v >> 1] = __builtin_bit_cast(uint32_t, p2);
                }
            // ---- O^T += V^T P^T : 2*NJ k-steps of 16 keys; step (jt, half) uses accumulator values
            //      v = half*8 .. half*8+7 of sub-tile jt, i.e. keys jt*32 + half*16 + {4*hh+0..3, 8+4*hh+0..3}
            //      Fragment g = (step, dt) is read VAHEAD MFMAs ahead, like the K fragments.
            {
                constexpr int ROW = 256 / 8;              // one key row in units of 8 bytes
                constexpr int NG = 8 * NJ, VAHEAD = 3;
                i16x4 vlo[VAHEAD + 1], vhi[VAHEAD + 1];
                auto ldv = [&](int g) {
                    const int r0 = (g >> 2) * 16 * ROW, b = g % (VAHEAD + 1);
                    vlo[b] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SLIM_LDS_PTR(i16x4, sb + voff[g & 3]) + r0);
                    vhi[b] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SLIM_LDS_PTR(i16x4, sb + voff[g & 3]) + r0 + 8 * ROW);
                };
#pragma unroll
                for (int g = 0; g < VAHEAD; ++g) ldv(g);
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const int step = g >> 2, jt = step >> 1, half = step & 1, dt = g & 3;
                    if (g + VAHEAD < NG) ldv(g + VAHEAD);
                    __builtin_amdgcn_sched_barrier(0);
                    const bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pb[jt][half * 4 + 0], pb[jt][half * 4 + 1],
                                                                            pb[jt][half * 4 + 2], pb[jt][half * 4 + 3]));
                    const uint2 lo2 = __builtin_bit_cast(uint2, vlo[g % (VAHEAD + 1)]);
                    const uint2 hi2 = __builtin_bit_cast(uint2, vhi[g % (VAHEAD + 1)]);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[dt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // Tile kt+1 has landed for this wave (the newer tile's loads may stay in flight); its own LDS
        // reads are done; after the barrier that holds for every wave.
        __builtin_amdgcn_s_waitcnt(0x0070 | ((BKV / 2 / ANW) * (NSTAGE - 2)));
        workgroup_barrier();
    }
    __builtin_amdgcn_s_waitcnt(0x0070);                   // drain the trailing loads before the wave ends

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
        const int smem = NSTAGE * STAGE_BYTES;
        if (!attr_done) {
            hipError_t e = hipFuncSetAttribute((const void*)attn_bf16_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return set_hip_error(e);
            attr_done = true;
        }
        const int n_qt = (n + BQ - 1) / BQ;
        hipLaunchKernelGGL(attn_bf16_kernel, dim3(n_qt * Hq), dim3(64 * ANW), smem, st, (const bf16_t*)q, (const bf16_t*)k,
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
