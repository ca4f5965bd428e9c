// Causal grouped-query prefill attention ("Attention" stage of Fig. 2) over the compacted sequence.
//
// bf16 path (head_dim 128): flash-style single pass with online softmax, v_mfma_f32_32x32x16_bf16.
// A workgroup of 4 waves (one per SIMD) owns 256 queries of one head, each wave 64 of them as two 32-query
// sub-tiles that share every K and V^T fragment read from LDS.  K/V tiles of 128 keys go from global memory
// straight into LDS (global_load_lds_dwordx4), both row-major, two stages (2 x 64 KB); V fragments are read
// with the transposing LDS read (ds_read_b64_tr_b16).
//
// Both products are computed transposed so that no register shuffle is needed between them:
//   S^T[key, query] = K . Q^T      (A operand = K rows from LDS, B operand = Q rows held in registers)
//   O^T[d,   query] = V^T . P^T    (A operand = V^T from LDS, B operand = P^T from the S^T
//                                   accumulators, converted to bf16)
// In the 32x32 accumulator layout a lane owns one query column, so the softmax statistics of a query
// live in two lanes (l and l^32).  The accumulator's row order (rows 8*(v/4) + 4*(lane/32) + v%4) is a
// permutation of the keys; the V^T fragments are read in the same permuted order, which leaves the
// contraction unchanged.
//
// Softmax: Q is pre-multiplied by scale*log2(e) (bf16), logits are kept relative to a per-query reference that
// enters through the S accumulators' initial value, so P = exp2(acc) with no multiply or subtract per element;
// the reference is the row maximum of the first 32 keys and moves only when the P of a later 32-key unit add up to
// more than 2^8 in some lane (a logit may then lie more than 8 above the reference; seen before those P are used:
// the reference moves up to the unit's maximum, O and the row sums are rescaled, the unit's P are formed again),
// so the result does not depend on it.  Row sums add the unrounded P.
//
// The kernel body (main loop, instruction order, register assignment: O accumulators and Q fragments in
// a0-a191, S tiles and everything the vector ALU touches in v0-v231) is the assembly that gen_attn_asm.py writes
// into attn_bf16_body.inc; the C++ below computes its per-lane and per-workgroup operands.
#include "slim_common.h"
#include <mutex>

namespace slim {

constexpr int AD = 128;          // head_dim of the MFMA path
constexpr int ANW = 4;           // waves per workgroup
constexpr int BQ = 64 * ANW;     // queries per workgroup
constexpr int BKV = 128;         // keys per tile
constexpr int NSTAGE = 2;        // K/V tiles resident in LDS
constexpr int TILE_BYTES = BKV * AD * 2;
constexpr int STAGE_BYTES = 2 * TILE_BYTES;             // K tile, then V tile

// Both tiles: row = key, 256 B = 16 chunks of 16 B.  K: chunk c of row r sits at slot c ^ (r & 15), so
// the 128-bit fragment reads (32 rows, one chunk column) are conflict-free.  V: slot c ^ (4 * (r & 3)),
// which spreads the 4 key rows x 4 chunks that one transposing read touches over all banks.
__device__ __forceinline__ int k_off(int r, int c) { return (r * 16 + (c ^ (r & 15))) * 16; }
__device__ __forceinline__ int v_off(int r, int c) { return (r * 16 + (c ^ ((r & 3) << 2))) * 16; }

// GROUPED (4 query heads per kv head): the four waves of a workgroup take the same 64 queries of the four heads
// that share a kv head, so all of them stop at the same diagonal and no wave runs units that are masked for it
// alone.  Otherwise the waves take 4 x 64 consecutive queries of one head.
template <bool GROUPED>
__global__ void __launch_bounds__(64 * ANW) __attribute__((amdgpu_waves_per_eu(1, 1)))
attn_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kg, const bf16_t* __restrict__ Vg,
                 bf16_t* __restrict__ O, int n, int Hq, int Hkv, float scale_log2e, int n_qt) {
    extern __shared__ __align__(16) unsigned char lds[];
    // Workgroup -> (head, query tile).  Ids are dealt round-robin to the 8 XCDs and each XCD hands its
    // workgroups to its CUs in id order.  Give each XCD a contiguous range of heads, so the query heads
    // sharing a kv head meet in one L2, and walk that range's query tiles from the one with the most keys
    // down, all heads of the range at each size: longest-first order per XCD keeps its CUs evenly loaded.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;
    const int n_units = GROUPED ? Hkv : Hq;               // (kv heads | heads) that the grid walks per query tile
    int u, qt_idx;
    if (n_units % 8 == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, upx = n_units >> 3;
        u = xcd * upx + j % upx;
        qt_idx = n_qt - 1 - j / upx;
    } else {
        u = blockIdx.x % n_units;
        qt_idx = n_qt - 1 - blockIdx.x / n_units;
    }
    const int h = GROUPED ? u * 4 + wave : u;
    const int g = GROUPED ? u : h / (Hq / Hkv);
    constexpr int WGQ = GROUPED ? 64 : BQ;                // query rows per workgroup
    const int q0 = qt_idx * WGQ;
    const int qw0 = GROUPED ? q0 : q0 + wave * 64;        // first query of this wave
    const size_t qstride = (size_t)Hq * AD;
    const unsigned lds_base = (unsigned)(uintptr_t)lds;

    // LDS byte addresses of this lane's fragment reads for k-step 0 / d-tile 0 of stage 0; the others differ
    // by an XOR (k-step st: st << 5, d-tile dt: dt << 6, stage 1: 1 << 16) and an immediate offset per key row.
    // K fragment: row l32 of a 32-key sub-tile, chunk 2*st + hh.  V^T fragment (transposing read): in each group
    // of 16 lanes, lane s supplies the address of 4 consecutive d of key s/4 and receives, for d = D0 + s, the
    // 4 consecutive keys; lane groups 0/1 cover d 0-15 / 16-31, groups 2/3 the keys 4-7.
    const unsigned koff0 = lds_base + k_off(l32, hh);
    const int G4 = lane >> 4, sl = lane & 15;
    const int key_lane = 4 * (G4 >> 1) + (sl >> 2);
    const unsigned voff0 = lds_base + TILE_BYTES + v_off(key_lane, 2 * (G4 & 1) + ((sl & 3) >> 1)) + (sl & 1) * 8;
    // Tile loads: a wave-load moves 4 key rows x 256 B; wave-load i of this wave covers rows 16*i + r0 .., lane l
    // lands at LDS slot l%16 of row l/16 and fetches the global chunk that the swizzle assigns to that slot.
    const unsigned r0 = wave * 4 + (lane >> 4), slot = lane & 15;
    const unsigned kchunk = (slot ^ (r0 & 15)) * 16, vchunk = (slot ^ ((r0 & 3) << 2)) * 16;
    const int qi0 = qw0 + l32, qi1 = qw0 + 32 + l32;      // this lane's two queries
    const bf16_t* qrow0 = Q + (size_t)min(qi0, n - 1) * qstride + (size_t)h * AD + hh * 8;
    const bf16_t* qrow1 = Q + (size_t)min(qi1, n - 1) * qstride + (size_t)h * AD + hh * 8;
    bf16_t* orow0 = O + (size_t)qi0 * qstride + (size_t)h * AD + 4 * hh;     // written only when the query exists
    bf16_t* orow1 = O + (size_t)qi1 * qstride + (size_t)h * AD + 4 * hh;
    // causal / ragged mask: key k0 + ko of a unit is visible to the lane's accumulator row ko iff ko <= limabs - k0
    const int limabs0 = min(qi0, n - 1) - 4 * hh, limabs1 = min(qi1, n - 1) - 4 * hh;
    const unsigned valid0 = qi0 < n, valid1 = qi1 < n;

    const unsigned rowbytes = (unsigned)Hkv * AD * 2, tile_bytes = rowbytes * BKV;
    const unsigned last_tile = (n + BKV - 1) / BKV - 1;   // tiles past it re-read it (into a stage nobody reads)
    const unsigned nl = n - last_tile * BKV, nl1 = nl - 1; // rows of the last tile; its loads clamp their rows to nl1
    const unsigned last_ragged = nl != BKV ? last_tile : 0xffffffffu;
    const int last_q = min(q0 + WGQ, n) - 1;
    const unsigned nkt = last_q / BKV + 1;                // causal: tiles up to the last query's diagonal
    const unsigned nmain = nkt > 3 ? nkt - 3 : 0;         // tiles that need no mask
    const uint64_t kb = (uint64_t)(uintptr_t)(Kg + (size_t)g * AD), vb = (uint64_t)(uintptr_t)(Vg + (size_t)g * AD);
    const unsigned kbase_lo = (unsigned)kb, kbase_hi = (unsigned)(kb >> 32);
    const unsigned vbase_lo = (unsigned)vb, vbase_hi = (unsigned)(vb >> 32);
    const unsigned ldsw = lds_base + wave * 1024;

    asm volatile(
#include "attn_bf16_body.inc"
        :
        : [koff0] "v"(koff0), [voff0] "v"(voff0), [r0] "v"(r0), [kchunk] "v"(kchunk), [vchunk] "v"(vchunk),
          [qrow0] "v"(qrow0), [qrow1] "v"(qrow1), [orow0] "v"(orow0), [orow1] "v"(orow1),
          [limabs0] "v"(limabs0), [limabs1] "v"(limabs1), [valid0] "v"(valid0), [valid1] "v"(valid1),
          [kbase_lo] "s"(kbase_lo), [kbase_hi] "s"(kbase_hi), [vbase_lo] "s"(vbase_lo), [vbase_hi] "s"(vbase_hi),
          [nkt] "s"(nkt), [nmain] "s"(nmain), [last_tile] "s"(last_tile), [last_ragged] "s"(last_ragged),
          [rowbytes] "s"(rowbytes), [tile_bytes] "s"(tile_bytes), [scale] "s"(scale_log2e), [nl1] "s"(nl1),
          [ldsw] "s"(ldsw), [qw0] "s"(qw0)
        :
#include "attn_bf16_clobbers.inc"
    );
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
        // rowbytes and the 24-bit multiplies of the tile-load offsets bound the number of kv heads
        if ((long long)Hkv * AD * 2 * BKV >= (1ll << 31) || Hkv > 4096) return SLIM_UNSUPPORTED;
        const int smem = NSTAGE * STAGE_BYTES;
        static std::once_flag attr_once;
        static hipError_t attr_err = hipSuccess;
        std::call_once(attr_once, [&] {
            attr_err = hipFuncSetAttribute((const void*)attn_bf16_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (attr_err == hipSuccess)
                attr_err = hipFuncSetAttribute((const void*)attn_bf16_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        });
        if (attr_err != hipSuccess) return set_hip_error(attr_err);
        if (Hq == 4 * Hkv) {
            const int n_qt = (n + 63) / 64;
            hipLaunchKernelGGL(attn_bf16_kernel<true>, dim3(n_qt * Hkv), dim3(64 * ANW), smem, st, (const bf16_t*)q,
                               (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, n, Hq, Hkv, scale * 1.4426950408889634f, n_qt);
        } else {
            const int n_qt = (n + BQ - 1) / BQ;
            hipLaunchKernelGGL(attn_bf16_kernel<false>, dim3(n_qt * Hq), dim3(64 * ANW), smem, st, (const bf16_t*)q,
                               (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, n, Hq, Hkv, scale * 1.4426950408889634f, n_qt);
        }
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
