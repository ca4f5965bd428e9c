// Dense projections of the layer ("QKV Generation", output projection and FFN of Fig. 2):
//   out[m, n] = sum_k a[m, k] * w[n, k]            (both operands contiguous along k)
// with five epilogues: plain, + bias[n] (Q/K/V projections of models that have one), + residual,
// SwiGLU (two weight matrices, silu(gate) * up), and RoPE (+ bias, + per-token score partials) for the
// Query/Key projections of 128-wide heads.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The weight tile is the MFMA "A" operand
// and the activation tile the "B" operand, so a lane ends up with 4 consecutive output features of
// one token and stores them as one 8-byte vector.
//
// Main path (k_in a multiple of 64, more than 128 rows): 4 waves per workgroup, one per SIMD, 256x256 output tile
// (128 features x 2 matrices x 256 tokens for SwiGLU), each wave 128 x 128 of it, so that every MFMA fragment read
// from LDS feeds four MFMAs.  Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
// VGPR staging), double-buffered; MFMA fragments are read one k-step ahead of their use, across k-tiles too.  The
// k-loop is generated assembly (gen_gemm_asm.py -> gemm_bf16_mainloops.inc): with a lone wave per SIMD the order of
// MFMA, LDS and tile-load instructions inside the wave is the schedule.  The residual epilogue (output and down
// projection) and few rows (<= 128, narrow tiles) use an 8-wave C++ tile with the same LDS layout and pipeline; a
// register-staged kernel with k predicates covers ragged k_in.
#include "slim_common.h"

#include <map>
#include <mutex>
#include <queue>
#include <tuple>
#include <type_traits>
#include <vector>

namespace slim {

enum { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_BIAS = 3, EPI_ROPE = 4 };
// EPI_BIAS: R is a bias vector [N].  EPI_ROPE: R is a bias vector or null, the rest comes in a EpiExtra.

// Extra operands: of the RoPE epilogue (heads of 128 features, one head per wave tile), of the fused RMSNorm, and
// of a second projection of the same rows carried by the same launch.
struct EpiExtra {
    const float* table = nullptr;        // [M][128]: cos of the 64 rotation angles of the token, then their sin
    const float* qt = nullptr;           // [N] float or null: head-group-summed window query (Eq. 2 by linearity)
    float* token_scores = nullptr;       // [M][N/128]: rotated, rounded key of (token, head) dotted with its part of qt
    const float* row_scale = nullptr;    // [M] float or null: out row m = row_scale[m] * (a[m,:] . w^T) (fused RMSNorm)
    // Second projection (two-size launch only): feature tiles tiles_n1.. belong to it.
    const bf16_t* w_2 = nullptr;         // [n_2][K]
    const bf16_t* r_2 = nullptr;         // its bias (EPI_BIAS)
    bf16_t* c_2 = nullptr;               // [M][ldo_2]
    int n_2 = 0, ldo_2 = 0, tiles_n1 = 0;
};

constexpr int BK = 64;                                   // k-depth of an LDS tile (8 chunks of 16 bytes)

// LDS tile: rows of 64 bf16 = 8 chunks of 16 B; chunk c of row r lives at chunk slot c ^ swz(r),
// so that the 16 lanes served together by a 128-bit LDS read hit distinct banks.
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }
__device__ __forceinline__ int lds_off(int r, int c) { return (r * 8 + (c ^ swz(r))) * 16; }   // bytes

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
#include "gemm_bf16_mainloops.inc"
#pragma clang diagnostic pop

// Epilogue shared by both bf16 kernels.  acc[w][i][j][v] is out[token m][feature n] with
//   m = mw + j*32 + l32,   n = nw + i*32 + 8*(v/4) + 4*hh + (v%4)      (mw, nw: the wave's origin)
template <int TW, int TA, int EPI>
__device__ __forceinline__ void store_tile(f32x16 (&acc)[EPI == EPI_SWIGLU ? 2 : 1][TW][TA], const bf16_t* R,
                                           bf16_t* C, int ldo, int M, int N, int mw, int nw, int l32, int hh) {
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    const bool vec_ok = (N % 4 == 0) && (ldo % 4 == 0);
#pragma unroll
    for (int j = 0; j < TA; ++j) {
        const int m = mw + j * 32 + l32;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < TW; ++i) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int n = nw + i * 32 + 8 * vg + 4 * hh;
                if (n >= N) continue;
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (EPI == EPI_SWIGLU) {
                        const float g = acc[0][i][j][vg * 4 + e], u = acc[NW - 1][i][j][vg * 4 + e];
                        o[e] = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;   // v_rcp_f32: 1 ulp, the result is rounded to bf16
                    } else {
                        o[e] = acc[0][i][j][vg * 4 + e];
                    }
                }
                bf16_t* dst = C + (size_t)m * ldo + n;
                if (vec_ok) {
                    if (EPI == EPI_RESIDUAL || EPI == EPI_BIAS) {
                        const uint2 r = *reinterpret_cast<const uint2*>(EPI == EPI_BIAS ? R + n : R + (size_t)m * ldo + n);
                        o[0] += lo_bf16(r.x); o[1] += hi_bf16(r.x); o[2] += lo_bf16(r.y); o[3] += hi_bf16(r.y);
                    }
                    *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (n + e < N) {
                            float val = o[e];
                            if (EPI == EPI_RESIDUAL) val += bf16_to_f32(R[(size_t)m * ldo + n + e]);
                            if (EPI == EPI_BIAS) val += bf16_to_f32(R[n + e]);
                            dst[e] = f32_to_bf16(val);
                        }
                    }
                }
            }
        }
    }
}

// Epilogue of the main kernel: the wave's tile goes through a wave-private LDS region so that global
// traffic is 16 bytes per lane and whole rows of the tile are contiguous (a lane of the accumulator
// layout owns only 4 consecutive features of one token).  Steps, all inside one wave (LDS operations
// of a wave complete in program order, so no barrier is needed):
//   residual only: rows of R are loaded coalesced and parked in the region;
//   each lane takes its accumulators, applies SiLU(gate)*up or adds its 4 residual values in fp32,
//   rounds once to bf16 and writes 8 bytes into the region;
//   rows are read back 16 bytes per lane and stored.
// Region layout: row = token (TA*32 rows of TW*64 bytes), 16-byte chunk c of row r at slot
// c ^ (r & (chunks per row - 1)).  Needs N % 8 == 0, ldo % 8 == 0 and 16-byte aligned out / residual.
template <int TW, int TA, int EPI>
__device__ __forceinline__ void store_tile_via_lds(f32x16 (&acc)[EPI == EPI_SWIGLU ? 2 : 1][TW][TA], const bf16_t* R,
                                                   bf16_t* C, int ldo, int M, int N, int mw, int nw, int lane,
                                                   unsigned char* region) {
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int CPR = TW * 4, RB = TW * 64, ROWS = TA * 32, RPI = 64 / CPR;
    const int l32 = lane & 31, hh = lane >> 5;
    const int rrow = lane / CPR, rchunk = lane % CPR;     // coalesced phases: lane -> (row in group, chunk)
    auto slot = [&](int row, int chunk) { return row * RB + ((chunk ^ (row & (CPR - 1))) << 4); };
    if (EPI == EPI_RESIDUAL) {
#pragma unroll
        for (int it = 0; it < ROWS / RPI; ++it) {
            const int row = it * RPI + rrow, m = mw + row, n = nw + rchunk * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < M && n < N) v = *reinterpret_cast<const uint4*>(R + (size_t)m * ldo + n);
            *reinterpret_cast<uint4*>(region + slot(row, rchunk)) = v;
        }
    }
    uint2 bias4[EPI == EPI_BIAS ? TW * 4 : 1];            // the lane's bias values, requested together
    if (EPI == EPI_BIAS) {
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int n = nw + i * 32 + 8 * vg + 4 * hh;
                bias4[i * 4 + vg] = n < N ? *reinterpret_cast<const uint2*>(R + n) : make_uint2(0, 0);
            }
    }
#pragma unroll
    for (int j = 0; j < TA; ++j)
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int row = j * 32 + l32;
                uint2* cell = reinterpret_cast<uint2*>(region + slot(row, i * 4 + vg) + hh * 8);
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (EPI == EPI_SWIGLU) {
                        const float g = acc[0][i][j][vg * 4 + e], u = acc[NW - 1][i][j][vg * 4 + e];
                        o[e] = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;   // v_rcp_f32: 1 ulp, the result is rounded to bf16
                    } else {
                        o[e] = acc[0][i][j][vg * 4 + e];
                    }
                }
                if (EPI == EPI_RESIDUAL) {
                    const uint2 r = *cell;
                    o[0] += lo_bf16(r.x); o[1] += hi_bf16(r.x); o[2] += lo_bf16(r.y); o[3] += hi_bf16(r.y);
                }
                if (EPI == EPI_BIAS) {                    // 4 consecutive features of the bias vector (N % 8 == 0 here)
                    const uint2 r = bias4[EPI == EPI_BIAS ? i * 4 + vg : 0];
                    o[0] += lo_bf16(r.x); o[1] += hi_bf16(r.x); o[2] += lo_bf16(r.y); o[3] += hi_bf16(r.y);
                }
                *cell = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
            }
#pragma unroll
    for (int it = 0; it < ROWS / RPI; ++it) {
        const int row = it * RPI + rrow, m = mw + row, n = nw + rchunk * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(region + slot(row, rchunk));
        if (m < M && n < N) *reinterpret_cast<uint4*>(C + (size_t)m * ldo + n) = v;
    }
}

// RoPE epilogue.  The wave tile is 128 features wide and starts at a multiple of 128, so it is one head and the
// rotate-half partner of feature f < 64 (sub-tile i = 0, 1) is the same accumulator element of sub-tile i + 2 in
// the same lane: the rotation needs no exchange.  out[f] = x[f] cos - x[f+64] sin, out[f+64] = x[f+64] cos +
// x[f] sin with the angle of (token, f) from the table; x includes the bias.  One rounding to bf16.  With a
// window query, the rounded values are dotted with it (64 of the head's features per lane, the other half in
// lane ^ 32) and the per-(token, head) partial goes to token_scores.
template <int TA>
__device__ __forceinline__ void store_tile_rope(f32x16 (&acc)[1][4][TA], const bf16_t* bias, bf16_t* C, int ldo, int M,
                                                int N, int mw, int nw, int lane, unsigned char* region,
                                                const EpiExtra& re) {
    constexpr int TW = 4, CPR = TW * 4, RB = TW * 64, ROWS = TA * 32, RPI = 64 / CPR;
    if (nw >= N) return;                                 // wave-uniform: no head here (N is a multiple of 128)
    const int l32 = lane & 31, hh = lane >> 5;
    const int rrow = lane / CPR, rchunk = lane % CPR;
    auto slot = [&](int row, int chunk) { return row * RB + ((chunk ^ (row & (CPR - 1))) << 4); };
    const bool score = re.qt != nullptr;
    float dot[TA];
#pragma unroll
    for (int j = 0; j < TA; ++j) dot[j] = 0.f;
    // Per half of the head's rotation indices (i), every table, bias and window-query value the lane needs is requested
    // first and used afterwards: 8 * TA + 16 loads in flight, one wait.  (Left to the compiler, the loads went out two
    // at a time, each pair waited for: forty memory round trips per tile.)
    const float* trow0[TA];
#pragma unroll
    for (int j = 0; j < TA; ++j) trow0[j] = re.table + (size_t)min(mw + j * 32 + l32, M - 1) * 128 + 4 * hh;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        float4 c4[4][TA], s4[4][TA], q1[4], q2[4];
        uint2 r1[4], r2[4];
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const int f = i * 32 + 8 * vg + 4 * hh;      // rotation index of element e = 0
#pragma unroll
            for (int j = 0; j < TA; ++j) {
                c4[vg][j] = *reinterpret_cast<const float4*>(trow0[j] + i * 32 + 8 * vg);
                s4[vg][j] = *reinterpret_cast<const float4*>(trow0[j] + i * 32 + 8 * vg + 64);
            }
            r1[vg] = r2[vg] = make_uint2(0, 0);
            if (bias) {
                r1[vg] = *reinterpret_cast<const uint2*>(bias + nw + f);
                r2[vg] = *reinterpret_cast<const uint2*>(bias + nw + 64 + f);
            }
            q1[vg] = q2[vg] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (score) {
                q1[vg] = *reinterpret_cast<const float4*>(re.qt + nw + f);
                q2[vg] = *reinterpret_cast<const float4*>(re.qt + nw + 64 + f);
            }
        }
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const float b1[4] = {lo_bf16(r1[vg].x), hi_bf16(r1[vg].x), lo_bf16(r1[vg].y), hi_bf16(r1[vg].y)};
            const float b2[4] = {lo_bf16(r2[vg].x), hi_bf16(r2[vg].x), lo_bf16(r2[vg].y), hi_bf16(r2[vg].y)};
#pragma unroll
            for (int j = 0; j < TA; ++j) {
                const int row = j * 32 + l32;
                const float c[4] = {c4[vg][j].x, c4[vg][j].y, c4[vg][j].z, c4[vg][j].w};
                const float sn[4] = {s4[vg][j].x, s4[vg][j].y, s4[vg][j].z, s4[vg][j].w};
                float o1[4], o2[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x1 = acc[0][i][j][vg * 4 + e] + b1[e], x2 = acc[0][i + 2][j][vg * 4 + e] + b2[e];
                    o1[e] = x1 * c[e] - x2 * sn[e];
                    o2[e] = x2 * c[e] + x1 * sn[e];
                }
                const uint2 p1 = make_uint2(pack_bf16x2(o1[0], o1[1]), pack_bf16x2(o1[2], o1[3]));
                const uint2 p2 = make_uint2(pack_bf16x2(o2[0], o2[1]), pack_bf16x2(o2[2], o2[3]));
                *reinterpret_cast<uint2*>(region + slot(row, i * 4 + vg) + hh * 8) = p1;
                *reinterpret_cast<uint2*>(region + slot(row, (i + 2) * 4 + vg) + hh * 8) = p2;
                if (score)
                    dot[j] += lo_bf16(p1.x) * q1[vg].x + hi_bf16(p1.x) * q1[vg].y + lo_bf16(p1.y) * q1[vg].z + hi_bf16(p1.y) * q1[vg].w +
                              lo_bf16(p2.x) * q2[vg].x + hi_bf16(p2.x) * q2[vg].y + lo_bf16(p2.y) * q2[vg].z + hi_bf16(p2.y) * q2[vg].w;
            }
        }
    }
    if (score) {
#pragma unroll
        for (int j = 0; j < TA; ++j) {
            const float tot = dot[j] + __shfl_xor(dot[j], 32, 64);
            const int m = mw + j * 32 + l32;
            if (hh == 0 && m < M) re.token_scores[(size_t)m * (N >> 7) + (nw >> 7)] = tot;
        }
    }
#pragma unroll
    for (int it = 0; it < ROWS / RPI; ++it) {
        const int row = it * RPI + rrow, m = mw + row, n = nw + rchunk * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(region + slot(row, rchunk));
        if (m < M && n < N) *reinterpret_cast<uint4*>(C + (size_t)m * ldo + n) = v;
    }
}

// Workgroup -> output tile.  Workgroup ids are dealt round-robin to the 8 XCDs, so each XCD gets a
// contiguous run of logical tiles; inside the run, bands of GM token-tiles are walked feature-tile by
// feature-tile, so the workgroups resident on one XCD share few distinct operand tiles in its L2 (GM = 8: 32
// resident tiles are 8 x 4, the fewest panels; GM = 2 reads each activation panel in one go, see the residual kernel).
// L is the workgroup's index inside a region of tiles_m x tiles_n tiles that starts at a workgroup id
// divisible by 8 when xcd_runs is set.
__device__ __forceinline__ void tile_of_workgroup(int L, bool xcd_runs, int tiles_m, int tiles_n, int& tm, int& tn,
                                                  int GM = 8) {
    const int total = tiles_m * tiles_n;
    if (xcd_runs && total % 8 == 0) L = (L & 7) * (total >> 3) + (L >> 3);
    const int band_sz = GM * tiles_n;
    const int band = L / band_sz;
    const int gm = min(GM, tiles_m - band * GM);
    const int rem = L - band * band_sz;
    tm = band * GM + rem % gm;
    tn = rem / gm;
}

// One output tile of the few-row kernel.  8 waves arranged WGN x WGM; requires K % 64 == 0 and 16-byte aligned
// rows.  The tile starts at token m0, feature n0; M and N bound the loads (clamped) and the stores.
// With re.row_scale the accumulators of token row m are multiplied by row_scale[m] before the epilogue: with
// row_scale = 1/sqrt(mean(a[m,:]^2) + eps) and a = the raw residual stream this is the projection of RMSNorm(a)
// (unit gain; a gain vector is folded into the weights beforehand), and the normalised rows are never stored.
template <int TW, int TA, int WGN, int WGM, int EPI>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W0,
                                          const bf16_t* __restrict__ W1, const bf16_t* R, bf16_t* C, int ldo, int M,
                                          int N, int K, int m0, int n0, unsigned char* lds, const EpiExtra& re) {
    static_assert(WGN * WGM == 8, "8 waves");
    static_assert(EPI != EPI_ROPE || TW == 4, "the RoPE epilogue needs one 128-wide head per wave");
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int BN = 32 * TW * WGN, BM = 32 * TA * WGM, WROWS = BN * NW;
    constexpr int STAGE = (WROWS + BM) * BK * 2;
    constexpr int WLD = WROWS / 64, ALD = BM / 64;       // wave-loads per k-tile per wave (8 rows each)
    static_assert(WLD * 64 == WROWS && ALD * 64 == BM && BN % 64 == 0, "tile rows must split over 8 waves x 8 rows");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % WGN, wm = wave / WGN;
    const int l32 = lane & 31, hh = lane >> 5;

    // Wave-load i covers rows (i*8 + wave)*8 + lane/8 of the tile; lane%8 is the LDS chunk slot, which
    // holds logical chunk slot ^ swz(row).  A load's address is a wave-uniform base (start of the tile's
    // rows + k offset, scalar registers) plus a loop-invariant per-lane byte offset inside the tile, so
    // the k-loop spends no vector instruction on addresses (a tile spans at most 256 rows: 32 bits do).
    unsigned woff[WLD], aoff[ALD];
#pragma unroll
    for (int i = 0; i < WLD; ++i) {
        const int r = (i * 8 + wave) * 8 + (lane >> 3);
        const int mat = NW == 2 ? r / BN : 0;
        const int n = min(n0 + r - mat * BN, N - 1) - n0;
        woff[i] = (unsigned)(((size_t)n * K + ((lane & 7) ^ swz(r)) * 8) * 2);
    }
#pragma unroll
    for (int i = 0; i < ALD; ++i) {
        const int r = (i * 8 + wave) * 8 + (lane >> 3);
        aoff[i] = (unsigned)(((size_t)(min(m0 + r, M - 1) - m0) * lda + ((lane & 7) ^ swz(r)) * 8) * 2);
    }
    const bf16_t* w0base = W0 + (size_t)n0 * K;
    const bf16_t* w1base = NW == 2 ? W1 + (size_t)n0 * K : W0;
    const bf16_t* abase = A + (size_t)m0 * lda;
    const unsigned lds_wave = (unsigned)(uintptr_t)lds + wave * 1024;
    auto issue_loads = [&](int k0, int stage) {
        const unsigned ws = lds_wave + stage * STAGE, as = ws + WROWS * BK * 2;
#pragma unroll
        for (int i = 0; i < WLD; ++i) {
            const bool second = NW == 2 && (i * 8 * 8 >= BN);   // rows of wave-load i lie in one matrix (BN % 64 == 0)
            load_global_to_lds16((second ? w1base : w0base) + k0, woff[i], ws + i * 8 * 1024);
        }
#pragma unroll
        for (int i = 0; i < ALD; ++i) load_global_to_lds16(abase + k0, aoff[i], as + i * 8 * 1024);
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

    const int KT = K / BK;
    bf16x8 af[2][TA], wf[2][NW][TW];
    // Fragment addresses: one per-lane base per (operand, stage, k-step), computed once; the MFMA tile
    // (i, j) and the matrix (gate/up) are immediate offsets of the LDS reads, so the k-loop spends no
    // vector instruction on them.  The swizzle term (row >> 1) & 7 depends only on lane % 32 because the
    // tile rows of a wave start at multiples of 32.
    const unsigned char* wfrag[2][BK / 16];
    const unsigned char* afrag[2][BK / 16];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            wfrag[st][ks] = lds + st * STAGE + lds_off(wn * TW * 32 + l32, ks * 2 + hh);
            afrag[st][ks] = lds + st * STAGE + WROWS * BK * 2 + lds_off(wm * TA * 32 + l32, ks * 2 + hh);
        }
    auto load_frags = [&](auto stage_c, int ks, int buf) {
        constexpr int stage = decltype(stage_c)::value;
#pragma unroll
        for (int j = 0; j < TA; ++j)
            af[buf][j] = *reinterpret_cast<const bf16x8*>(afrag[stage][ks] + j * 32 * BK * 2);
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int i = 0; i < TW; ++i)
                wf[buf][w][i] = *reinterpret_cast<const bf16x8*>(wfrag[stage][ks] + (w * BN + i * 32) * BK * 2);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int i = 0; i < TW; ++i)
#pragma unroll
                for (int j = 0; j < TA; ++j)
                    acc[w][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][w][i], af[buf][j], acc[w][i][j], 0, 0, 0);
    };
    // Two LDS stages.  Fragments are read one k-step ahead of their MFMAs, also across k-tiles: the
    // workgroup barrier of a k-tile sits before its last k-step, when every wave has pulled that step's
    // fragments into registers.  Past the barrier the stage is free, so tile kt+2 is sent into it, tile
    // kt+1 (sent one iteration earlier, waited for just before the barrier) is visible to all waves, and
    // its first fragments are read while the last k-step's MFMAs run.  The loop is unrolled by two so the
    // stage of every read is a compile-time constant.
    using Stage0 = std::integral_constant<int, 0>;
    using Stage1 = std::integral_constant<int, 1>;
    auto k_tile = [&](int kt, auto stage_c, auto other_c) {
        constexpr int stage = decltype(stage_c)::value;
#pragma unroll
        for (int ks = 0; ks < BK / 16 - 1; ++ks) {
            load_frags(stage_c, ks + 1, (ks + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);           // keep the next step's LDS reads ahead of these MFMAs
            mfmas(ks & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_waitcnt(0x0070);              // own reads of this stage and own part of tile kt+1 done
        workgroup_barrier();
        if (kt + 2 < KT) issue_loads((kt + 2) * BK, stage);
        if (kt + 1 < KT) load_frags(other_c, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas((BK / 16 - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    issue_loads(0, 0);
    if (KT > 1) {
        // only the first k-tile has to be there; the second stays in flight until the first k-tile's own wait
        constexpr unsigned kStageLoads = WLD + ALD;
        issue_loads(BK, 1);
        __builtin_amdgcn_s_waitcnt((kStageLoads & 15) | 0x0070 | ((kStageLoads >> 4) << 14));
    } else {
        __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0) lgkmcnt(0)
    }
    workgroup_barrier();
    load_frags(Stage0{}, 0, 0);
    for (int kt = 0; kt < KT; kt += 2) {
        k_tile(kt, Stage0{}, Stage1{});
        if (kt + 1 < KT) k_tile(kt + 1, Stage1{}, Stage0{});
    }
    if (re.row_scale) {
        float inv[TA];                                   // all requested before the first is used: one wait, not TA
#pragma unroll
        for (int j = 0; j < TA; ++j) inv[j] = re.row_scale[min(m0 + (wm * TA + j) * 32 + l32, M - 1)];
#pragma unroll
        for (int j = 0; j < TA; ++j)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < TW; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[w][i][j][v] *= inv[j];
    }
    // The epilogue reuses the stage buffers: every wave must be past its last fragment reads.
    __builtin_amdgcn_s_waitcnt(0x0070);
    workgroup_barrier();
    const bool wide = (N % 8 == 0) && (ldo % 8 == 0) && (((uintptr_t)C & 15) == 0) &&
                      (EPI != EPI_RESIDUAL || ((uintptr_t)R & 15) == 0) && (EPI != EPI_BIAS || ((uintptr_t)R & 7) == 0);
    if constexpr (EPI == EPI_ROPE) {                     // the launcher has checked what `wide` checks
        store_tile_rope<TA>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, lane,
                            lds + wave * (TA * 32 * TW * 64), re);
    } else {
        if (wide)
            store_tile_via_lds<TW, TA, EPI>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, lane,
                                            lds + wave * (TA * 32 * TW * 64));
        else
            store_tile<TW, TA, EPI>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, l32, hh);
    }
}

// One output tile of the main path: 4 waves arranged 2 (features) x 2 (tokens), each with TW x TA MFMA tiles (of
// each weight matrix); requires K % 64 == 0, 16-byte aligned rows and row strides below 2^23 elements.  The k-loop
// is gemm_mainloop_<TW>_<TA>_<NW>; its operands:
//   wfrag0 / afrag0   LDS byte address of the lane's weight / activation fragment of k-step 0 in stage 0;
//   r0, chunk         the lane's row inside a group of 32 tile rows and its (swizzled) 16-byte chunk of a 128-byte
//                     row: wave-load i of a k-tile covers tile rows 32 i + r0 and lands at ldsw + i * 4096;
//   wlim / alim       last valid row of the tile (loads of rows beyond it are clamped to it; never stored);
//   strides in bytes, kt = K / 64, and the three tile origins.
// The tile starts at token m0, feature n0; M and N bound the loads and the stores.  row_scale as in gemm_tile.
template <int TW, int TA, int EPI>
__device__ __forceinline__ void gemm_tile4(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W0,
                                           const bf16_t* __restrict__ W1, const bf16_t* R, bf16_t* C, int ldo, int M,
                                           int N, int K, int m0, int n0, unsigned char* lds, const EpiExtra& re) {
    static_assert(EPI != EPI_ROPE || TW == 4, "the RoPE epilogue needs one 128-wide head per wave");
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int BN = 64 * TW, WROWS = BN * NW;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    const int l32 = lane & 31, hh = lane >> 5;
    const unsigned lds_base = (unsigned)(uintptr_t)lds;
    const unsigned wfrag0 = lds_base + lds_off(wn * TW * 32 + l32, hh);
    const unsigned afrag0 = lds_base + WROWS * BK * 2 + lds_off(wm * TA * 32 + l32, hh);
    const unsigned r0 = wave * 8 + (lane >> 3), chunk = ((lane & 7) ^ swz(r0)) * 16;
    const uint64_t w0base = (uint64_t)(uintptr_t)(W0 + (size_t)n0 * K);
    const uint64_t w1base = NW == 2 ? (uint64_t)(uintptr_t)(W1 + (size_t)n0 * K) : w0base;
    const uint64_t abase = (uint64_t)(uintptr_t)(A + (size_t)m0 * lda);
    f32x16 acc[NW][TW][TA];
#define SLIM_LOOP_ARGS wfrag0, afrag0, r0, chunk, N - 1 - n0, M - 1 - m0, (unsigned)K * 2, (unsigned)lda * 2,          \
                       (unsigned)(K / BK), lds_base + wave * 1024, w0base, w1base, abase, acc
    // With a residual the k-loop itself adds the tile of R to the accumulators (it fetches the tile as MFMA fragments
    // and multiplies it by identity slices), and the tile is then stored as a plain one.  The launcher has checked that
    // the tile has all its features and that the rows of R are 16-byte aligned.
    constexpr int EPI_OUT = EPI == EPI_RESIDUAL ? (int)EPI_PLAIN : EPI;
    if constexpr (EPI == EPI_RESIDUAL) {
        const unsigned rrow0 = wm * TA * 32 + l32;                              // the lane's token row of the tile (j = 0)
        const unsigned rcol0 = (unsigned)(n0 + wn * TW * 32 + 8 * hh) * 2;      // byte column of its 8 features
        const bf16_t* rbase = R + (size_t)m0 * ldo;
        if constexpr (TA == 4) gemm_mainloop_4_4_1_resid(SLIM_LOOP_ARGS, rrow0, rcol0, (unsigned)ldo * 2, rbase);
        else gemm_mainloop_4_2_1_resid(SLIM_LOOP_ARGS, rrow0, rcol0, (unsigned)ldo * 2, rbase);
    } else if constexpr (TW == 4 && TA == 4) gemm_mainloop_4_4_1(SLIM_LOOP_ARGS);
    else if constexpr (TW == 4 && TA == 2) gemm_mainloop_4_2_1(SLIM_LOOP_ARGS);
    else if constexpr (TW == 2 && TA == 4) gemm_mainloop_2_4_2(SLIM_LOOP_ARGS);
    else gemm_mainloop_2_2_2(SLIM_LOOP_ARGS);
#undef SLIM_LOOP_ARGS
    // The epilogue's per-lane values are formed again behind the loop from a lane id that the compiler must take as
    // new: anything it derived from the lane id earlier would otherwise be kept in VGPRs across the loop, which has
    // few to spare, and be spilled to scratch memory.
    int tid_e = tid;
    asm volatile("" : "+v"(tid_e));
    const int lane_e = tid_e & 63, l32_e = lane_e & 31, hh_e = lane_e >> 5;
    static_assert((TW == 4 && NW == 1 && (TA == 4 || TA == 2)) || (TW == 2 && NW == 2 && (TA == 4 || TA == 2)),
                  "no generated k-loop for this wave tile");
    if (re.row_scale) {
        float inv[TA];                                   // all requested before the first is used: one wait, not TA
#pragma unroll
        for (int j = 0; j < TA; ++j) inv[j] = re.row_scale[min(m0 + (wm * TA + j) * 32 + l32_e, M - 1)];
#pragma unroll
        for (int j = 0; j < TA; ++j)
#pragma unroll
            for (int w = 0; w < NW; ++w)
#pragma unroll
                for (int i = 0; i < TW; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[w][i][j][v] *= inv[j];
    }
    // The epilogue reuses the stage buffers: every wave must be past its last fragment reads and tile loads.
    __builtin_amdgcn_s_waitcnt(0x0070);
    workgroup_barrier();
    const bool wide = (N % 8 == 0) && (ldo % 8 == 0) && (((uintptr_t)C & 15) == 0) &&
                      (EPI != EPI_BIAS || ((uintptr_t)R & 7) == 0);
    if constexpr (EPI == EPI_ROPE) {                     // the launcher has checked what `wide` checks
        store_tile_rope<TA>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, lane_e,
                            lds + wave * (TA * 32 * TW * 64), re);
    } else {
        if (wide)
            store_tile_via_lds<TW, TA, EPI_OUT>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, lane_e,
                                            lds + wave * (TA * 32 * TW * 64));
        else
            store_tile<TW, TA, EPI_OUT>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, l32_e, hh_e);
    }
}

// Few-row kernel: every workgroup computes one tile of the same shape.
template <int TW, int TA, int WGN, int WGM, int EPI>
__global__ void __launch_bounds__(512) gemm_bf16_kernel(const bf16_t* __restrict__ A, int lda,
                                                        const bf16_t* __restrict__ W0,
                                                        const bf16_t* __restrict__ W1, const bf16_t* R, bf16_t* C,
                                                        int ldo, int M, int N, int K, int tiles_m, int tiles_n,
                                                        EpiExtra re) {
    extern __shared__ __align__(16) unsigned char lds[];
    int tm, tn;
    tile_of_workgroup(blockIdx.x, true, tiles_m, tiles_n, tm, tn);
    gemm_tile<TW, TA, WGN, WGM, EPI>(A, lda, W0, W1, R, C, ldo, M, N, K, tm * 32 * TA * WGM, tn * 32 * TW * WGN, lds, re);
}

// Shapes of the two-size launch: 256-token tiles for the first big_tiles_m token-tiles, 128-token tiles
// (same feature width) for the rest.  Wave tiles: 128 features x 128 tokens (large), 128 x 64 (small); for SwiGLU
// the 128 features are 64 gate + 64 up.  Either way a wave of the plain shapes holds one 128-wide head (RoPE).
template <int EPI> struct TileShapes {
    static constexpr int TW = EPI == EPI_SWIGLU ? 2 : 4;
    static constexpr int TA_BIG = 4, TA_SMALL = 2;
    static constexpr int BN = 64 * TW;
    static constexpr int BM_BIG = 64 * TA_BIG, BM_SMALL = 64 * TA_SMALL;
};

// Two tile sizes in one launch.  Workgroups are started in id order, so the 256-token tiles run first
// and the 128-token tiles fill the last, partly empty round of workgroups: the tail of the launch costs
// about half a tile time instead of a whole one, and a ragged last token-tile wastes no MFMA work.
template <int EPI>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
gemm_bf16_two_size_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W0,
                          const bf16_t* __restrict__ W1, const bf16_t* R, bf16_t* C, int ldo, int M, int N, int K,
                          int big_tiles_m, int small_tiles_m, int tiles_n, EpiExtra re) {
    using S = TileShapes<EPI>;
    extern __shared__ __align__(16) unsigned char lds[];
    const int n_big = big_tiles_m * tiles_n;
    const bool big = (int)blockIdx.x < n_big;
    int tm, tn;
    if (big) tile_of_workgroup(blockIdx.x, true, big_tiles_m, tiles_n, tm, tn);
    else tile_of_workgroup(blockIdx.x - n_big, n_big % 8 == 0, small_tiles_m, tiles_n, tm, tn);
    if (re.w_2 && tn >= re.tiles_n1) {                   // a feature tile of the second projection
        W0 = re.w_2; R = re.r_2; C = re.c_2; N = re.n_2; ldo = re.ldo_2;
        tn -= re.tiles_n1;
    }
    if (big)
        gemm_tile4<S::TW, S::TA_BIG, EPI>(A, lda, W0, W1, R, C, ldo, M, N, K, tm * S::BM_BIG, tn * S::BN, lds, re);
    else
        gemm_tile4<S::TW, S::TA_SMALL, EPI>(A, lda, W0, W1, R, C, ldo, M, N, K,
                                            big_tiles_m * S::BM_BIG + tm * S::BM_SMALL, tn * S::BN, lds, re);
}

// The residual epilogue reads a second tile through LDS; with a lone wave per SIMD nothing hides that pass, and the
// launch measured slower than with the 8-wave tile (two waves per SIMD: one wave's epilogue steps overlap the
// other's).  So output and down projection keep 8 waves: wave tiles of 64 tokens x 128 features (large) and
// 64 x 64 (small), the same workgroup tiles as above.
__global__ void __launch_bounds__(512)
gemm_bf16_two_size_residual_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W0, const bf16_t* R,
                                   bf16_t* C, int ldo, int M, int N, int K, int big_tiles_m, int small_tiles_m,
                                   int tiles_n, int band) {
    using S = TileShapes<EPI_RESIDUAL>;
    extern __shared__ __align__(16) unsigned char lds[];
    const int n_big = big_tiles_m * tiles_n;
    const bool big = (int)blockIdx.x < n_big;
    int tm, tn;
    if (big) tile_of_workgroup(blockIdx.x, true, big_tiles_m, tiles_n, tm, tn, band);
    else tile_of_workgroup(blockIdx.x - n_big, n_big % 8 == 0, small_tiles_m, tiles_n, tm, tn, band);
    const EpiExtra none;
    if (big)
        gemm_tile<4, 2, 2, 4, EPI_RESIDUAL>(A, lda, W0, nullptr, R, C, ldo, M, N, K, tm * S::BM_BIG, tn * S::BN, lds, none);
    else
        gemm_tile<2, 2, 4, 2, EPI_RESIDUAL>(A, lda, W0, nullptr, R, C, ldo, M, N, K,
                                            big_tiles_m * S::BM_BIG + tm * S::BM_SMALL, tn * S::BN, lds, none);
}

// Generic kernel (any k_in that is a multiple of 8): register-staged loads with k predicates.
// TW x TA: number of 32-row MFMA tiles per wave along the weight (n) and activation (m) directions.
// Workgroup = 4 waves arranged WGN x WGM.  SwiGLU uses two weight tiles per n (gate, up).
template <int TW, int TA, int WGN, int WGM, int EPI>
__global__ void __launch_bounds__(256) gemm_bf16_generic_kernel(const bf16_t* __restrict__ A, int lda,
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

    int tm, tn;
    tile_of_workgroup(blockIdx.x, true, tiles_m, tiles_n, tm, tn);
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

    store_tile<TW, TA, EPI>(acc, R, C, ldo, M, N, m0 + wm * TA * 32, n0 + wn * TW * 32, l32, hh);
}

template <int TW, int TA, int WGN, int WGM, int EPI, bool GENERIC>
static int launch_bf16(const bf16_t* A, int lda, const bf16_t* W0, const bf16_t* W1, const bf16_t* R, bf16_t* C,
                       int ldo, int M, int N, int K, hipStream_t st, const EpiExtra& re = EpiExtra()) {
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr int BN = 32 * TW * WGN, BM = 32 * TA * WGM;
    constexpr size_t smem = 2 * (size_t)(BN * NW + BM) * BK * 2;
    const void* kern;
    if constexpr (GENERIC) kern = (const void*)gemm_bf16_generic_kernel<TW, TA, WGN, WGM, EPI>;
    else kern = (const void*)gemm_bf16_kernel<TW, TA, WGN, WGM, EPI>;
    static std::once_flag attr_once;                     // raising the LDS limit is per function, once
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] { attr_err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); });
    if (attr_err != hipSuccess) return set_hip_error(attr_err);
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    if constexpr (GENERIC)
        hipLaunchKernelGGL((gemm_bf16_generic_kernel<TW, TA, WGN, WGM, EPI>), dim3(tiles_m * tiles_n), dim3(64 * WGN * WGM),
                           smem, st, A, lda, W0, W1, R, C, ldo, M, N, K, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((gemm_bf16_kernel<TW, TA, WGN, WGM, EPI>), dim3(tiles_m * tiles_n), dim3(64 * WGN * WGM), smem,
                           st, A, lda, W0, W1, R, C, ldo, M, N, K, tiles_m, tiles_n, re);
    return check_launch();
}

// How many 256-token tiles to run before the 128-token tiles.  Workgroups are handed to free CUs in id
// order, which is list scheduling; it is simulated for each candidate and the shortest makespan wins.
// The model, fitted to sweeps of the split on the layer's shapes:
//   a 128-token tile costs small_cost of a 256-token one (small_tile_cost);
//   CU speeds are spread over +-8 % (tiles do not run equally fast on all CUs, which is what makes a
//   fine-grained tail pay even when the large tiles fill whole rounds);
//   for the 8-wave tiles only (the sweeps of the 4-wave tiles show neither effect):
//     +1 % / +3 % when the per-XCD run of large tiles is not a multiple of 8 / of 4 tiles (the run then
//     straddles columns of the band walk and shares fewer operand panels in that XCD's L2);
//     +5 % for fewer than 4 token-tiles of small tiles (too few rows to share a weight panel between the
//     workgroups that run together).
// The result is a pure function of its arguments; the cache only remembers it (guarded, never invalidated).
static int plan_big_tiles(int M, int tiles_n, int n_cu, double small_cost, bool eight_waves) {
    static std::mutex mu;
    static std::map<std::tuple<int, int, int, bool>, int> cache;
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_tuple(M, tiles_n, (int)(small_cost * 1000), eight_waves);
    const auto hit = cache.find(key);
    if (hit != cache.end()) return hit->second;
    std::vector<double> speed(n_cu);
    for (int c = 0; c < n_cu; ++c) speed[c] = 1.0 + 0.08 * ((double)((c * 97) % n_cu) / (n_cu - 1) * 2.0 - 1.0);
    const int mb_max = M / 256;
    int best_mb = mb_max;
    double best = 1e300;
    typedef std::pair<double, int> Slot;                 // (time the CU becomes free, CU)
    for (int mb = mb_max; mb >= 0 && mb >= mb_max - 24; --mb) {
        const int small_tiles_m = (M - mb * 256 + 127) / 128;
        const long nb = (long)mb * tiles_n, ns = (long)small_tiles_m * tiles_n;
        std::priority_queue<Slot, std::vector<Slot>, std::greater<Slot>> free_at;
        for (int c = 0; c < n_cu; ++c) free_at.push(Slot(0.0, c));
        double makespan = 0.0;
        for (long i = 0; i < nb + ns; ++i) {
            Slot s = free_at.top();
            free_at.pop();
            s.first += speed[s.second] * (i < nb ? 1.0 : small_cost);
            if (s.first > makespan) makespan = s.first;
            free_at.push(s);
        }
        if (eight_waves && nb > 0 && nb % 8 == 0) {
            const long run = nb / 8;
            if (run % 8 != 0) makespan *= 1.01;
            if (run % 4 != 0) makespan *= 1.03;
        }
        if (eight_waves && small_tiles_m > 0 && small_tiles_m < 4 && mb > 0) makespan *= 1.05;
        if (makespan < best) { best = makespan; best_mb = mb; }
    }
    cache[key] = best_mb;
    return best_mb;
}

// Which tile the residual epilogue runs in.  The 4-wave tile takes the residual tile in as MFMA fragments (16-byte loads
// at the lane's own rows and features), which needs every tile to have all of its features and 16-byte aligned rows of
// R.  Measured against the 8-wave tile on one machine, 4096 features out: with rows of 4096 (output projection) it is
// the faster one at every token count from 2048 to 32768 (-1.5 % to -6 %; -4 % inside the layer at 9856 tokens); with
// rows of 14336 (down projection) it is 1-2 % faster while the activation matrix sits in the 256 MB memory-side cache
// and 4-7 % slower once that matrix streams from HBM (282 MB at 9856 tokens), where the 8-wave tile, which issues a
// k-tile's loads at once and so leaves them longest to arrive, wins.  The 8-wave tile's epilogue parks a coalesced copy
// of the tile of R in LDS and takes any shape.
static bool residual_in_four_waves(const bf16_t* R, int M, int N, int K, int ldo) {
    const size_t activation_bytes = (size_t)M * K * sizeof(bf16_t);
    return N % 256 == 0 && ldo % 8 == 0 && ((uintptr_t)R & 15) == 0 &&
           (K <= 8192 || activation_bytes <= ((size_t)160 << 20));
}

// What a 128-token tile costs next to a 256-token one of the same launch (measured k-loop + epilogue times): the
// 4-wave small tiles run 8 MFMAs per k-step against 6 fragment reads and 3 tile loads (SwiGLU: 8 against 6 and 3,
// with the longer epilogue per output), the 8-wave ones keep the ratio of the large tile.
template <int EPI> constexpr double small_tile_cost(bool eight_waves) {
    return eight_waves ? 0.5 : (EPI == EPI_SWIGLU ? 0.7 : 0.6);
}

template <int EPI>
static int launch_two_size(const bf16_t* A, int lda, const bf16_t* W0, const bf16_t* W1, const bf16_t* R, bf16_t* C,
                           int ldo, int M, int N, int K, int big_tiles_m, bool eight_waves, hipStream_t st,
                           const EpiExtra& re = EpiExtra()) {
    using S = TileShapes<EPI>;
    constexpr int NW = EPI == EPI_SWIGLU ? 2 : 1;
    constexpr size_t smem = 2 * (size_t)(S::BN * NW + S::BM_BIG) * BK * 2;
    static std::once_flag attr_once, attr8_once;
    static hipError_t attr_err = hipSuccess, attr8_err = hipSuccess;
    if ((size_t)K >= (1u << 23) || (size_t)lda >= (1u << 23) || (size_t)ldo >= (1u << 23))
        return SLIM_UNSUPPORTED;                         // 32-bit byte offsets inside a tile
    const int tiles_n = (N + S::BN - 1) / S::BN + (re.w_2 ? (re.n_2 + S::BN - 1) / S::BN : 0);
    const int small_tiles_m = (M - big_tiles_m * S::BM_BIG + S::BM_SMALL - 1) / S::BM_SMALL;
    const dim3 grid((big_tiles_m + small_tiles_m) * tiles_n);
    if (EPI == EPI_RESIDUAL && eight_waves) {
        auto kern = gemm_bf16_two_size_residual_kernel;
        std::call_once(attr8_once, [&] {
            attr8_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        });
        if (attr8_err != hipSuccess) return set_hip_error(attr8_err);
        // Long activation rows that stream from HBM (the matrix does not fit the memory-side cache): bands of 2
        // token-tiles, so that the tiles resident on an XCD cover every feature tile of a token band and each
        // activation panel is fetched once instead of once per group of 4 feature tiles (down projection of 9856
        // tokens -1.8 %, of 32768 tokens -2.6 %; with rows of 4096 the same walk is 6 % slower, so it is not used there).
        const int band = ((size_t)M * K * sizeof(bf16_t) > ((size_t)160 << 20) && K > 8192) ? 2 : 8;
        hipLaunchKernelGGL(kern, grid, dim3(512), smem, st, A, lda, W0, R, C, ldo, M, N, K, big_tiles_m, small_tiles_m, tiles_n,
                           band);
    } else {
        auto kern = gemm_bf16_two_size_kernel<EPI>;
        std::call_once(attr_once, [&] {
            attr_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        });
        if (attr_err != hipSuccess) return set_hip_error(attr_err);
        hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, A, lda, W0, W1, R, C, ldo, M, N, K, big_tiles_m, small_tiles_m,
                           tiles_n, re);
    }
    return check_launch();
}

static int cu_count() {
    static std::once_flag once;                          // immutable once read: a property of the device
    static int n = 256;
    std::call_once(once, [] {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
            n = prop.multiProcessorCount;
    });
    return n;
}

template <int EPI>
static int dispatch_bf16(const bf16_t* A, int lda, const bf16_t* W0, const bf16_t* W1, const bf16_t* R, bf16_t* C,
                         int ldo, int M, int N, int K, hipStream_t st, const EpiExtra& re = EpiExtra()) {
    if constexpr (EPI != EPI_ROPE) {                     // (row_scale and RoPE callers have checked K % 64 == 0)
        if (K % BK != 0) return launch_bf16<2, 2, 2, 2, EPI, true>(A, lda, W0, W1, R, C, ldo, M, N, K, st);
    }
    if ((size_t)K >= (1u << 23) || (size_t)lda >= (1u << 23)) {   // 32-bit byte offsets inside a tile of 256 rows
        if constexpr (EPI == EPI_ROPE) return SLIM_UNSUPPORTED;
        else if (!re.row_scale && !re.w_2) return launch_bf16<2, 2, 2, 2, EPI, true>(A, lda, W0, W1, R, C, ldo, M, N, K, st);
        else return SLIM_UNSUPPORTED;
    }
    if (M <= 128) {
        // Few rows: the launch streams the weights once and is bound by how many workgroups pull on memory at the same
        // time, so wide outputs use 64-feature tiles (twice the workgroups of the 128-feature ones).
        if constexpr (EPI == EPI_SWIGLU) return launch_bf16<1, 1, 2, 4, EPI, false>(A, lda, W0, W1, R, C, ldo, M, N, K, st, re);
        else if constexpr (EPI == EPI_ROPE) return launch_bf16<4, 1, 2, 4, EPI, false>(A, lda, W0, W1, R, C, ldo, M, N, K, st, re);
        else if (N >= 2048) return launch_bf16<1, 1, 2, 4, EPI, false>(A, lda, W0, W1, R, C, ldo, M, N, K, st, re);
        else return launch_bf16<2, 1, 2, 4, EPI, false>(A, lda, W0, W1, R, C, ldo, M, N, K, st, re);
    }
    const int tiles_n = (N + TileShapes<EPI>::BN - 1) / TileShapes<EPI>::BN;
    const bool eight = EPI == EPI_RESIDUAL && !residual_in_four_waves(R, M, N, K, ldo);
    return launch_two_size<EPI>(A, lda, W0, W1, R, C, ldo, M, N, K,
                                plan_big_tiles(M, tiles_n, cu_count(), small_tile_cost<EPI>(eight), eight), eight, st, re);
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
            if (EPI == EPI_BIAS) o += R[n];
            C[(size_t)m * ldo + n] = o;
        }
    }
}

// Query/Key projection with the RoPE epilogue (bf16, heads of 128, k_in a multiple of 64; checked by the caller).
// row_scale != null: the rows of a are the raw residual stream and row_scale their 1/rms (fused RMSNorm).
int launch_linear_rope(const void* a, int lda, const void* w, const void* bias, const float* table, const float* qt,
                       float* token_scores, const float* row_scale, int m, int n_heads, int k_in, int ldo, void* out,
                       hipStream_t st) {
    EpiExtra re;
    re.table = table;
    re.qt = qt;
    re.token_scores = token_scores;
    re.row_scale = row_scale;
    return dispatch_bf16<EPI_ROPE>((const bf16_t*)a, lda, (const bf16_t*)w, nullptr, (const bf16_t*)bias, (bf16_t*)out, ldo, m,
                                   n_heads * 128, k_in, st, re);
}

// Projection of row-scaled activations: plain, + bias, or SwiGLU (w1).  bf16, k_in a multiple of 64 (checked by
// the caller).
int launch_linear_scaled(const void* a, int lda, const void* w0, const void* w1, const void* bias, const float* row_scale,
                         int m, int n_out, int k_in, int ldo, void* out, hipStream_t st) {
    EpiExtra re;
    re.row_scale = row_scale;
    const bf16_t *A = (const bf16_t*)a, *W0 = (const bf16_t*)w0, *W1 = (const bf16_t*)w1, *B = (const bf16_t*)bias;
    bf16_t* C = (bf16_t*)out;
    if (w1) return dispatch_bf16<EPI_SWIGLU>(A, lda, W0, W1, nullptr, C, ldo, m, n_out, k_in, st, re);
    if (bias) return dispatch_bf16<EPI_BIAS>(A, lda, W0, nullptr, B, C, ldo, m, n_out, k_in, st, re);
    return dispatch_bf16<EPI_PLAIN>(A, lda, W0, nullptr, nullptr, C, ldo, m, n_out, k_in, st, re);
}

// Two projections of the same rows in one launch (the Query and Value projections of the continuing tokens): the
// second one's feature tiles follow the first one's, so the launch fills the chip as one problem of n_1 + n_2
// features.  Both with a bias or both without.  bf16, k_in % 64 == 0, m > 128 (checked by the caller).
int launch_linear_pair(const void* a, int lda, const void* w_1, const void* bias_1, int n_1, int ldo_1, void* out_1,
                       const void* w_2, const void* bias_2, int n_2, int ldo_2, void* out_2, const float* row_scale,
                       int m, int k_in, hipStream_t st) {
    EpiExtra re;
    re.row_scale = row_scale;
    re.w_2 = (const bf16_t*)w_2;
    re.r_2 = (const bf16_t*)bias_2;
    re.c_2 = (bf16_t*)out_2;
    re.n_2 = n_2;
    re.ldo_2 = ldo_2;
    const bf16_t *A = (const bf16_t*)a, *W = (const bf16_t*)w_1, *B = (const bf16_t*)bias_1;
    if (bias_1) {
        using S = TileShapes<EPI_BIAS>;
        re.tiles_n1 = (n_1 + S::BN - 1) / S::BN;
        const int tiles_n = re.tiles_n1 + (n_2 + S::BN - 1) / S::BN;
        return launch_two_size<EPI_BIAS>(A, lda, W, nullptr, B, (bf16_t*)out_1, ldo_1, m, n_1, k_in,
                                         plan_big_tiles(m, tiles_n, cu_count(), small_tile_cost<EPI_BIAS>(false), false),
                                         false, st, re);
    }
    using S = TileShapes<EPI_PLAIN>;
    re.tiles_n1 = (n_1 + S::BN - 1) / S::BN;
    const int tiles_n = re.tiles_n1 + (n_2 + S::BN - 1) / S::BN;
    return launch_two_size<EPI_PLAIN>(A, lda, W, nullptr, nullptr, (bf16_t*)out_1, ldo_1, m, n_1, k_in,
                                      plan_big_tiles(m, tiles_n, cu_count(), small_tile_cost<EPI_PLAIN>(false), false),
                                      false, st, re);
}

// At most one of w1 (SwiGLU), residual and bias is set.
int launch_linear(const void* a, int lda, const void* w0, const void* w1, const void* residual, const void* bias,
                  int m, int n_out, int k_in, int ldo, int dtype, void* out, hipStream_t st) {
    if (dtype == SLIM_F32) {
        dim3 grid((n_out + 63) / 64, (m + 63) / 64);
#define SLIM_F32_GEMM(E) hipLaunchKernelGGL(gemm_f32_kernel<E>, grid, dim3(256), 0, st, (const float*)a, lda, \
        (const float*)w0, (const float*)w1, (const float*)(bias ? bias : residual), (float*)out, ldo, m, n_out, k_in)
        if (w1) SLIM_F32_GEMM(EPI_SWIGLU); else if (residual) SLIM_F32_GEMM(EPI_RESIDUAL);
        else if (bias) SLIM_F32_GEMM(EPI_BIAS); else SLIM_F32_GEMM(EPI_PLAIN);
#undef SLIM_F32_GEMM
        return check_launch();
    }
    const bf16_t *A = (const bf16_t*)a, *W0 = (const bf16_t*)w0, *W1 = (const bf16_t*)w1, *R = (const bf16_t*)residual;
    bf16_t* C = (bf16_t*)out;
    if (w1) return dispatch_bf16<EPI_SWIGLU>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
    if (residual) return dispatch_bf16<EPI_RESIDUAL>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
    if (bias) return dispatch_bf16<EPI_BIAS>(A, lda, W0, W1, (const bf16_t*)bias, C, ldo, m, n_out, k_in, st);
    return dispatch_bf16<EPI_PLAIN>(A, lda, W0, W1, R, C, ldo, m, n_out, k_in, st);
}

}  // namespace slim
