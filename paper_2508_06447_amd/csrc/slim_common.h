// Shared device/host helpers for libslim (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "slim.h"

namespace slim {

typedef unsigned short bf16_t;                       // storage type of a bfloat16
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __builtin_bit_cast(float, (uint32_t)v << 16);
}
// Round-to-nearest-even (hardware v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// Two values in one v_cvt_pk_bf16_f32 (converted one by one they cost a shift and an or on top of two conversions).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// Element access templated on the storage type (float or bf16_t).
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kVec = 4;                   // elements per 16-byte chunk
    __device__ static float ld(const float* p) { return *p; }
    __device__ static void st(float* p, float v) { *p = v; }
    __device__ static void unpack(const uint4& c, float* f) {
        f[0] = __builtin_bit_cast(float, c.x); f[1] = __builtin_bit_cast(float, c.y);
        f[2] = __builtin_bit_cast(float, c.z); f[3] = __builtin_bit_cast(float, c.w);
    }
    __device__ static uint4 pack(const float* f) {
        return make_uint4(__builtin_bit_cast(uint32_t, f[0]), __builtin_bit_cast(uint32_t, f[1]),
                          __builtin_bit_cast(uint32_t, f[2]), __builtin_bit_cast(uint32_t, f[3]));
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int kVec = 8;
    __device__ static float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    __device__ static void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    __device__ static void unpack(const uint4& c, float* f) {
        f[0] = lo_bf16(c.x); f[1] = hi_bf16(c.x); f[2] = lo_bf16(c.y); f[3] = hi_bf16(c.y);
        f[4] = lo_bf16(c.z); f[5] = hi_bf16(c.z); f[6] = lo_bf16(c.w); f[7] = hi_bf16(c.w);
    }
    __device__ static uint4 pack(const float* f) {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]),
                          pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// One 16-byte-per-lane load from global memory straight into LDS.  The LDS address of lane l is
// (wave-uniform base) + 16*l; the base travels in M0.  The compiler does not see this as an LDS write,
// so callers order it against LDS reads themselves: s_waitcnt vmcnt + workgroup barrier.
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_global_to_lds16(const void* g, void* lds_wave_base) {
    const unsigned la = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)lds_wave_base);
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(la) : "memory", "m0");
}
// Same, with the global address split into a wave-uniform 64-bit base (scalar registers) and a per-lane
// 32-bit byte offset: a load whose base moves every iteration then costs scalar instructions only.
__device__ __forceinline__ void load_global_to_lds16(const void* uniform_base, unsigned lane_byte_offset,
                                                     unsigned lds_wave_base) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_byte_offset), "s"(uniform_base), "s"(lds_wave_base) : "memory", "m0");
}
__device__ __forceinline__ void workgroup_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ---- host side ---------------------------------------------------------------------------------
int set_hip_error(hipError_t e);                      // records text, returns SLIM_HIP_ERROR
inline int check_launch() {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? SLIM_OK : set_hip_error(e);
}
inline size_t elem_size(int dtype) { return dtype == SLIM_BF16 ? 2 : 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Internal launchers (each validates nothing: the C entry points do).
int launch_rmsnorm(const void* x, const void* gain, int n, int hidden, float eps, int dtype, void* out, hipStream_t st);
int launch_rope(void* x, const int* pos, int pos0, int n, int H, int d, float theta, int dtype, hipStream_t st);
int launch_linear(const void* a, int lda, const void* w0, const void* w1, const void* residual, const void* bias, int m,
                  int n_out, int k_in, int ldo, int dtype, void* out, hipStream_t st);
int launch_score(const void* q_win, const void* k, int N, int w, int Hq, int Hkv, int d, int block, int unit,
                 int pooling, int dtype, float* scores, float* qtilde, hipStream_t st);
int launch_rope_table(const int* pos, int pos0, int n, int d, float theta, float* table, hipStream_t st);
int launch_linear_rope(const void* a, int lda, const void* w, const void* bias, const float* table, const float* qt,
                       float* token_scores, const float* row_scale, int m, int n_heads, int k_in, int ldo, void* out,
                       hipStream_t st);
int launch_linear_scaled(const void* a, int lda, const void* w0, const void* w1, const void* bias, const float* row_scale,
                         int m, int n_out, int k_in, int ldo, void* out, hipStream_t st);
int launch_linear_pair(const void* a, int lda, const void* w_1, const void* bias_1, int n_1, int ldo_1, void* out_1,
                       const void* w_2, const void* bias_2, int n_2, int ldo_2, void* out_2, const float* row_scale,
                       int m, int k_in, hipStream_t st);
int launch_row_rstd(const void* x, int n, int hidden, float eps, int dtype, float* rstd, hipStream_t st,
                    const int* pos = nullptr, int d = 0, float theta = 0.f, float* table = nullptr);
int launch_fold_gain(const void* w, const void* gain, int n_out, int k_in, int dtype, void* out, hipStream_t st);
int launch_window_query(const void* q_win, int w, int Hq, int Hkv, int d, int dtype, float* qtilde, hipStream_t st);
// Window query from the hidden rows of the window (skinny split projection + rotation + means); `partial` holds
// kWindowSplitsMax * w * Hq * 128 floats.
constexpr int kWindowSplitsMax = 4;
constexpr int kWindowRowsMax = 256;
int launch_window_query_rows(const void* x, int lda, const void* wq, const void* bias, const float* rstd,
                             const float* table, int w, int Hq, int Hkv, int k_in, float* partial, float* qt,
                             hipStream_t st);
int launch_token_score_blocks(const float* token_scores, int N, int H, int block, int unit, float* scores, hipStream_t st);
int launch_unit_keys(const void* k, int N, int E, int block, int unit, int dtype, float* k_rep, hipStream_t st);
int launch_score_from_unit_keys(const void* q_win, const float* k_rep, int N, int w, int Hq, int Hkv, int d,
                                int block, int unit, int dtype, float* scores, float* qtilde, hipStream_t st);
int launch_kv_swap(const int* candidate, int n_candidates, int n_blocks, double gamma, int* slot_of_block,
                   int* block_of_slot, int* in_memory, int n_slots, void* gpu_pool, void* host_pool,
                   size_t block_bytes, int* info, int* workspace, hipStream_t st);
int launch_positions(const int* pos_in, int* pos_out, int n, hipStream_t st);
int launch_select(const float* scores, int nb, int n_keep, unsigned flags, int* kept, hipStream_t st);
int launch_compact(const void* src, const int* pos_in, const int* kept, int n_keep, int block, int N,
                   int row_elems, int dtype, void* dst, int* pos_out, hipStream_t st);
int launch_compact_multi(int n_arrays, const void* const* src, void* const* dst, const size_t* row_bytes, const int* pos_in,
                         int* pos_out, const int* kept, int n_keep, int block, int N, hipStream_t st);
int launch_decode_attn(const void* q, const void* pool, size_t slot_bytes, size_t layer_offset, const int* block_of_slot,
                       int n_slots, int block, int n_prompt, const void* k_resp, const void* v_resp, int n_resp, int Hq,
                       int Hkv, float scale, int dtype, void* out, float* part, hipStream_t st);
int launch_gemv(const void* w0, const void* w1, const void* x, const float* scale, float norm_eps, const void* bias,
                const void* residual, int n_out, int k_in, int dtype, void* out, hipStream_t st);
int launch_gemv_qkv(const void* wq, const void* wk, const void* wv, const void* bq, const void* bk, const void* bv,
                    const void* x, float norm_eps, int n_q, int n_kv, int k_in, int position, float theta, int dtype,
                    void* q, void* k, void* v, hipStream_t st);
int launch_attn(const void* q, const void* k, const void* v, int n, int Hq, int Hkv, int d, float scale,
                int dtype, void* out, hipStream_t st);

}  // namespace slim
