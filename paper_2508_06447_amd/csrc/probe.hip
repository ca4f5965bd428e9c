// Two measurement kernels that give the rooflines a measured counterpart on the same machine and in
// the same run: a register-only MFMA loop (what the matrix pipes sustain at the clocks the chip holds
// under that load, with constant or with changing operand bits) and a plain 16-byte-per-lane copy (what HBM sustains for a read+write stream).
#include "slim_common.h"
#include "slim_probe.h"

namespace slim {

constexpr int kProbeWaves = 8;                // waves per workgroup, two per SIMD
constexpr int kProbeAcc = 8;                  // independent accumulators per wave

// RANDOM = false: both operands constant small integers (few bits toggle between MFMAs).
// RANDOM = true: four pseudo-random operand pairs in [-1, 1) used in rotation, so the operand bits change
// from one MFMA to the next as they do with real activations and weights; the chip holds a lower clock
// under that load, which makes this the ceiling a real bf16 kernel can approach.
template <bool RANDOM>
__global__ void __launch_bounds__(64 * kProbeWaves) mfma_loop_kernel(int iters, float* sink) {
    constexpr int NP = RANDOM ? 4 : 1;
    bf16x8 a[NP], b[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RANDOM) {
                unsigned h = (threadIdx.x * 8u + i) * 2654435761u + p * 40503u + 12345u;
                h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
                a[p][i] = (__bf16)((float)(h & 0xffff) * (1.0f / 32768.0f) - 1.0f);
                b[p][i] = (__bf16)((float)(h >> 16) * (1.0f / 32768.0f) - 1.0f);
            } else {
                a[p][i] = (__bf16)(float)((threadIdx.x + i) & 3);
                b[p][i] = (__bf16)0.5f;
            }
        }
    f32x16 acc[kProbeAcc];
#pragma unroll
    for (int k = 0; k < kProbeAcc; ++k)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[k][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kProbeAcc; ++k)
            acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k % NP], b[(k / NP + k) % NP], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kProbeAcc; ++k) s += acc[k][0];
    if (s == -1.2345e30f) sink[0] = s;        // never true; keeps the loop alive
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 t[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n_vec) t[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) if (base + u * 256 < n_vec) __builtin_nontemporal_store(t[u], dst + base + u * 256);
}

}  // namespace slim

using namespace slim;

extern "C" {

double slim_probe_mfma_flops(int n_workgroups, int iters) {
    return (double)n_workgroups * kProbeWaves * (double)iters * kProbeAcc * 2.0 * 32 * 32 * 16;
}

int slim_probe_mfma(int n_workgroups, int iters, int random_operands, float* sink, void* stream) {
    if (n_workgroups < 1 || iters < 1 || !sink) return SLIM_INVALID_ARG;
    if (random_operands)
        hipLaunchKernelGGL(mfma_loop_kernel<true>, dim3(n_workgroups), dim3(64 * kProbeWaves), 0, (hipStream_t)stream, iters, sink);
    else
        hipLaunchKernelGGL(mfma_loop_kernel<false>, dim3(n_workgroups), dim3(64 * kProbeWaves), 0, (hipStream_t)stream, iters, sink);
    return hipGetLastError() == hipSuccess ? SLIM_OK : SLIM_HIP_ERROR;
}

int slim_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || bytes < 16 || bytes % 16 != 0) return SLIM_INVALID_ARG;
    if (!aligned16(src) || !aligned16(dst)) return SLIM_UNSUPPORTED;
    const size_t n_vec = bytes / 16;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n_vec + 1023) / 1024)), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)src, (u32x4*)dst, n_vec);
    return hipGetLastError() == hipSuccess ? SLIM_OK : SLIM_HIP_ERROR;
}

}  // extern "C"
