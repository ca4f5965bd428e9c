/*
 * libslim_probe -- measurement probes for bench.py.  Not part of the method and not part of libslim's ABI: a
 * library of its own (libslim_probe.so) with two kernels that give measured ceilings to set beside the nameplate
 * rooflines.  Conventions (device pointers, stream as void*, status codes) as in slim.h.
 */
#ifndef SLIM_PROBE_H
#define SLIM_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* slim_probe_mfma runs a register-only loop of v_mfma_f32_32x32x16_bf16 (n_workgroups
 * workgroups of 8 waves, `iters` rounds of 8 independent MFMAs per wave) and slim_probe_mfma_flops
 * returns the flop count of such a launch; `sink` is a device float that is never written.
 * random_operands = 0: constant small-integer operands; != 0: pseudo-random operands in [-1, 1) that
 * change from one MFMA to the next, as real activations and weights do (the chip clocks lower then).
 * slim_probe_copy copies `bytes` (multiple of 16, 16-byte aligned pointers) device to device with
 * 16-byte accesses.  Both only enqueue work.  Errors: INVALID_ARG, UNSUPPORTED (alignment).
 */
double slim_probe_mfma_flops(int n_workgroups, int iters);
int slim_probe_mfma(int n_workgroups, int iters, int random_operands, float* sink, void* stream);
int slim_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIM_PROBE_H */
