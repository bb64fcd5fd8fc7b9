/*
 * cce_probe.h - measurement helpers of the benchmark, built into their own shared
 * object (libcce_probe.so), not into the product library.  They are not part of the
 * method: bench.py uses them to state the bf16 MFMA rate this GPU sustains and to
 * scale the profiler's HBM byte counters.
 * All pointers are DEVICE pointers; calls are asynchronous on `stream`
 * (hipStream_t, NULL = null stream) and return a hipError_t value (0 = success).
 */
#ifndef CCE_PROBE_H_
#define CCE_PROBE_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Register-resident MFMA loop: `blocks` workgroups of 512 lanes, every wavefront issuing
 * 8 * iters v_mfma_f32_32x32x16_bf16 on operand fragments read once from `frags`
 * (384 * 16 bytes of bf16 data chosen by the caller: the sustained clock depends on how
 * much the operand bits toggle).  `out`: blocks * 512 floats.
 * flop = blocks * 8 * iters * 8 * 32768. */
int cce_probe_mfma(const void* frags, float* out, int blocks, int iters, void* stream);

/* Plain copy of `bytes` (a multiple of 16) from src to dst: reads and writes exactly
 * `bytes` of HBM, the reference for scaling FETCH_SIZE / WRITE_SIZE counters. */
int cce_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CCE_PROBE_H_ */
