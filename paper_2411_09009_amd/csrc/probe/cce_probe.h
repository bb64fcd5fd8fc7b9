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

/* The MFMA loop with the tile engine's other activities added one at a time (lds_reads = 0, 4 or 6
 * ds_read_b128 per 8 MFMAs: none, the rate of a 128 x 128 wave tile, the rate of the library's 128 x 64 one;
 * 12: the same bytes as twelve ds_read_b64_tr_b16, as when both operands are K-major;
 * dma = 1: direct-to-LDS loads from an L2-resident buffer at the rate of a 256 x 256 x 64 stage).  `data`:
 * at least 8 MiB + 64 KiB of bf16 operand data; `out`: blocks * 512 floats; iters even.
 * flop = blocks * 8 * iters * 8 * 32768. */
int cce_probe_engine(const void* data, float* out, int blocks, int iters, int lds_reads, int dma, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CCE_PROBE_H_ */
