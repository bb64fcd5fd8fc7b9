// Register-resident MFMA loop: measures the bf16 MFMA rate this GPU sustains when
// nothing else (LDS, memory, barriers) is in the way.  The operand fragments are
// read once from `frags`, so the caller chooses the bit patterns: the sustained
// clock, and with it the rate, depends on how much the operand bits toggle.
// Used only by the benchmark to report the attainable ceiling beside the vendor peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__global__ __launch_bounds__(512) void mfma_probe_kernel(const bf16x8* __restrict__ frags, float* out, int iters) {
  // 4 "A" and 2 "B" fragments per lane, as in the 128 x 64 wave tile of the real kernels
  bf16x8 a[4], b[2];
  const int lane = threadIdx.x & 63;
  for (int i = 0; i < 4; ++i) a[i] = frags[(i * 64 + lane) % 384];
  for (int i = 0; i < 2; ++i) b[i] = frags[((4 + i) * 64 + lane) % 384];
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j)
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j >> 1], b[j & 1], acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j)
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Plain 16-byte-per-lane copy: the known-size reference against which the hardware's
// HBM byte counters are scaled when a profile is read.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

// Copies `bytes` (a multiple of 16) from src to dst, both device pointers, on `stream`.
// Returns a hipError_t value.
extern "C" int cce_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes % 16) return (int)hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  if (n16 == 0) return 0;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                     (uint4*)dst, n16);
  return (int)hipGetLastError();
}

// Launches `blocks` workgroups of 512 lanes, each wavefront issuing 8 * iters
// v_mfma_f32_32x32x16_bf16 on fragments taken from `frags` (device, 384 * 16 bytes of
// bf16 data).  `out` is a device buffer of blocks * 512 floats.
// flops = blocks * 8 waves * iters * 8 * 32768.  Returns a hipError_t value.
extern "C" int cce_probe_mfma(const void* frags, float* out, int blocks, int iters, void* stream) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)stream, (const bf16x8*)frags, out,
                     iters);
  return (int)hipGetLastError();
}
