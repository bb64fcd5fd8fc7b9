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

// The same loop with the tile engine's other activities added one at a time, to see what each costs when
// the chip is limited by power rather than by issue slots: LDS fragment reads at the rate of a 128 x 64 wave
// tile (6 ds_read_b128 per 8 MFMAs, or 12 transposing 8-byte reads when both operands are K-major) or of a
// 128 x 128 one (4 per 8), and direct-to-LDS loads from a buffer
// that stays in the L2 at the rate of a 256 x 256 x 64 stage (8 KB per wave per 32 MFMAs).
#define CCE_PROBE_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define CCE_PROBE_GLB(p) ((const __attribute__((address_space(1))) void*)(p))
template <int READS, int DMA>
__global__ __launch_bounds__(512) void engine_probe_kernel(const uint4* __restrict__ data, const char* __restrict__ gbuf,
                                                           float* out, int iters) {
  __shared__ __attribute__((aligned(1024))) char lds[131072];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 65536 / 16; i += 512) ((uint4*)lds)[i] = data[i];   // 64 KB of operand data
  __syncthreads();
  const uint32_t base = (uint32_t)(uintptr_t)CCE_PROBE_LDS(lds) + (uint32_t)lane * 16u + (uint32_t)(wave & 3) * 1024u;
  bf16x8 f[2][6];
  for (int j = 0; j < 6; ++j) {
    f[0][j] = ((bf16x8*)lds)[(j * 64 + lane) & 4095];
    f[1][j] = ((bf16x8*)lds)[((j + 6) * 64 + lane) & 4095];
  }
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j)
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  char* dma_dst = lds + 65536 + wave * 8192;   // 8 KB per wave, written by the loads, never read
  const char* gsrc = gbuf + (size_t)(blockIdx.x & 15) * 65536 + wave * 8192 + lane * 16;
  // reads of iteration `it` fill nxt (highest byte touched: 53248 < 65536); cur feeds the MFMAs
  auto step = [&](int it, bf16x8 (&cur)[6], bf16x8 (&nxt)[6]) {
    const uint32_t a = base + (uint32_t)((it & 7) * 4096);
    if (READS == 12) {
      // both operands K-major: two 8-byte transposing reads per fragment (highest byte touched: 55296 < 65536)
      typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
      typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
      u32x2_t t[12];
#define CCE_PROBE_TR(i, off) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:" #off : "=v"(t[i]) : "v"(a));
      CCE_PROBE_TR(0, 0) CCE_PROBE_TR(1, 2048) CCE_PROBE_TR(2, 4096) CCE_PROBE_TR(3, 6144) CCE_PROBE_TR(4, 8192)
      CCE_PROBE_TR(5, 10240) CCE_PROBE_TR(6, 12288) CCE_PROBE_TR(7, 14336) CCE_PROBE_TR(8, 16384)
      CCE_PROBE_TR(9, 18432) CCE_PROBE_TR(10, 20480) CCE_PROBE_TR(11, 22528)
#undef CCE_PROBE_TR
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]), "+v"(t[5]), "+v"(t[6]), "+v"(t[7]),
                     "+v"(t[8]), "+v"(t[9]), "+v"(t[10]), "+v"(t[11]));
#pragma unroll
      for (int j = 0; j < 6; ++j)
        nxt[j] = __builtin_bit_cast(bf16x8, (u32x4_t)__builtin_shufflevector(t[2 * j], t[2 * j + 1], 0, 1, 2, 3));
    } else if (READS >= 4) {
      asm volatile("ds_read_b128 %0, %1" : "=v"(nxt[0]) : "v"(a));
      asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(nxt[1]) : "v"(a));
      asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(nxt[4]) : "v"(a));
      asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(nxt[5]) : "v"(a));
    }
    if (READS >= 6) {
      asm volatile("ds_read_b128 %0, %1 offset:16384" : "=v"(nxt[2]) : "v"(a));
      asm volatile("ds_read_b128 %0, %1 offset:20480" : "=v"(nxt[3]) : "v"(a));
    }
    if (DMA && (it & 3) == 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the previous batch has landed before its LDS is rewritten
#pragma unroll
      for (int j = 0; j < 8; ++j)   // source stays inside the 8 MiB buffer: at most 15 * 64 K + 64 K + 7 * 1 M
        __builtin_amdgcn_global_load_lds(CCE_PROBE_GLB(gsrc + j * 1024 + ((it >> 2) & 7) * 1048576),
                                         CCE_PROBE_LDS(dma_dst + j * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[j >> 1], cur[4 + (j & 1)], acc[j], 0, 0, 0);
    if (READS && READS != 12)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(nxt[0]), "+v"(nxt[1]), "+v"(nxt[2]), "+v"(nxt[3]), "+v"(nxt[4]), "+v"(nxt[5]));
  };
  for (int it = 0; it < iters; it += 2) {
    step(it, f[0], f[1]);
    step(it + 1, f[1], f[0]);
  }
  if (DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float s = 0.f;
  for (int j = 0; j < 8; ++j)
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  out[blockIdx.x * 512 + tid] = s;
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


// Launches the engine-activity probe: `data` is a device buffer of at least 8 MiB + 64 KiB of bf16 operand
// data (its first 64 KiB become the LDS contents, the rest is the source of the direct loads), `out` holds
// blocks * 512 floats, `iters` is even.  lds_reads: 0, 4 or 6 ds_read_b128 per 8 MFMAs, or 12
// ds_read_b64_tr_b16 (both operands K-major); dma: 0 / 1.
// flop = blocks * 8 waves * iters * 8 * 32768.  Returns a hipError_t value.
extern "C" int cce_probe_engine(const void* data, float* out, int blocks, int iters, int lds_reads, int dma, void* stream) {
  if (!data || !out || blocks <= 0 || iters <= 0 || (iters & 1)) return (int)hipErrorInvalidValue;
  const dim3 g(blocks), b(512);
  hipStream_t st = (hipStream_t)stream;
  const uint4* d = (const uint4*)data;
  const char* gb = (const char*)data;
#define CCE_PROBE_LAUNCH(R, M) hipLaunchKernelGGL((engine_probe_kernel<R, M>), g, b, 0, st, d, gb, out, iters)
  if (lds_reads == 0 && !dma) CCE_PROBE_LAUNCH(0, 0);
  else if (lds_reads == 4 && !dma) CCE_PROBE_LAUNCH(4, 0);
  else if (lds_reads == 6 && !dma) CCE_PROBE_LAUNCH(6, 0);
  else if (lds_reads == 0 && dma) CCE_PROBE_LAUNCH(0, 1);
  else if (lds_reads == 4 && dma) CCE_PROBE_LAUNCH(4, 1);
  else if (lds_reads == 6 && dma) CCE_PROBE_LAUNCH(6, 1);
  else if (lds_reads == 12 && !dma) CCE_PROBE_LAUNCH(12, 0);
  else if (lds_reads == 12 && dma) CCE_PROBE_LAUNCH(12, 1);
  else return (int)hipErrorInvalidValue;
#undef CCE_PROBE_LAUNCH
  return (int)hipGetLastError();
}
