// Vocabulary sorting (paper Section 4.3, "Vocabulary sorting"), gfx950.
//
// The paper orders the vocabulary by the average logit of each entry so that the entries
// with non-negligible softmax mass fall into the same blocks and the gradient filter can
// skip the others.  It accumulates that average with atomics inside the forward kernel.
// Before the soft-cap the logit is linear in E, so the average over the batch is
//     mean_i <E_i, C_j>  =  <C_j, mean_i E_i>,
// one matrix-vector product with C: that is how the key is computed here (two small
// kernels, fixed summation order), at the start of the backward pass that uses it.
// The keys are then sorted (descending, stable) with rocPRIM's device radix sort, and the
// backward pass walks the vocabulary in that order:
//   perm[p]   original vocabulary index at sorted position p
//   targets'  = inverse permutation applied to the targets (ignored tokens stay ignored)
//   each slab's rows of C are gathered into a contiguous buffer in sorted order, and the
//   rows of dC are scattered back through perm when they are written.
// The unfiltered result does not depend on the order (up to fp32 summation order in dE).
#include "kernels.h"

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>

namespace cce {

namespace {

constexpr int kMeanRowBlocks = 64;

// partial[rb][d] = sum over the rb-th block of rows of E[i][d]
__global__ __launch_bounds__(256) void col_sum_partial_kernel(const bf16* __restrict__ E, int N, int D,
                                                              float* __restrict__ partial) {
  const int d = blockIdx.x * 256 + threadIdx.x;
  const int rows_per = (N + kMeanRowBlocks - 1) / kMeanRowBlocks;
  const int r0 = blockIdx.y * rows_per, r1 = min(N, r0 + rows_per);
  if (d >= D) return;
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += (float)E[(int64_t)r * D + d];
  partial[(int64_t)blockIdx.y * D + d] = s;
}

__global__ __launch_bounds__(256) void col_mean_kernel(const float* __restrict__ partial, int N, int D,
                                                       float* __restrict__ mean) {
  const int d = blockIdx.x * 256 + threadIdx.x;
  if (d >= D) return;
  float s = 0.f;
  for (int b = 0; b < kMeanRowBlocks; ++b) s += partial[(int64_t)b * D + d];
  mean[d] = s / (float)N;
}

// key[j] = <C_j, mean>, one wavefront per vocabulary entry; value[j] = j
__global__ __launch_bounds__(256) void mean_logit_kernel(const bf16* __restrict__ C, const float* __restrict__ mean,
                                                         int V, int D, float* __restrict__ key,
                                                         int* __restrict__ index) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= V) return;
  const bf16* row = C + (int64_t)j * D;
  float s = 0.f;
  for (int d = lane; d < D; d += 64) s = fmaf((float)row[d], mean[d], s);
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if (lane == 0) {
    key[j] = s;
    index[j] = j;
  }
}

__global__ __launch_bounds__(256) void invert_perm_kernel(const int* __restrict__ perm, int V, int* __restrict__ inv) {
  const int p = blockIdx.x * 256 + threadIdx.x;
  if (p < V) inv[perm[p]] = p;
}

__global__ __launch_bounds__(256) void remap_targets_kernel(const int64_t* __restrict__ targets, int N, int V,
                                                            int64_t ignore_index, const int* __restrict__ inv,
                                                            int64_t* __restrict__ out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= N) return;
  const int64_t t = targets[i];
  out[i] = (t != ignore_index && t >= 0 && t < V) ? (int64_t)inv[t] : ignore_index;
}

// out[r][:] = C[perm[p0 + r]][:] for r < rows; 16 bytes per lane (D is a multiple of 8)
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ C, const int* __restrict__ perm,
                                                          int p0, int rows, int chunks_per_row,
                                                          uint4* __restrict__ out) {
  const int64_t total = (int64_t)rows * chunks_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / chunks_per_row), ch = (int)(i % chunks_per_row);
    out[i] = C[(int64_t)perm[p0 + r] * chunks_per_row + ch];
  }
}

}  // namespace

size_t vocab_sort_temp_bytes(int64_t V) {
  // bound on rocPRIM's radix-sort scratch for V (float key, int value) pairs: its own
  // alternate key / value buffers plus histograms; checked against the real figure at run time
  return (size_t)V * 16 + (1u << 20);
}

hipError_t vocab_sort_temp_needed(int64_t V, size_t* bytes) {
  const float* key = nullptr;
  float* key_out = nullptr;
  const int* val = nullptr;
  int* val_out = nullptr;
  *bytes = 0;
  return rocprim::radix_sort_pairs_desc((void*)nullptr, *bytes, key, key_out, val, val_out, (size_t)V, 0u, 32u,
                                        (hipStream_t) nullptr);
}

size_t vocab_sort_partial_bytes(int64_t D) { return (size_t)kMeanRowBlocks * (size_t)D * sizeof(float); }

hipError_t launch_vocab_sort(const VocabSortParams& p, hipStream_t stream) {
  dim3 g1((p.D + 255) / 256, kMeanRowBlocks);
  hipLaunchKernelGGL(col_sum_partial_kernel, g1, dim3(256), 0, stream, p.E, p.N, p.D, p.partial);
  hipLaunchKernelGGL(col_mean_kernel, dim3((p.D + 255) / 256), dim3(256), 0, stream, p.partial, p.N, p.D, p.mean);
  hipLaunchKernelGGL(mean_logit_kernel, dim3((p.V + 3) / 4), dim3(256), 0, stream, p.C, p.mean, p.V, p.D, p.key,
                     p.index);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  size_t need = 0;
  e = rocprim::radix_sort_pairs_desc((void*)nullptr, need, p.key, p.key_sorted, p.index, p.perm, (size_t)p.V, 0u, 32u,
                                     stream);
  if (e != hipSuccess) return e;
  if (need > p.temp_bytes) return hipErrorOutOfMemory;
  size_t have = p.temp_bytes;
  e = rocprim::radix_sort_pairs_desc(p.temp, have, p.key, p.key_sorted, p.index, p.perm, (size_t)p.V, 0u, 32u, stream);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(invert_perm_kernel, dim3((p.V + 255) / 256), dim3(256), 0, stream, p.perm, p.V, p.inverse);
  hipLaunchKernelGGL(remap_targets_kernel, dim3((p.N + 255) / 256), dim3(256), 0, stream, p.targets, p.N, p.V,
                     p.ignore_index, p.inverse, p.targets_sorted);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const bf16* C, const int* perm, int p0, int rows, int D, bf16* out, hipStream_t stream) {
  const int chunks = D / 8;
  const int64_t total = (int64_t)rows * chunks;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) return hipSuccess;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)C, perm, p0, rows,
                     chunks, (uint4*)out);
  return hipGetLastError();
}

}  // namespace cce
