/* A plain C99 user of the library on a real GPU: no Python, no PyTorch.  The program owns every buffer
 * (hipMalloc here, in the caller), lends the library its scratch with cce_set_workspace and calls the two
 * plain entry points.  Inputs are chosen so that the results have closed forms:
 *   C = 0                =>  every logit is 0: LSE_i = loss_i = log |V| (ignored tokens: loss 0)
 *   E_i = (1, 1, ..., 1) =>  dE = 0 and dC_j[d] = lambda * (N_valid / |V| - #{i : x_i = j})  for every d
 * Built and run by tests/test_abi_gpu.py. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "cce.h"

#define HIP_OK(call)                                                         \
  do {                                                                       \
    hipError_t e_ = (call);                                                  \
    if (e_ != hipSuccess) {                                                  \
      printf("FAILED %s: %s\n", #call, hipGetErrorString(e_));               \
      return 2;                                                              \
    }                                                                        \
  } while (0)

static float bf16_to_float(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

int main(void) {
  const int64_t N = 700, D = 128, V = 1500, ignore_index = -100;
  const size_t e_bytes = (size_t)N * D * 2, c_bytes = (size_t)V * D * 2;
  uint16_t* hE = (uint16_t*)malloc(e_bytes);
  int64_t* hx = (int64_t*)malloc((size_t)N * 8);
  float* hlam = (float*)malloc((size_t)N * 4);
  int* count = (int*)calloc((size_t)V, sizeof(int));
  int n_valid = 0;
  for (int64_t i = 0; i < N * D; ++i) hE[i] = 0x3f80; /* bf16 1.0 */
  for (int64_t i = 0; i < N; ++i) {
    hx[i] = (i % 10 == 3) ? ignore_index : (i * 37) % V;
    if (hx[i] != ignore_index) { ++n_valid; ++count[hx[i]]; }
  }
  const float lambda = 1.0f / (float)n_valid;
  for (int64_t i = 0; i < N; ++i) hlam[i] = lambda;

  void *E, *C, *x, *loss, *lse, *lam, *dE, *dC, *ws;
  cce_opts o;
  cce_default_opts(CCE_BF16, &o);
  const size_t ws_bytes = cce_workspace_bytes(CCE_OP_BACKWARD, N, D, V, &o);
  HIP_OK(hipMalloc(&E, e_bytes));
  HIP_OK(hipMalloc(&C, c_bytes));
  HIP_OK(hipMalloc(&x, (size_t)N * 8));
  HIP_OK(hipMalloc(&loss, (size_t)N * 4));
  HIP_OK(hipMalloc(&lse, (size_t)N * 4));
  HIP_OK(hipMalloc(&lam, (size_t)N * 4));
  HIP_OK(hipMalloc(&dE, e_bytes));
  HIP_OK(hipMalloc(&dC, c_bytes));
  HIP_OK(hipMalloc(&ws, ws_bytes));
  HIP_OK(hipMemcpy(E, hE, e_bytes, hipMemcpyHostToDevice));
  HIP_OK(hipMemset(C, 0, c_bytes));
  HIP_OK(hipMemcpy(x, hx, (size_t)N * 8, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(lam, hlam, (size_t)N * 4, hipMemcpyHostToDevice));

  /* without a lent workspace the plain calls refuse */
  int st = cce_forward(E, C, (const int64_t*)x, N, D, V, 0.0f, ignore_index, (float*)loss, (float*)lse);
  if (st != CCE_EWORKSPACE) { printf("FAILED: expected CCE_EWORKSPACE, got %d\n", st); return 3; }
  st = cce_set_workspace(ws, ws_bytes);
  if (st != CCE_OK) { printf("FAILED cce_set_workspace: %s\n", cce_strerror(st)); return 3; }
  st = cce_forward(E, C, (const int64_t*)x, N, D, V, 0.0f, ignore_index, (float*)loss, (float*)lse);
  if (st != CCE_OK) { printf("FAILED cce_forward: %s\n", cce_strerror(st)); return 3; }
  st = cce_backward(E, C, (const int64_t*)x, N, D, V, 0.0f, ignore_index, (const float*)lse, (const float*)lam, dE, dC);
  if (st != CCE_OK) { printf("FAILED cce_backward: %s\n", cce_strerror(st)); return 3; }
  HIP_OK(hipDeviceSynchronize());

  float* hloss = (float*)malloc((size_t)N * 4);
  float* hlse = (float*)malloc((size_t)N * 4);
  uint16_t* hdE = (uint16_t*)malloc(e_bytes);
  uint16_t* hdC = (uint16_t*)malloc(c_bytes);
  HIP_OK(hipMemcpy(hloss, loss, (size_t)N * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hlse, lse, (size_t)N * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hdE, dE, e_bytes, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hdC, dC, c_bytes, hipMemcpyDeviceToHost));
  const float logV = logf((float)V);
  for (int64_t i = 0; i < N; ++i) {
    const float want = hx[i] == ignore_index ? 0.0f : logV;
    if (fabsf(hlse[i] - logV) > 1e-4f || fabsf(hloss[i] - want) > 1e-4f) {
      printf("FAILED token %lld: lse %g loss %g, expected %g / %g\n", (long long)i, hlse[i], hloss[i], logV, want);
      return 4;
    }
  }
  for (int64_t i = 0; i < N * D; ++i)
    if (fabsf(bf16_to_float(hdE[i])) > 1e-7f) { printf("FAILED dE[%lld] = %g, expected 0\n", (long long)i, bf16_to_float(hdE[i])); return 5; }
  for (int64_t j = 0; j < V; ++j) {
    const float want = lambda * ((float)n_valid / (float)V - (float)count[j]);
    for (int64_t d = 0; d < D; d += 17) {
      const float got = bf16_to_float(hdC[j * D + d]);
      if (fabsf(got - want) > 1e-2f * fabsf(want) + 1e-9f) {   /* bf16 storage of GZ and of the result */
        printf("FAILED dC[%lld][%lld] = %g, expected %g\n", (long long)j, (long long)d, got, want);
        return 6;
      }
    }
  }
  uint64_t total = 0, kept = 0, bad = 0;
  if (cce_backward_filter_stats(NULL, NULL, &total, &kept) != CCE_OK || total == 0 || kept > total) return 7;
  if (cce_set_workspace(NULL, 0) != CCE_OK) return 8;
  (void)bad;
  printf("gpu run ok: lse = loss = log %lld = %.6f on %d valid tokens, dE = 0, dC closed form, %llu / %llu filter blocks kept\n",
         (long long)V, logV, n_valid, (unsigned long long)kept, (unsigned long long)total);
  return 0;
}
