// Plain fp32-FMA kernels: the path for float32 inputs and for shapes the MFMA
// kernels do not take (D not a multiple of 64), plus the small kernels both
// paths share (finalize / indexed dot product, dE store, counters).
//
// These are straightforward LDS-tiled kernels (64 x 64 output tile, 16-deep
// K steps, 4 x 4 outputs per lane); they follow the same algorithms as the MFMA
// path - Alg. 2 with per-split partials for the forward, Alg. 4 split into
// "form the gradient-of-logits slab" + two products for the backward - at the
// precision of fp32 FMA.
#include "cce.h"
#include "kernels.h"

namespace cce {

namespace {

constexpr int kT = 64;     // output tile edge
constexpr int kK = 16;     // contraction depth per step
constexpr int kBlock = 256;

template <typename T> __device__ inline float to_f(T x);
template <> __device__ inline float to_f<float>(float x) { return x; }
template <> __device__ inline float to_f<bf16>(bf16 x) { return (float)x; }

template <typename T> __device__ inline T from_f(float x);
template <> __device__ inline float from_f<float>(float x) { return x; }
template <> __device__ inline bf16 from_f<bf16>(float x) { return (bf16)x; }

// out[a][b] += sum_k  A(row0 + ty*4 + a, k) * B(col0 + tx*4 + b, k)   for k in [k0, k1)
// A(r, k) / B(c, k) are functors returning 0 outside their valid range.
template <class FA, class FB>
__device__ inline void tile_fma(float (&As)[kK][kT + 1], float (&Bs)[kK][kT + 1], int k0, int k1, FA A, FB B,
                                float (&out)[4][4]) {
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  for (int kk = k0; kk < k1; kk += kK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int idx = t + kBlock * j;
      int r = idx / kK, k = idx % kK;
      As[k][r] = A(r, kk + k);
      Bs[k][r] = B(r, kk + k);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) out[i][j] = fmaf(a[i], b[j], out[i][j]);
    }
    __syncthreads();
  }
}

__device__ inline float softcap_fn(float z, float cap) { return cap > 0.f ? cap * tanhf(z / cap) : z; }

// ------------------------------------------------------------------ forward
template <typename T>
__global__ __launch_bounds__(kBlock) void fwd_lse_plain_kernel(FwdPlainParams p) {
  __shared__ float As[kK][kT + 1], Bs[kK][kT + 1];
  __shared__ float Ls[kT][kT + 1];
  const T* E = (const T*)p.E;
  const T* C = (const T*)p.C;
  const int n0 = blockIdx.x * kT, split = blockIdx.y;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  if (p.bad_targets && blockIdx.x == 0 && blockIdx.y == 0 && t == 0) *p.bad_targets = 0ull;
  const int vt0 = split * p.tiles_per_split;
  const int v_tiles = (p.V + kT - 1) / kT;
  const int vt1 = min(vt0 + p.tiles_per_split, v_tiles);
  float m = -INFINITY, s = 0.f;   // thread t < 64 owns row n0 + t
  for (int vt = vt0; vt < vt1; ++vt) {
    const int v0 = vt * kT;
    float out[4][4] = {};
    auto A = [&](int r, int k) { int n = n0 + r; return (n < p.N && k < p.D) ? to_f<T>(E[(int64_t)n * p.D + k]) : 0.f; };
    auto B = [&](int c, int k) { int v = v0 + c; return (v < p.V && k < p.D) ? to_f<T>(C[(int64_t)v * p.D + k]) : 0.f; };
    tile_fma(As, Bs, 0, p.D, A, B, out);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int v = v0 + tx * 4 + j;
        Ls[ty * 4 + i][tx * 4 + j] = v < p.V ? softcap_fn(out[i][j], p.softcap) : -INFINITY;
      }
    __syncthreads();
    if (t < kT) {
      float tm = -INFINITY;
      for (int c = 0; c < kT; ++c) tm = fmaxf(tm, Ls[t][c]);
      float mn = fmaxf(m, tm);
      float acc = 0.f;
      for (int c = 0; c < kT; ++c) acc += expf(Ls[t][c] - mn);
      s = s * expf(m - mn) + acc;
      m = mn;
    }
    __syncthreads();
  }
  if (t < kT && n0 + t < p.N) p.partial[(int64_t)split * p.N + n0 + t] = make_float2(m * kLog2e, s);
}

// --------------------------------------------------- finalize + indexed dot (Alg. 1)
// One wavefront per token: merge the per-split partials into LSE_i, compute the
// target logit a_{i,x_i} = softcap(<E_i, C_{x_i}>) in fp32, and write the NLL.
template <typename T>
__global__ __launch_bounds__(kBlock) void finalize_kernel(FinalizeParams p) {
  const T* E = (const T*)p.E;
  const T* C = (const T*)p.C;
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
  int n_tokens = p.N, splits = p.splits, stride = p.N;
  if (p.n_dev) {
    // ignored tokens removed: the forward kernel planned its splits for the tokens present
    n_tokens = *p.n_dev;
    if (n >= n_tokens) return;
    const SplitPlan plan = make_split_plan(n_tokens, p.v_tiles, p.want_wgs, p.round_cap);
    splits = plan.splits;
    stride = plan.n_tiles * 256;
  }
  if (n >= n_tokens) return;
  const int o = p.idx ? p.idx[n] : n;    // the caller's index of this token
  float m2 = -INFINITY;
  for (int sp = lane; sp < splits; sp += 64) m2 = fmaxf(m2, p.partial[(int64_t)sp * stride + n].x);
  for (int o = 32; o > 0; o >>= 1) m2 = fmaxf(m2, __shfl_xor(m2, o));
  float s = 0.f;
  for (int sp = lane; sp < splits; sp += 64) {
    LsePartial q = p.partial[(int64_t)sp * stride + n];
    if (q.y > 0.f) s += q.y * exp2f(q.x - m2);
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  const float lse = (m2 + log2f(s)) * kLn2;
  const int64_t tgt = p.targets[o];
  const bool valid = tgt != p.ignore_index && tgt >= 0 && tgt < p.V;
  float dot = 0.f;
  if (valid) {
    const T* e = E + (int64_t)n * p.D;
    const T* c = C + tgt * p.D;
    for (int d = lane; d < p.D; d += 64) dot = fmaf(to_f<T>(e[d]), to_f<T>(c[d]), dot);
    for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
  }
  if (lane == 0) {
    p.out_lse[o] = lse;
    p.out_loss[o] = valid ? lse - softcap_fn(dot, p.softcap) : 0.f;
    if (p.bad_targets && !valid && tgt != p.ignore_index) atomicAdd(p.bad_targets, 1ull);   // integer count: order-free
  }
}

// ------------------------------------------------------------------ backward
// GZ slab: gz_ij = dloss_i * (exp(a_ij - lse_i) - [j == x_i]) * a'_ij, fp32 [N, vs].
template <typename T>
__global__ __launch_bounds__(kBlock) void bwd_gz_plain_kernel(BwdCommon c, BwdPlainSlab sl) {
  __shared__ float As[kK][kT + 1], Bs[kK][kT + 1];
  __shared__ int any_sig;
  const T* E = (const T*)c.E;
  const T* C = (const T*)c.C;
  const int n0 = blockIdx.x * kT, vl0 = blockIdx.y * kT, v0 = sl.v0 + vl0;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  if (t == 0) any_sig = 0;
  float out[4][4] = {};
  auto A = [&](int r, int k) { int n = n0 + r; return (n < c.N && k < c.D) ? to_f<T>(E[(int64_t)n * c.D + k]) : 0.f; };
  auto B = [&](int cc, int k) { int v = v0 + cc; return (v < c.V && k < c.D) ? to_f<T>(C[(int64_t)v * c.D + k]) : 0.f; };
  tile_fma(As, Bs, 0, c.D, A, B, out);
  bool sig = false;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = n0 + ty * 4 + i;
    if (n >= c.N) continue;
    const int64_t tgt = c.targets[n];
    const bool valid = tgt != c.ignore_index && tgt >= 0 && tgt < c.V;
    const float lse = c.lse[n];
    const float lam = valid ? c.dloss[n] : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int v = v0 + tx * 4 + j;
      float gz = 0.f;
      if (valid && v < c.V) {
        float a = out[i][j], dcap = 1.f;
        if (c.softcap > 0.f) {
          float th = tanhf(a / c.softcap);
          a = c.softcap * th;
          dcap = 1.f - th * th;
        }
        float g = expf(a - lse) - (v == tgt ? 1.f : 0.f);
        sig |= fabsf(g) >= c.eps;
        gz = lam * g * dcap;
      }
      sl.GZ[(int64_t)n * sl.vs + vl0 + tx * 4 + j] = gz;
    }
  }
  if (sig) any_sig = 1;
  __syncthreads();
  if (t == 0) {
    sl.flags[(int64_t)blockIdx.x * (sl.vs / kT) + blockIdx.y] = (uint8_t)any_sig;
    if (v0 < c.V) {
      atomicAdd(&c.stats->blocks_total, 1ull);
      if (any_sig) atomicAdd(&c.stats->blocks_kept, 1ull);
    }
  }
}

// dEacc[n, d] (+)= sum_v GZ[n, v] * C[v0 + v, d]
template <typename T>
__global__ __launch_bounds__(kBlock) void bwd_dE_plain_kernel(BwdCommon c, BwdPlainSlab sl) {
  __shared__ float As[kK][kT + 1], Bs[kK][kT + 1];
  const T* C = (const T*)c.C;
  const int n0 = blockIdx.x * kT, d0 = blockIdx.y * kT;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  float out[4][4] = {};
  const int nvb = sl.vs / kT;
  const bool use_flags = c.filter_dE && c.eps > 0.f;
  for (int vb = 0; vb < nvb; ++vb) {
    if (use_flags && !sl.flags[(int64_t)blockIdx.x * nvb + vb]) continue;   // block-uniform
    auto A = [&](int r, int k) { int n = n0 + r; return n < c.N ? sl.GZ[(int64_t)n * sl.vs + k] : 0.f; };
    auto B = [&](int cc, int k) {
      int d = d0 + cc, v = sl.v0 + k;
      return (d < c.D && v < c.V) ? to_f<T>(C[(int64_t)v * c.D + d]) : 0.f;
    };
    tile_fma(As, Bs, vb * kT, (vb + 1) * kT, A, B, out);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + ty * 4 + i, d = d0 + tx * 4 + j;
      if (n < c.N && d < c.D) {
        float* dst = sl.dEacc + (int64_t)n * c.D + d;
        *dst = sl.first ? out[i][j] : *dst + out[i][j];
      }
    }
}

// dC[v0 + v, d] = sum_n GZ[n, v] * E[n, d]
template <typename T>
__global__ __launch_bounds__(kBlock) void bwd_dC_plain_kernel(BwdCommon c, BwdPlainSlab sl, T* out_dC) {
  __shared__ float As[kK][kT + 1], Bs[kK][kT + 1];
  const T* E = (const T*)c.E;
  const int vl0 = blockIdx.x * kT, d0 = blockIdx.y * kT;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  float out[4][4] = {};
  const int nvb = sl.vs / kT;
  const int nnb = (c.N + kT - 1) / kT;
  const bool use_flags = c.filter_dC && c.eps > 0.f;
  for (int nb = 0; nb < nnb; ++nb) {
    if (use_flags && !sl.flags[(int64_t)nb * nvb + blockIdx.x]) continue;
    auto A = [&](int r, int k) { return k < c.N ? sl.GZ[(int64_t)k * sl.vs + vl0 + r] : 0.f; };
    auto B = [&](int cc, int k) { int d = d0 + cc; return (d < c.D && k < c.N) ? to_f<T>(E[(int64_t)k * c.D + d]) : 0.f; };
    tile_fma(As, Bs, nb * kT, (nb + 1) * kT, A, B, out);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int v = sl.v0 + vl0 + ty * 4 + i, d = d0 + tx * 4 + j;
      if (v < c.V && d < c.D) out_dC[(int64_t)v * c.D + d] = from_f<T>(out[i][j]);
    }
}

template <typename T, typename A>
__global__ void store_dE_kernel(const A* __restrict__ acc, int parts, T* __restrict__ out, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) {
    float v = to_f<A>(acc[i]);
    for (int p = 1; p < parts; ++p) v += to_f<A>(acc[(int64_t)p * count + i]);   // fixed order
    out[i] = from_f<T>(v);
  }
}

// ignored tokens removed: row k of acc belongs to the caller's token idx[k]
// (`parts` running sums were planned for the N tokens of the call; the kernels planned again for the tokens present)
template <typename T, typename A>
__global__ void scatter_dE_kernel(const A* __restrict__ acc, int parts, int64_t N, T* __restrict__ out,
                                  int64_t D, const int* __restrict__ idx, const int* __restrict__ n_dev) {
  const int64_t count = (int64_t)*n_dev * D;
  const DEParts pp = dE_parts_present(*n_dev, N, D, parts);
  parts = pp.parts;
  const int64_t part_stride = pp.stride;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) {
    const int64_t k = i / D, d = i % D;
    float v = to_f<A>(acc[i]);
    for (int p = 1; p < parts; ++p) v += to_f<A>(acc[(int64_t)p * part_stride + i]);
    out[(int64_t)idx[k] * D + d] = from_f<T>(v);
  }
}

template <typename T>
__global__ void fill_kernel(T* __restrict__ p, int64_t count, T value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) p[i] = value;
}

// Appendix B: the tokens that carry a loss, in order.  One workgroup walks the batch.
__global__ __launch_bounds__(1024) void compact_tokens_kernel(const int64_t* __restrict__ targets, int N, int V,
                                                              int64_t ignore_index, int* __restrict__ idx,
                                                              int* __restrict__ count,
                                                              unsigned long long* __restrict__ bad_targets) {
  __shared__ int wave_count[16];
  __shared__ int base_s;
  __shared__ int bad_s;
  if (threadIdx.x == 0) bad_s = 0;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base_s = 0;
  __syncthreads();
  for (int i0 = 0; i0 < N; i0 += 1024) {
    const int i = i0 + threadIdx.x;
    bool on = false, bad = false;
    if (i < N) {
      const int64_t t = targets[i];
      on = t != ignore_index && t >= 0 && t < V;
      bad = !on && t != ignore_index;
    }
    const uint64_t mask = __builtin_amdgcn_ballot_w64(on);
    const uint64_t bad_mask = __builtin_amdgcn_ballot_w64(bad);
    if (lane == 0) wave_count[wave] = __builtin_popcountll(mask);
    if (lane == 0 && bad_mask) atomicAdd(&bad_s, __builtin_popcountll(bad_mask));
    __syncthreads();
    int pos = base_s + __builtin_popcountll(mask & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) pos += wave_count[w];
    if (on) idx[pos] = i;
    __syncthreads();
    if (threadIdx.x == 0) {
      int total = 0;
      for (int w = 0; w < 16; ++w) total += wave_count[w];
      base_s += total;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *count = base_s;
    if (bad_targets) *bad_targets = (unsigned long long)bad_s;
  }
}

// out[k][:] = E[idx[k]][:] for k < *count, 16 bytes per lane
__global__ __launch_bounds__(256) void gather_tokens_kernel(const uint4* __restrict__ E, const int* __restrict__ idx,
                                                            const int* __restrict__ count, int chunks_per_row,
                                                            uint4* __restrict__ out) {
  const int64_t total = (int64_t)*count * chunks_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / chunks_per_row), ch = (int)(i % chunks_per_row);
    out[i] = E[(int64_t)idx[k] * chunks_per_row + ch];
  }
}

__global__ void clear_stats_kernel(FilterStats* s) {
  s->blocks_total = 0ull;
  s->blocks_kept = 0ull;
}

}  // namespace

hipError_t launch_fwd_lse_plain(const FwdPlainParams& p, hipStream_t stream) {
  dim3 grid((p.N + kT - 1) / kT, p.splits);
  if (p.dtype == CCE_F32)
    hipLaunchKernelGGL(fwd_lse_plain_kernel<float>, grid, dim3(kBlock), 0, stream, p);
  else
    hipLaunchKernelGGL(fwd_lse_plain_kernel<bf16>, grid, dim3(kBlock), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_finalize(const FinalizeParams& p, hipStream_t stream) {
  dim3 grid((p.N + 3) / 4);
  if (p.dtype == CCE_F32)
    hipLaunchKernelGGL(finalize_kernel<float>, grid, dim3(kBlock), 0, stream, p);
  else
    hipLaunchKernelGGL(finalize_kernel<bf16>, grid, dim3(kBlock), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_bwd_gz_plain(const BwdCommon& c, const BwdPlainSlab& s, hipStream_t stream) {
  dim3 grid((c.N + kT - 1) / kT, s.vs / kT);
  if (c.dtype == CCE_F32)
    hipLaunchKernelGGL(bwd_gz_plain_kernel<float>, grid, dim3(kBlock), 0, stream, c, s);
  else
    hipLaunchKernelGGL(bwd_gz_plain_kernel<bf16>, grid, dim3(kBlock), 0, stream, c, s);
  return hipGetLastError();
}

hipError_t launch_bwd_dE_plain(const BwdCommon& c, const BwdPlainSlab& s, hipStream_t stream) {
  dim3 grid((c.N + kT - 1) / kT, (c.D + kT - 1) / kT);
  if (c.dtype == CCE_F32)
    hipLaunchKernelGGL(bwd_dE_plain_kernel<float>, grid, dim3(kBlock), 0, stream, c, s);
  else
    hipLaunchKernelGGL(bwd_dE_plain_kernel<bf16>, grid, dim3(kBlock), 0, stream, c, s);
  return hipGetLastError();
}

hipError_t launch_bwd_dC_plain(const BwdCommon& c, const BwdPlainSlab& s, void* out_dC, hipStream_t stream) {
  dim3 grid(s.vs / kT, (c.D + kT - 1) / kT);
  if (c.dtype == CCE_F32)
    hipLaunchKernelGGL(bwd_dC_plain_kernel<float>, grid, dim3(kBlock), 0, stream, c, s, (float*)out_dC);
  else
    hipLaunchKernelGGL(bwd_dC_plain_kernel<bf16>, grid, dim3(kBlock), 0, stream, c, s, (bf16*)out_dC);
  return hipGetLastError();
}

hipError_t launch_store_dE(const float* dEacc, int parts, void* out_dE, int dtype, int64_t N, int64_t D,
                           const int* idx, const int* n_dev, bool acc_bf16, hipStream_t stream) {
  const int64_t count = N * D;
  int blocks = (int)((count + 1023) / 1024);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  const dim3 g(blocks), b(256);
  if (acc_bf16) {
    // bf16 running sums exist on the bf16 MFMA path only
    const bf16* acc = (const bf16*)dEacc;
    if (idx) {
      hipLaunchKernelGGL(fill_kernel<bf16>, g, b, 0, stream, (bf16*)out_dE, count, (bf16)0.f);
      hipLaunchKernelGGL((scatter_dE_kernel<bf16, bf16>), g, b, 0, stream, acc, parts, N, (bf16*)out_dE, D, idx, n_dev);
    } else {
      hipLaunchKernelGGL((store_dE_kernel<bf16, bf16>), g, b, 0, stream, acc, parts, (bf16*)out_dE, count);
    }
  } else if (idx) {
    if (dtype == CCE_F32) {
      hipLaunchKernelGGL(fill_kernel<float>, g, b, 0, stream, (float*)out_dE, count, 0.f);
      hipLaunchKernelGGL((scatter_dE_kernel<float, float>), g, b, 0, stream, dEacc, parts, N, (float*)out_dE, D, idx, n_dev);
    } else {
      hipLaunchKernelGGL(fill_kernel<bf16>, g, b, 0, stream, (bf16*)out_dE, count, (bf16)0.f);
      hipLaunchKernelGGL((scatter_dE_kernel<bf16, float>), g, b, 0, stream, dEacc, parts, N, (bf16*)out_dE, D, idx, n_dev);
    }
  } else if (dtype == CCE_F32) {
    hipLaunchKernelGGL((store_dE_kernel<float, float>), g, b, 0, stream, dEacc, parts, (float*)out_dE, count);
  } else {
    hipLaunchKernelGGL((store_dE_kernel<bf16, float>), g, b, 0, stream, dEacc, parts, (bf16*)out_dE, count);
  }
  return hipGetLastError();
}

hipError_t launch_compact_tokens(const int64_t* targets, int N, int V, int64_t ignore_index, int* idx, int* count,
                                 unsigned long long* bad_targets, hipStream_t stream) {
  hipLaunchKernelGGL(compact_tokens_kernel, dim3(1), dim3(1024), 0, stream, targets, N, V, ignore_index, idx, count,
                     bad_targets);
  return hipGetLastError();
}

hipError_t launch_gather_tokens(const bf16* E, const int* idx, const int* count, int N, int D, bf16* out,
                                hipStream_t stream) {
  const int chunks = D / 8;
  int64_t blocks = ((int64_t)N * chunks + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(gather_tokens_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)E, idx, count,
                     chunks, (uint4*)out);
  return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t stream) {
  int blocks = (int)((count + 1023) / 1024);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fill_kernel<float>, dim3(blocks), dim3(256), 0, stream, p, count, value);
  return hipGetLastError();
}

hipError_t launch_clear_stats(FilterStats* stats, hipStream_t stream) {
  hipLaunchKernelGGL(clear_stats_kernel, dim3(1), dim3(1), 0, stream, stats);
  return hipGetLastError();
}

}  // namespace cce
