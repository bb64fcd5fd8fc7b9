// Forward linear-log-sum-exp on MFMA (paper Section 4.2, Alg. 2), gfx950.
//
// A workgroup owns 256 tokens and a contiguous range of 256-wide vocabulary
// tiles.  For every vocabulary tile it forms the 256 x 256 logit tile in
// registers (rows = vocabulary, columns = tokens, see mfma_tile.h), applies the
// optional soft-cap, and folds the tile into a running (max, sum-exp) pair per
// token that never leaves registers.  Where Alg. 2 merges blocks of one token
// through a spin-lock on the global LSE vector, this kernel writes one
// (max, sum) partial per token per vocabulary split and a second tiny kernel
// merges them in a fixed order (bitwise reproducible).
#include "kernels.h"
#include "mfma_tile.h"

namespace cce {

// Soft-cap handling of the logit tile:
//   kNoCap    a = z
//   kCapFixed a = cap*tanh(z/cap) with cap <= 40: |a| <= cap, so cap itself serves as the
//             reference "maximum" and no running maximum is tracked (2^(-2*cap*log2e) is
//             still a normal float)
//   kCapMax   a = cap*tanh(z/cap), running maximum tracked like kNoCap
enum { kNoCap = 0, kCapFixed = 1, kCapMax = 2 };

// Fold one finished logit tile (this lane's 4 x 2 blocks) into the running base-2
// statistics m2 = max(a)*log2e and s = sum 2^(a*log2e - m2) of the lane's two token
// columns, and clear the accumulators.  RAGGED masks vocabulary rows >= V.
// REC additionally returns, per token column, the largest logit of the tile in base-2 units
// (a * log2(e)) over this lane's rows, for the block-maximum record.
template <int MODE, bool RAGGED, bool REC>
__device__ inline void fold_tile(f32x16 (&acc)[kRB][kCB], float (&m2)[kCB], float (&s)[kCB], int lane,
                                 int v_base, int V, float cap_scale, float cap_l2, float (&amax2)[kCB]) {
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    if (MODE == kCapFixed) {
      // a*log2e - cap*log2e = -2*cap_l2 / (1 + 2^(z*cap_scale))
      float sum = 0.f;
      float rmin = INFINITY;   // REC: the largest logit has the smallest r = 1 / (1 + 2^(z * cap_scale))
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float e = __builtin_amdgcn_exp2f(acc[rb][cb][i] * cap_scale);
          float r = __builtin_amdgcn_rcpf(1.f + e);
          float t = __builtin_amdgcn_exp2f(-2.f * cap_l2 * r);
          if (RAGGED && v_base + rb * 32 + acc_row(lane, i) >= V) {
            t = 0.f;
            r = INFINITY;
          }
          if (REC) rmin = fminf(rmin, r);
          sum += t;
          acc[rb][cb][i] = 0.f;
        }
      s[cb] += sum;
      m2[cb] = cap_l2;
      if (REC) amax2[cb] = rmin == INFINITY ? -INFINITY : fmaf(-2.f * cap_l2, rmin, cap_l2);
    } else if (MODE == kNoCap) {
      float tmax = -INFINITY;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          if (RAGGED && v_base + rb * 32 + acc_row(lane, i) >= V) acc[rb][cb][i] = -INFINITY;
          tmax = fmaxf(tmax, acc[rb][cb][i]);
        }
      if (REC) amax2[cb] = tmax * kLog2e;
      const float m_new = fmaxf(m2[cb], tmax * kLog2e);
      // a lane whose rows are all masked so far has m_new = -inf: subtract 0 instead, every
      // term is then 2^(-inf) = 0 and no inf - inf arises
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][cb][i], kLog2e, -m_ref));
          acc[rb][cb][i] = 0.f;
        }
      s[cb] = s[cb] * __builtin_amdgcn_exp2f(m2[cb] - m_ref) + sum;
      m2[cb] = m_new;
    } else {
      float tmax = -INFINITY;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float e = __builtin_amdgcn_exp2f(acc[rb][cb][i] * cap_scale);
          float r = __builtin_amdgcn_rcpf(1.f + e);
          float a2 = fmaf(-2.f * cap_l2, r, cap_l2);
          if (RAGGED && v_base + rb * 32 + acc_row(lane, i) >= V) a2 = -INFINITY;
          acc[rb][cb][i] = a2;
          tmax = fmaxf(tmax, a2);
        }
      if (REC) amax2[cb] = tmax;
      const float m_new = fmaxf(m2[cb], tmax);
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          sum += __builtin_amdgcn_exp2f(acc[rb][cb][i] - m_ref);
          acc[rb][cb][i] = 0.f;
        }
      s[cb] = s[cb] * __builtin_amdgcn_exp2f(m2[cb] - m_ref) + sum;
      m2[cb] = m_new;
    }
  }
}

// bf16 bit pattern of x rounded towards +infinity (never below x)
__device__ inline uint16_t bf16_round_up(float x) {
  const uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);     // inf / nan: keep
  return (uint16_t)((x >= 0.f ? u + 0xffffu : u) >> 16);                  // negative: truncation moves up
}

template <int MODE, bool REC>
__global__ __launch_bounds__(kThreads) void fwd_lse_mfma_kernel(FwdMfmaParams p) {
  __shared__ __attribute__((aligned(1024))) char lds[kLdsBytes3];   // five-slice operand ring

  TileCoords tc;
  tc.init();
  if (p.bad_targets && blockIdx.x == 0 && threadIdx.x == 0) *p.bad_targets = 0ull;   // the finalize kernel counts into it

  // each XCD works on a compact rectangle of (token tile, vocabulary split) pairs, so that
  // its L2 sees every E slice and C slice from several workgroups at about the same time
  const int n_tokens = p.n_dev ? *p.n_dev : p.N;   // ignored tokens may have been removed from E
  if (n_tokens <= 0) return;
  const SplitPlan plan = p.n_dev ? make_split_plan(n_tokens, p.v_tiles, p.want_wgs, p.round_cap) : p.plan;
  const int partial_stride = p.n_dev ? plan.n_tiles * kTileC : p.N;
  int n_tile, split;
  if (!xcd_map_decode(plan.map, blockIdx.x, n_tile, split)) return;
  // When all workgroups start together (one round of token tiles), odd vocabulary tiles walk K
  // backwards (see sweep_tiles).  With an odd number of tiles per split, splits s and s + 1 are
  // then on tiles of opposite parity at any moment; the splits are dealt to the XCD rectangles
  // so that those resident on one XCD have the same parity and its workgroups keep meeting on
  // the same E slices.  (With several rounds the workgroups of an XCD are out of step anyway
  // and the reversal only costs: measured 2 % at 64 token tiles.)
  const bool serpentine = plan.n_tiles <= p.round_cap;
  if (serpentine) {
    const int gb = plan.map.group_b, groups = plan.splits / gb;
    if ((plan.tiles_per_split & 1) && gb > 1 && (groups & 1) == 0) split = (split % gb) * groups + split / gb;
  }
  const int vt0 = split * plan.tiles_per_split;
  const int vt1 = min(vt0 + plan.tiles_per_split, p.v_tiles);
  const int n0 = n_tile * kTileC;
  const int64_t ld_bytes = (int64_t)p.D * 2;
  const int KT = p.D / kTileK;

  uint32_t offQ[4];
  dma_offsets(tc, min(kTileC, n_tokens - n0), ld_bytes, offQ);
  const char* gQ = (const char*)p.E + (int64_t)n0 * ld_bytes;

  // running statistics, base-2 domain: m2 = max(a) * log2(e), s = sum 2^(a*log2e - m2)
  float m2[kCB], s[kCB];
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) { m2[cb] = -INFINITY; s[cb] = 0.f; }

  f32x16 acc[kRB][kCB];
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  const float cap_scale = MODE != kNoCap ? 2.f * kLog2e / p.softcap : 0.f;   // exp(2z/cap) = 2^(z*cap_scale)
  const float cap_l2 = MODE != kNoCap ? p.softcap * kLog2e : kLog2e;

  sweep_tiles<REC ? 2 : 0, true>(tc, lds, (const char*)p.C, p.V, ld_bytes, vt0, vt1, gQ, offQ, KT, acc, [&](int vt) {
    // fold the finished logit tile into the running (max, sum)
    const int v_base = vt * kTileR + tc.wave_r * kWaveRows;
    float amax2[kCB] = {-INFINITY, -INFINITY};
    if ((vt + 1) * kTileR > p.V)
      fold_tile<MODE, true, REC>(acc, m2, s, tc.lane, v_base, p.V, cap_scale, cap_l2, amax2);
    else
      fold_tile<MODE, false, REC>(acc, m2, s, tc.lane, v_base, p.V, cap_scale, cap_l2, amax2);
    if (REC && v_base < p.V) {
      // this wave's 128 vocabulary rows are one block of the record: merge the two lane halves
      // and store one value per token (natural-log units, rounded up to bf16); 32-bit element
      // offsets keep the address in one register
      const uint32_t row = (uint32_t)(v_base / kWaveRows) * (uint32_t)p.block_max_stride +
                           (uint32_t)(n0 + tc.wave_c * kWaveCols + (tc.lane & 31));
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        const float a = fmaxf(amax2[cb], __shfl_xor(amax2[cb], 32)) * kLn2;
        if (tc.lane < 32) p.block_max[row + (uint32_t)(cb * 32)] = bf16_round_up(a);
      }
      return true;    // two stores, the last vector-memory operations issued
    }
    return false;
  }, serpentine);

  // ---- merge the two lane halves, then the two row-waves, and write the partial ----
  __syncthreads();
  float2* red = (float2*)lds;   // [2 row-waves][256 tokens]
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    float mo = __shfl_xor(m2[cb], 32);
    float so = __shfl_xor(s[cb], 32);
    float mn = fmaxf(m2[cb], mo);
    float sn = (mn == -INFINITY) ? 0.f
             : s[cb] * __builtin_amdgcn_exp2f(m2[cb] - mn) + so * __builtin_amdgcn_exp2f(mo - mn);   // 2^(-inf) = 0
    if (tc.lane < 32) {
      int col = tc.wave_c * kWaveCols + cb * 32 + tc.lane;
      red[tc.wave_r * kTileC + col] = make_float2(mn, sn);
    }
  }
  __syncthreads();
  if (threadIdx.x < kTileC) {
    int col = threadIdx.x;
    float2 a = red[col], b = red[kTileC + col];
    float mn = fmaxf(a.x, b.x);
    float sn = (mn == -INFINITY) ? 0.f
             : a.y * __builtin_amdgcn_exp2f(a.x - mn) + b.y * __builtin_amdgcn_exp2f(b.x - mn);
    int n = n0 + col;
    if (n < n_tokens) p.partial[(int64_t)split * partial_stride + n] = make_float2(mn, sn);
  }
}

hipError_t launch_fwd_lse_mfma(const FwdMfmaParams& p, hipStream_t stream) {
  dim3 grid(p.grid), block(kThreads);
  const int mode = p.softcap > 40.f ? kCapMax : p.softcap > 0.f ? kCapFixed : kNoCap;
#define CCE_LAUNCH_FWD(M, R) hipLaunchKernelGGL((fwd_lse_mfma_kernel<M, R>), grid, block, 0, stream, p)
  if (p.block_max) {
    if (mode == kCapMax) CCE_LAUNCH_FWD(kCapMax, true);
    else if (mode == kCapFixed) CCE_LAUNCH_FWD(kCapFixed, true);
    else CCE_LAUNCH_FWD(kNoCap, true);
  } else {
    if (mode == kCapMax) CCE_LAUNCH_FWD(kCapMax, false);
    else if (mode == kCapFixed) CCE_LAUNCH_FWD(kCapFixed, false);
    else CCE_LAUNCH_FWD(kNoCap, false);
  }
#undef CCE_LAUNCH_FWD
  return hipGetLastError();
}

}  // namespace cce
