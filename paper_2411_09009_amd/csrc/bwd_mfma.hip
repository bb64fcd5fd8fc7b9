// Backward pass on MFMA (paper Alg. 4, merged linear-cross-entropy backward), gfx950.
//
// The algorithm of the paper walks all (token block, vocabulary block) pairs,
// recomputes the logit block, forms G = softmax - onehot, and immediately adds
// the block's contribution to dE and dC in global memory under locks.  On this
// chip a dense sweep of that form is bound by the read-modify-write traffic of
// the two fp32 output tiles, so the pass is restructured around vocabulary
// slabs; within a slab
//   1. recompute kernel: logit tiles as in the forward pass, then
//      gz = dloss * (exp(a - lse) - onehot) * a'  written once as bf16,
//      token-major (GZ [Np, vs]), plus block flags for the gradient filter;
//   2. dC[slab] = GZ^T E product (contraction over tokens), final after one pass;
//   3. dE += GZ C[slab] product (contraction over the slab), accumulated in fp32
//      across slabs by plain (exclusive-owner) read-modify-write.
// All three run on the same MFMA tile engine (mfma_tile.h).  Operands whose
// contracted index is not contiguous in memory (E and GZ over tokens, the rows of C
// over the vocabulary) are read in place as "K-major" operands through the LDS
// transposing reads; nothing is transposed in memory.
#include "kernels.h"
#include "mfma_tile.h"

#include <type_traits>

namespace cce {

namespace {

// ------------------------------------------------------------------ tiles that cannot be skipped
// A 256-token x 256-vocabulary tile needs recomputing only if some valid token of it has a
// softmax entry that can reach the filter threshold, S_ij = exp(a_ij - lse_i) >= eps, or has
// its target inside the tile (|G| = 1 - S there).  max_j a_ij over 128-wide blocks comes from
// the forward pass (rounded up), so the test never skips a tile the filter would keep.
__global__ __launch_bounds__(256) void tile_flag_kernel(TileListParams p) {
  const int vt = blockIdx.x, nt = blockIdx.y;
  const int tok = nt * 256 + threadIdx.x;
  const int n_tokens = p.n_dev ? *p.n_dev : p.N;
  bool sig = false;
  if (tok < n_tokens) {
    const int orig = p.idx ? p.idx[tok] : tok;
    const int64_t t = p.targets[orig];
    if (t != p.ignore_index && t >= 0 && t < p.V) {
      const int b0 = vt * 2, blocks = (p.V + 127) / 128;
      uint32_t u0 = p.block_max[(int64_t)b0 * p.stride + tok];
      float a = __uint_as_float(u0 << 16);
      if (b0 + 1 < blocks) {
        uint32_t u1 = p.block_max[(int64_t)(b0 + 1) * p.stride + tok];
        a = fmaxf(a, __uint_as_float(u1 << 16));
      }
      sig = (a - p.lse[orig] >= p.log_eps) || (t >= (int64_t)vt * 256 && t < (int64_t)vt * 256 + 256);
    }
  }
  const bool any = __syncthreads_or(sig);
  if (threadIdx.x == 0) p.tile_flag[(int64_t)nt * p.v_tiles + vt] = any ? 1 : 0;
}

// one workgroup per slab: compact the slab's flagged tiles, token-tile major
__global__ __launch_bounds__(256) void tile_compact_kernel(TileListParams p) {
  __shared__ int wave_count[4];
  __shared__ int base_s;
  const int slab = blockIdx.x;
  const int vt0 = slab * p.slab_tiles;
  const int tiles_here = min(p.slab_tiles, p.v_tiles - vt0);
  const int total = p.n_tiles * tiles_here;
  uint32_t* list = p.tile_list + (int64_t)slab * p.n_tiles * p.slab_tiles;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base_s = 0;
  __syncthreads();
  for (int i0 = 0; i0 < total; i0 += 256) {
    const int i = i0 + threadIdx.x;
    const int nt = i / tiles_here, tl = i % tiles_here;
    const bool on = i < total && p.tile_flag[(int64_t)nt * p.v_tiles + vt0 + tl] != 0;
    const uint64_t mask = __builtin_amdgcn_ballot_w64(on);
    if (lane == 0) wave_count[wave] = __builtin_popcountll(mask);
    __syncthreads();
    int pos = base_s + __builtin_popcountll(mask & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) pos += wave_count[w];
    if (on) list[pos] = ((uint32_t)nt << 16) | (uint32_t)tl;
    __syncthreads();
    if (threadIdx.x == 0) base_s += wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
    __syncthreads();
  }
  if (threadIdx.x == 0) p.tile_count[slab] = (uint32_t)base_s;
}

enum { kNoCap = 0, kCap = 1 };
enum { kAccF32 = 0, kAccBf16 = 1, kAccBf16Kahan = 2 };
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int kMaxKSteps = 2048;   // longest filtered contraction: 131072 / 64

// ------------------------------------------------------------------ recompute + G
// LIST: the workgroup takes an equal share of the slab's work list (tiles the filter cannot
// skip) instead of a fixed rectangle of tiles.
template <int MODE, bool LIST>
__global__ __launch_bounds__(kThreads) void bwd_recompute_mfma_kernel(BwdCommon c, BwdMfmaSlab sl, SplitPlan plan,
                                                                      int want_wgs) {
  __shared__ __attribute__((aligned(1024))) char lds[kLdsBytes + 8 * 4096];   // operand ring + store staging
  TileCoords tc;
  tc.init();
  if (c.n_dev) c.N = *c.n_dev;   // ignored tokens removed: E holds this many tokens
  const int v_tiles = sl.vs / kTileR;
  const int64_t ld_bytes = (int64_t)c.D * 2;
  const int KT = c.D / kTileK;
  int n_tile = 0, t0 = 0, t1 = 0;   // fixed rectangle: token tile and vocabulary tile range
  int e0 = 0, e1 = 0;               // work list: entry range
  if (LIST) {
    // consecutive entries share a token tile: give each XCD a run of consecutive shares
    const int groups = (int)gridDim.x, per_xcd = groups / kXcds;
    const int logical = ((int)blockIdx.x % kXcds) * per_xcd + (int)blockIdx.x / kXcds;
    const int count = (int)*sl.tile_count;
    e0 = (int)((int64_t)logical * count / groups);        // shares differ by at most one entry
    e1 = (int)((int64_t)(logical + 1) * count / groups);
    if (e0 >= e1) return;
    n_tile = (int)(sl.tile_list[e0] >> 16);
  } else {
    if (c.n_dev) {
      if (c.N <= 0) return;
      plan = make_split_plan(c.N, v_tiles, want_wgs, 1 << 30);   // planned again for the tokens present
    }
    int split;
    if (!xcd_map_decode(plan.map, blockIdx.x, n_tile, split)) return;
    t0 = split * plan.tiles_per_split;
    t1 = min(t0 + plan.tiles_per_split, v_tiles);
  }
  int n0 = n_tile * kTileC;

  // per-lane token data for the lane's two token columns of token tile `n_tile`
  float lse2[kCB], lam[kCB];
  int tgt[kCB], ncol[kCB];
  auto load_tokens = [&]() {
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      const int n = n0 + tc.wave_c * kWaveCols + cb * 32 + (tc.lane & 31);
      ncol[cb] = n;
      // a token that takes no part (ignored, target out of range, past N): with lse = +inf every
      // 2^(a - lse) of its column is exactly 0, so its column of G needs no masking below
      lse2[cb] = INFINITY;
      lam[cb] = 0.f;
      tgt[cb] = -1;
      if (n < c.N) {
        const int o = c.idx ? c.idx[n] : n;
        const int64_t t = c.targets[o];
        if (t != c.ignore_index && t >= 0 && t < c.V) {
          tgt[cb] = (int)t;
          lam[cb] = c.dloss[o];
          lse2[cb] = c.lse[o] * kLog2e;
        }
      }
    }
  };
  load_tokens();

  f32x16 acc[kRB][kCB];
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  const float cap_scale = MODE == kCap ? 2.f * kLog2e / c.softcap : 0.f;
  const float cap_l2 = MODE == kCap ? c.softcap * kLog2e : kLog2e;
  const float eps = c.eps;
  const char* P = (const char*)sl.Crows;

  // Staging area for the token-major store: 4 KB per wave beyond the operand ring.  A lane
  // owns one token column of the logit tile, so written straight from registers the
  // token-major copy would touch 64 different rows per store instruction; through LDS a
  // store instruction covers 8 rows x 128 contiguous bytes instead.  The 32 x 128 B staging
  // tile uses the ring's swizzle (16-byte chunk c of row r at position c ^ ((r >> 1) & 7)).
  // Wave-private, accessed through inline assembly like the ring (see mfma_tile.h); the
  // LDS executes one wave's accesses in order, so a read sees the writes issued before it.
  const uint32_t stage_base = lds_addr(lds) + kLdsBytes + (uint32_t)tc.wave * 4096u;
  const uint32_t st_row = (uint32_t)(tc.lane & 31), st_half = (uint32_t)(tc.lane >> 5);
  const uint32_t st_wr = stage_base + st_row * 128u + st_half * 8u;       // + ((chunk ^ swz) * 16)
  const uint32_t st_wswz = (st_row >> 1) & 7u;
  // read side: instruction rr covers rows rr * 8 + lane / 8, logical chunk lane % 8
  const uint32_t rd_row = (uint32_t)(tc.lane >> 3), rd_chunk = (uint32_t)(tc.lane & 7);

  // G and GZ of one of the lane's two token columns (cb): 4 blocks x 16 rows.  Straight-line
  // code: the 64 elements are independent chains the scheduler interleaves.  CAREFUL adds what
  // few column blocks need: the onehot term (a target inside the wave's 128 rows) and the mask of
  // rows past |V| (last vocabulary tile).  gmax[h] collects max |G| over rows h * 64 .. h * 64 + 63.
  auto column = [&](auto careful_tag, int cb, int vl_base, float (&gmax)[2]) {
    constexpr bool CAREFUL = decltype(careful_tag)::value;
    const float l2 = lse2[cb], lm = lam[cb];
    const int tg = tgt[cb];
#pragma unroll
    for (int rbp = 0; rbp < 2; ++rbp) {
#pragma unroll
      for (int rbl = 0; rbl < 2; ++rbl) {
        const int rb = rbp * 2 + rbl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float gz[4];
          const int v = sl.v0 + vl_base + rb * 32 + 8 * g + 4 * (tc.lane >> 5);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float z = acc[rb][cb][g * 4 + j];
            acc[rb][cb][g * 4 + j] = 0.f;
            float x, dcap;
            if (MODE == kCap) {
              const float e = __builtin_amdgcn_exp2f(z * cap_scale);
              const float r = __builtin_amdgcn_rcpf(1.f + e);
              const float th = fmaf(-2.f, r, 1.f);           // tanh(z / cap)
              x = fmaf(cap_l2, th, -l2);
              dcap = fmaf(-th, th, 1.f);
            } else {
              x = fmaf(z, kLog2e, -l2);
              dcap = 1.f;
            }
            float gval = __builtin_amdgcn_exp2f(x);
            if (CAREFUL) {
              gval -= (v + j == tg) ? 1.f : 0.f;
              // rows past |V|: cleared by a bit mask, which keeps the arithmetic above unconditional
              const uint32_t keep = (v + j < c.V) ? 0xffffffffu : 0u;
              gval = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, gval) & keep);
            }
            gmax[rbp] = fmaxf(gmax[rbp], fabsf(gval));
            gz[j] = MODE == kCap ? lm * gval * dcap : lm * gval;
          }
          f32x2 lo = {gz[0], gz[1]}, hi = {gz[2], gz[3]};
          bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
          uint2 packed;
          packed.x = __builtin_bit_cast(uint32_t, blo);
          packed.y = __builtin_bit_cast(uint32_t, bhi);
          // staging row = token (lane & 31), 16-byte chunk = rbl * 4 + g, half = lane >> 5
          const uint32_t wa = st_wr + ((((uint32_t)(rbl * 4 + g)) ^ st_wswz) << 4);
          asm volatile("ds_write_b64 %0, %1" ::"v"(wa), "v"(packed));
        }
      }
      // 32 tokens x 64 vocabulary entries are staged: write them out, 128 contiguous bytes per token.
      // Instruction rr covers staging rows rr * 8 + lane / 8; the four reads are issued together
      // and waited for once.
      u32x4 val[4];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const uint32_t row = (uint32_t)rr * 8u + rd_row;
        const uint32_t ra = stage_base + row * 128u + ((rd_chunk ^ ((row >> 1) & 7u)) << 4);
        asm volatile("ds_read_b128 %0, %1" : "=v"(val[rr]) : "v"(ra));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(val[0]), "+v"(val[1]), "+v"(val[2]), "+v"(val[3]));
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        // token of this staging row: same wave column block, row-th of the 32 tokens of cb.
        // The address is derived from an opaque copy so that it is computed here and not
        // hoisted out of the tile loop into registers that stay live across the MFMA stages.
        uint32_t tok_row = (uint32_t)(n0 + tc.wave_c * kWaveCols + cb * 32) + (uint32_t)rr * 8u + rd_row;
        asm volatile("" : "+v"(tok_row));
        bf16* dst = sl.GZ + ((size_t)tok_row * (uint32_t)sl.vs + (uint32_t)(vl_base + rbp * 64) + rd_chunk * 8u);
        *(u32x4*)dst = val[rr];
      }
    }
  };

  auto epilogue = [&](int t) {
    const int vl_base = t * kTileR + tc.wave_r * kWaveRows;   // slab-local vocabulary row of this wave
    const int v_wave = sl.v0 + vl_base;
    const bool ragged = v_wave + kWaveRows > c.V;              // wave-uniform
    float gmax[2] = {0.f, 0.f};                                // halves rb {0,1} and {2,3}
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      const bool target_here = (uint32_t)(tgt[cb] - v_wave) < (uint32_t)kWaveRows;
      if (ragged || __builtin_amdgcn_ballot_w64(target_here) != 0) column(std::true_type{}, cb, vl_base, gmax);
      else column(std::false_type{}, cb, vl_base, gmax);
    }
    bool sig[2];
    if (eps > 0.f) {
      sig[0] = gmax[0] >= eps;
      sig[1] = gmax[1] >= eps;
    } else {
      // filter off: a block counts as kept when it holds an element of a token that takes part
      const bool tok = tgt[0] >= 0 || tgt[1] >= 0;
      sig[0] = tok && v_wave < c.V;
      sig[1] = tok && v_wave + 64 < c.V;
    }
    // block flags for the gradient filter (an OR, so the order of arrival is immaterial)
    const bool any0 = __builtin_amdgcn_ballot_w64(sig[0]) != 0;
    const bool any1 = __builtin_amdgcn_ballot_w64(sig[1]) != 0;
    if (tc.lane == 0) {
      const int vsteps = sl.vs / 64;
      uint32_t* f_nv = sl.flags_nv + (int64_t)n_tile * vsteps + t * 4 + tc.wave_r * 2;
      if (any0) atomicOr(f_nv, 1u);
      if (any1) atomicOr(f_nv + 1, 1u);
      if (any0 || any1) atomicOr(sl.flags_vn + (int64_t)t * (sl.Np / 64) + n_tile * 4 + tc.wave_c, 1u);
    }
    return true;   // the 16 staged stores (and up to 3 flag updates after them) are this wave's last memory operations
  };

  if (LIST) {
    const int slab_rows = c.V - sl.v0;
    sweep_entries<16>(
        tc, lds, e0, e1, KT, acc,
        [&](int e, const char*& gP, uint32_t (&offP)[4], const char*& gQ, uint32_t (&offQ)[4]) {
          const uint32_t entry = sl.tile_list[e];
          const int nt = (int)(entry >> 16), tl = (int)(entry & 0xffffu);
          gP = P + (int64_t)tl * kTileR * ld_bytes;
          dma_offsets(tc, min(kTileR, slab_rows - tl * kTileR), ld_bytes, offP);
          gQ = (const char*)c.E + (int64_t)nt * kTileC * ld_bytes;
          dma_offsets(tc, min(kTileC, c.N - nt * kTileC), ld_bytes, offQ);
        },
        [&](int e) {
          const uint32_t entry = sl.tile_list[e];
          const int nt = (int)(entry >> 16);
          if (nt != n_tile) {
            n_tile = nt;
            n0 = nt * kTileC;
            load_tokens();
          }
          return epilogue((int)(entry & 0xffffu));
        });
  } else {
    uint32_t offQ[4];
    dma_offsets(tc, min(kTileC, c.N - n0), ld_bytes, offQ);
    const char* gQ = (const char*)c.E + (int64_t)n0 * ld_bytes;
    sweep_tiles<16>(tc, lds, P, c.V - sl.v0, ld_bytes, t0, t1, gQ, offQ, KT, acc, epilogue);
  }
}

// ------------------------------------------------------------------ gradient products
// out tile [256 d x 256 c]:  acc[d][c] = sum_k P[d][k] * Q[c][k],  k stepping over 64-wide
// blocks; with FILTERED only the blocks whose flag (row tile_c of `flags`) is set.
//   DC = false:  P = C slab [vs, D] (K-major), Q = GZ [Np, vs] rows,      c = token      -> dEacc[c][d] (+)= acc
//   DC = true :  P = E [N, D] (K-major),       Q = GZ [Np, vs] (K-major), c = vocabulary -> dC[v0 + c][d] = bf16(acc)
// ACC (dE only): how the sum over vocabulary slabs is kept in device memory between launches:
//   kAccF32        fp32 accumulator (this library's default)
//   kAccBf16       bf16 accumulator: the running sum is rounded to the gradient's storage type after every
//                  slab, as the paper's kernels do for their sums in global memory (Section 5)
//   kAccBf16Kahan  bf16 accumulator plus a bf16 compensation term (the paper's "CCE-Kahan")
template <bool DC, bool FILTERED, int ACC = kAccF32>
__global__ __launch_bounds__(kThreads) void bwd_product_mfma_kernel(BwdCommon c, BwdMfmaSlab sl, bf16* out_dC,
                                                                    XcdMap map) {
  __shared__ __attribute__((aligned(1024))) char lds[kLdsBytes];
  __shared__ uint16_t klist[kMaxKSteps];
  __shared__ int kcount_s;
  TileCoords tc;
  tc.init();
  // dE of a small batch has fewer tiles than CUs: the slab's K steps are then cut into ksplit
  // parts, each with its own running sum (added up when dE is stored)
  int ksplit = sl.ksplit;
  int64_t part_stride = sl.dE_part_stride;
  if (c.n_dev) {
    // ignored tokens removed: E and GZ hold this many tokens, and the dE product is planned again for them
    const int n_all = c.N;
    c.N = *c.n_dev;
    if (!DC) {
      if (c.N <= 0) return;   // no token present: dE is zeroed when it is stored (dC still writes its zeros below)
      const DEParts pp = dE_parts_present(c.N, n_all, c.D, sl.ksplit);
      ksplit = pp.parts;
      part_stride = pp.stride;
      map = make_xcd_map(map.dim_a, ((c.N + kTileC - 1) / kTileC) * ksplit);
    }
  }
  int tile_r, tile_c;   // a = 256-wide slice of D, b = token tile x part of the slab (dE) or vocabulary tile (dC)
  if (!xcd_map_decode(map, blockIdx.x, tile_r, tile_c)) return;
  const int part = DC ? 0 : tile_c % ksplit;
  if (!DC) tile_c /= ksplit;
  const int d0 = tile_r * kTileR, c0 = tile_c * kTileC;
  if (!DC && c0 >= c.N) return;   // a token tile past the tokens present
  // token tiles past the tokens present were not recomputed: the contraction over tokens stops before them
  const int K = DC ? (c.N + kTileC - 1) / kTileC * kTileC : sl.vs;
  // P is always K-major: E [N, D] contracted over tokens (dC) or the slab's rows of C [vs, D]
  // contracted over the vocabulary (dE); its tile is columns d0 .. d0 + 255 of every K-row.
  // Q is GZ [Np, vs]: K-major for dC (columns = vocabulary tile), K-contiguous for dE (rows = token tile).
  const uint32_t ldP = (uint32_t)c.D * 2u, ldQ = (uint32_t)sl.vs * 2u;
  const char* P = (const char*)(DC ? c.E : (const void*)sl.Crows) + (int64_t)d0 * 2;
  const int kP_last = DC ? c.N - 1 : min(sl.vs, c.V - sl.v0) - 1;   // K-rows past the operand's end repeat the last one
                                                                     // (the matching GZ entries are zero)
  const char* Q = (const char*)sl.GZ + (DC ? (int64_t)c0 * 2 : (int64_t)c0 * ldQ);
  const int ksteps = K / kTileK;
  const int steps_per_part = DC ? ksteps : (ksteps + ksplit - 1) / ksplit;
  const int k_lo = min(ksteps, part * steps_per_part), k_hi = min(ksteps, k_lo + steps_per_part);

  int kcount = k_hi - k_lo;
  if (FILTERED) {
    const uint32_t* flags = (DC ? sl.flags_vn : sl.flags_nv) + (int64_t)tile_c * ((DC ? sl.Np : sl.vs) / kTileK);
    if (tc.wave == 0) {
      int count = 0;
      for (int base = k_lo; base < k_hi; base += 64) {
        int idx = base + tc.lane;
        bool on = idx < k_hi && flags[idx] != 0;
        uint64_t mask = __builtin_amdgcn_ballot_w64(on);
        int pos = count + __builtin_popcountll(mask & ((1ull << tc.lane) - 1ull));
        if (on) klist[pos] = (uint16_t)idx;
        count += __builtin_popcountll(mask);
      }
      if (tc.lane == 0) kcount_s = count;
    }
    __syncthreads();
    kcount = __builtin_amdgcn_readfirstlane(kcount_s);
  }

  f32x16 acc[kRB][kCB];
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.f;

  if (kcount > 0) {
    KMajorLane laneP, laneQ;
    laneP.init(tc, min(32, (c.D - d0) / 8));
    uint32_t offQ[4];
    if (DC) laneQ.init(tc, 32);
    else dma_offsets(tc, kTileC, ldQ, offQ);     // GZ rows are padded to full tiles in the workspace
    const uint32_t klist_addr = lds_addr(klist);
    int cursor = 0;
    mma_pipeline<true, DC>(
        tc, lds, kcount, acc,
        [&](StageSrc& src) {
          int kstep = k_lo + cursor;
          if (FILTERED) {
            // the list lives in LDS; read it past the compiler (it would otherwise wait for
            // every direct load in flight before any LDS access it can see)
            uint32_t v;
            asm volatile("ds_read_u16 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(klist_addr + 2u * (uint32_t)cursor));
            kstep = __builtin_amdgcn_readfirstlane((int)v);
          }
          if (cursor + 1 < kcount) ++cursor;   // past the end: surplus loads repeat the last step
          src.gP = P;
          laneP.offsets(kstep * kTileK, kP_last, ldP, src.offP);
          if (DC) {
            src.gQ = Q;
            laneQ.offsets(kstep * kTileK, sl.Np - 1, ldQ, src.offQ);
          } else {
            src.gQ = Q + (int64_t)kstep * (kTileK * 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) src.offQ[j] = offQ[j];
          }
        },
        [&](int) { return false; });
  }

  // rows of dC go back to their original vocabulary index when the slab was walked in sorted order
  int out_row[kCB] = {0, 0};
  if (DC) {
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      const int vv = sl.v0 + c0 + tc.wave_c * kWaveCols + cb * 32 + (tc.lane & 31);
      out_row[cb] = (sl.perm && vv < c.V) ? sl.perm[vv] : vv;
    }
  }
  // D is a multiple of 64, so each of the wave's four 32-row blocks lies inside D or outside as a whole
  const int d_wave = d0 + tc.wave_r * kWaveRows;
  const int rb_valid = (c.D - d_wave) / 32;   // blocks inside D (may be <= 0 or > kRB)
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    const int col = c0 + tc.wave_c * kWaveCols + cb * 32 + (tc.lane & 31);
    if (DC) {
      if (sl.v0 + col < c.V) {
        bf16* row = out_dC + (int64_t)out_row[cb] * c.D + d_wave + 4 * (tc.lane >> 5);
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
          if (rb < rb_valid) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              f32x2 lo = {acc[rb][cb][g * 4 + 0], acc[rb][cb][g * 4 + 1]};
              f32x2 hi = {acc[rb][cb][g * 4 + 2], acc[rb][cb][g * 4 + 3]};
              uint2 packed;
              packed.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
              packed.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
              *(uint2*)(row + rb * 32 + 8 * g) = packed;
            }
          }
      }
    } else if (col < c.N) {
      if constexpr (ACC == kAccF32) {
        float* row = sl.dEacc + (int64_t)part * part_stride + (int64_t)col * c.D + d_wave + 4 * (tc.lane >> 5);
        if (!sl.first) {
          // every read of the column is issued before the first is waited for: 16 loads in
          // flight instead of one round trip to memory after the other
          float4 old[kRB][4];
#pragma unroll
          for (int rb = 0; rb < kRB; ++rb)
            if (rb < rb_valid) {
#pragma unroll
              for (int g = 0; g < 4; ++g) old[rb][g] = *(const float4*)(row + rb * 32 + 8 * g);
            }
#pragma unroll
          for (int rb = 0; rb < kRB; ++rb)
            if (rb < rb_valid) {
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                acc[rb][cb][g * 4 + 0] += old[rb][g].x;
                acc[rb][cb][g * 4 + 1] += old[rb][g].y;
                acc[rb][cb][g * 4 + 2] += old[rb][g].z;
                acc[rb][cb][g * 4 + 3] += old[rb][g].w;
              }
            }
        }
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
          if (rb < rb_valid) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *(float4*)(row + rb * 32 + 8 * g) = make_float4(acc[rb][cb][g * 4 + 0], acc[rb][cb][g * 4 + 1],
                                                              acc[rb][cb][g * 4 + 2], acc[rb][cb][g * 4 + 3]);
          }
      } else {
        // running sum kept in bf16 (+ bf16 compensation): element (part, token, d) of [ksplit, N, D], the
        // compensation terms in a second array of the same shape right after it
        bf16* sum_row = (bf16*)sl.dEacc + (int64_t)part * part_stride + (int64_t)col * c.D + d_wave + 4 * (tc.lane >> 5);
        bf16* comp_row = sum_row + (int64_t)ksplit * part_stride;
        uint2 old_sum[kRB][4], old_comp[kRB][4];
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            old_sum[rb][g] = make_uint2(0u, 0u);
            old_comp[rb][g] = make_uint2(0u, 0u);
            if (!sl.first && rb < rb_valid) {
              old_sum[rb][g] = *(const uint2*)(sum_row + rb * 32 + 8 * g);
              if (ACC == kAccBf16Kahan) old_comp[rb][g] = *(const uint2*)(comp_row + rb * 32 + 8 * g);
            }
          }
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
          if (rb < rb_valid) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const uint32_t sw[2] = {old_sum[rb][g].x, old_sum[rb][g].y}, cw[2] = {old_comp[rb][g].x, old_comp[rb][g].y};
              float t[4], cn[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                // bf16 -> fp32 is exact: the 16 bits become the upper half of the word
                const float sum = __uint_as_float((j & 1) ? (sw[j >> 1] & 0xffff0000u) : (sw[j >> 1] << 16));
                const float comp = __uint_as_float((j & 1) ? (cw[j >> 1] & 0xffff0000u) : (cw[j >> 1] << 16));
                const float y = acc[rb][cb][g * 4 + j] - comp;            // comp = 0 without compensation
                t[j] = (float)(bf16)(sum + y);                            // the new running sum, as it will be stored
                cn[j] = (t[j] - sum) - y;                                 // what the rounding added
              }
              f32x2 lo = {t[0], t[1]}, hi = {t[2], t[3]};
              uint2 packed;
              packed.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
              packed.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
              *(uint2*)(sum_row + rb * 32 + 8 * g) = packed;
              if (ACC == kAccBf16Kahan) {
                f32x2 clo = {cn[0], cn[1]}, chi = {cn[2], cn[3]};
                uint2 cp;
                cp.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(clo, bf16x2));
                cp.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(chi, bf16x2));
                *(uint2*)(comp_row + rb * 32 + 8 * g) = cp;
              }
            }
          }
      }
    }
  }
}

// counts the (256 token x 64 vocabulary) filter blocks of every slab and how many were kept;
// one workgroup per slab, whose flags start at flags + slab * region_words
__global__ __launch_bounds__(256) void count_flags_kernel(const uint32_t* flags, int64_t region_words, int n_tiles,
                                                          int vs, int V, FilterStats* stats, const int* n_dev) {
  const int slab = blockIdx.x;
  if (n_dev) n_tiles = (*n_dev + 255) / 256;   // token tiles actually present
  const int v0 = slab * vs;
  const int vs_this = min(vs, (V - v0 + 255) / 256 * 256);
  const int vsteps = vs_this / 64;
  const uint32_t* flags_nv = flags + (int64_t)slab * region_words;
  unsigned long long total = 0, kept = 0;
  for (int i = threadIdx.x; i < n_tiles * vsteps; i += blockDim.x) {
    int vstep = i % vsteps;
    if (v0 + vstep * 64 < V) {
      ++total;
      kept += flags_nv[i] != 0;
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    total += __shfl_xor(total, o);
    kept += __shfl_xor(kept, o);
  }
  if ((threadIdx.x & 63) == 0 && total) {
    atomicAdd(&stats->blocks_total, total);   // integer sums: order-independent
    atomicAdd(&stats->blocks_kept, kept);
  }
}

__global__ void zero_u32_kernel(uint32_t* p, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i < count; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0u;
}

}  // namespace

hipError_t launch_tile_lists(const TileListParams& p, hipStream_t stream) {
  hipLaunchKernelGGL(tile_flag_kernel, dim3(p.v_tiles, p.n_tiles), dim3(256), 0, stream, p);
  hipLaunchKernelGGL(tile_compact_kernel, dim3(p.slabs), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_bwd_recompute_mfma(const BwdCommon& c, const BwdMfmaSlab& s, int cus, hipStream_t stream) {
  const int n_tiles = s.Np / kTileC, v_tiles = s.vs / kTileR;
  const int want = cus > 0 ? cus : 256;
  const SplitPlan plan = make_split_plan(c.N, v_tiles, want, 1 << 30);
  if (s.tile_list) {
    // one share of the work list per CU, at most one per tile
    int groups = (want + kXcds - 1) / kXcds * kXcds;
    if (groups > n_tiles * v_tiles) groups = (n_tiles * v_tiles + kXcds - 1) / kXcds * kXcds;
    dim3 grid(groups);
    if (c.softcap > 0.f)
      hipLaunchKernelGGL((bwd_recompute_mfma_kernel<kCap, true>), grid, dim3(kThreads), 0, stream, c, s, plan, want);
    else
      hipLaunchKernelGGL((bwd_recompute_mfma_kernel<kNoCap, true>), grid, dim3(kThreads), 0, stream, c, s, plan, want);
  } else {
    dim3 grid(c.n_dev ? split_plan_max_grid(c.N, v_tiles, want, 1 << 30) : xcd_map_grid(plan.map));
    if (c.softcap > 0.f)
      hipLaunchKernelGGL((bwd_recompute_mfma_kernel<kCap, false>), grid, dim3(kThreads), 0, stream, c, s, plan, want);
    else
      hipLaunchKernelGGL((bwd_recompute_mfma_kernel<kNoCap, false>), grid, dim3(kThreads), 0, stream, c, s, plan, want);
  }
  return hipGetLastError();
}

hipError_t launch_zero_flags(uint32_t* flags, int64_t words, hipStream_t stream) {
  int64_t blocks = (words + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, flags, words);
  return hipGetLastError();
}

hipError_t launch_count_flags(const uint32_t* flags, int64_t region_words, int slabs, int n_tiles, int vs, int V,
                              FilterStats* stats, const int* n_dev, hipStream_t stream) {
  hipLaunchKernelGGL(count_flags_kernel, dim3(slabs), dim3(256), 0, stream, flags, region_words, n_tiles, vs, V, stats,
                     n_dev);
  return hipGetLastError();
}

hipError_t launch_bwd_dE_mfma(const BwdCommon& c, const BwdMfmaSlab& s, hipStream_t stream) {
  const int tiles_r = (c.D + kTileR - 1) / kTileR;
  const XcdMap map = make_xcd_map(tiles_r, (s.Np / kTileC) * s.ksplit);
  unsigned wgs = xcd_map_grid(map);
  if (c.n_dev) {
    // the device plans again for the tokens present: t tiles cut into k(t) <= (256 + t / 2) / t parts make
    // at most 256 + t / 2 workgroups while k >= 2 (t <= 170), and t workgroups otherwise
    const unsigned most = (unsigned)((256 + 85 + kXcds - 1) / kXcds * kXcds + kXcds);
    if (wgs < most) wgs = most;
  }
  dim3 grid(wgs);
  const bool filtered = c.filter_dE && c.eps > 0.f;
#define CCE_LAUNCH_DE(F, A) \
  hipLaunchKernelGGL((bwd_product_mfma_kernel<false, F, A>), grid, dim3(kThreads), 0, stream, c, s, (bf16*)nullptr, map)
  if (s.acc_mode == kAccBf16Kahan) { if (filtered) CCE_LAUNCH_DE(true, kAccBf16Kahan); else CCE_LAUNCH_DE(false, kAccBf16Kahan); }
  else if (s.acc_mode == kAccBf16) { if (filtered) CCE_LAUNCH_DE(true, kAccBf16); else CCE_LAUNCH_DE(false, kAccBf16); }
  else { if (filtered) CCE_LAUNCH_DE(true, kAccF32); else CCE_LAUNCH_DE(false, kAccF32); }
#undef CCE_LAUNCH_DE
  return hipGetLastError();
}

hipError_t launch_bwd_dC_mfma(const BwdCommon& c, const BwdMfmaSlab& s, void* out_dC, hipStream_t stream) {
  const int tiles_r = (c.D + kTileR - 1) / kTileR;
  const XcdMap map = make_xcd_map(tiles_r, s.vs / kTileC);
  dim3 grid(xcd_map_grid(map));
  if (c.filter_dC && c.eps > 0.f)
    hipLaunchKernelGGL((bwd_product_mfma_kernel<true, true>), grid, dim3(kThreads), 0, stream, c, s, (bf16*)out_dC, map);
  else
    hipLaunchKernelGGL((bwd_product_mfma_kernel<true, false>), grid, dim3(kThreads), 0, stream, c, s, (bf16*)out_dC, map);
  return hipGetLastError();
}

}  // namespace cce
