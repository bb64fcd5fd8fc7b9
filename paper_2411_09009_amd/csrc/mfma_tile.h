// 256 x 256 x 64 bf16 MFMA tile engine for gfx950 (CDNA4), shared by the forward
// linear-log-sum-exp kernel, the backward logit-recompute kernel and the two
// gradient products.
//
// Every product on this path is an "NT" contraction: both operands are row-major
// with the contracted index contiguous,
//     acc[r][c] = sum_k  P[r][k] * Q[c][k].
// A workgroup of 8 wavefronts (512 lanes, two wavefronts per SIMD) owns one
// 256 x 256 output tile.  Wave w computes rows (w / 4) * 128 .. +128 and columns
// (w % 4) * 64 .. +64 as 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 fp32
// accumulators per lane).  P plays the MFMA "A" role and Q the "B" role, so a
// lane holds ONE column c = lane % 32 of each 32 x 32 block and sixteen of its
// rows: reductions along r (the vocabulary axis in the forward pass) are
// lane-local.
//
// Operand K-slices (256 rows x 64 bf16 = 32 KB each) are brought in by
// global_load_lds_dwordx4 straight into LDS, two stages deep (128 KB of the
// CU's 160 KB).  A row of a K-slice is 128 B = 8 chunks of 16 B; chunk c of row
// r is stored at chunk position c ^ (r & 7), so the 16-byte ds_read_b128 of 8
// consecutive rows at one logical chunk touches all 8 chunk positions.  Because
// the LDS destination of a direct load is fixed (lane i of the instruction
// writes bytes [16 i, 16 i + 16) of a 1 KB span), the swizzle is applied on the
// global side: lane i fetches the chunk that belongs at its position.
//
// LDS reads are issued through inline assembly with explicit s_waitcnt: the
// compiler does not see them as LDS accesses, so it does not serialise them
// against the direct loads still in flight for the other stage.  All waits are
// lgkmcnt(0) / vmcnt(0) (no partial counts), which stays correct even if the
// compiler keeps a scalar load in flight.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cce {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kTileR = 256;        // rows of P per tile
constexpr int kTileC = 256;        // rows of Q per tile (columns of the output tile)
constexpr int kTileK = 64;         // contraction depth per stage
constexpr int kThreads = 512;
constexpr int kSliceBytes = 256 * kTileK * 2;   // one operand K-slice in LDS (32 KB)
constexpr int kStageBytes = 2 * kSliceBytes;    // P slice then Q slice
constexpr int kLdsBytes = 2 * kStageBytes;      // two stages
constexpr int kWaveRows = 128, kWaveCols = 64;
constexpr int kRB = 4, kCB = 2;    // 32x32 blocks per wave along rows / columns

#define CCE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define CCE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ inline uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)CCE_LDS_PTR(p); }

template <int IMM>
__device__ inline bf16x8 lds_read_b128(uint32_t addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM));
  return v;
}

// Wait for every outstanding LDS read; the operands tie the wait to the
// registers it guards so that no consumer can be scheduled above it.
__device__ inline void lds_wait(bf16x8 (&p)[kRB], bf16x8 (&q)[kCB]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(p[0]), "+v"(p[1]), "+v"(p[2]), "+v"(p[3]), "+v"(q[0]), "+v"(q[1]));
}

__device__ inline void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

struct TileCoords {
  int lane, wave, wave_r, wave_c;
  // LDS byte offsets (relative to a stage's start) of this lane's P row and Q
  // row at each of the four 16-deep MFMA steps of a stage, swizzle included
  uint32_t p_off[4], q_off[4];
  __device__ void init() {
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wave_r = wave >> 2;
    wave_c = wave & 3;
    uint32_t p_row = (uint32_t)(wave_r * kWaveRows + (lane & 31)) * 128u;
    uint32_t q_row = (uint32_t)(wave_c * kWaveCols + (lane & 31)) * 128u + kSliceBytes;
    uint32_t x = (uint32_t)((lane >> 5) ^ (lane & 7));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint32_t k = ((uint32_t)(ks * 2) ^ x) * 16u;
      p_off[ks] = p_row + k;
      q_off[ks] = q_row + k;
    }
  }
};

// Per-lane byte offsets (relative to the K-slice's first row, first column) of
// the four 16-byte chunks this lane brings in per operand per stage.  Rows at or
// beyond `rows_valid` are clamped to the last valid row: they are read (never
// out of bounds) and their results masked or discarded by the caller.
__device__ inline void dma_offsets(const TileCoords& tc, int rows_valid, int64_t ld_bytes,
                                   uint32_t (&off)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int r = (tc.wave * 4 + j) * 8 + (tc.lane >> 3);
    int chunk = (tc.lane & 7) ^ (r & 7);
    int rr = r < rows_valid ? r : rows_valid - 1;
    off[j] = (uint32_t)((int64_t)rr * ld_bytes + chunk * 16);
  }
}

// Issue the direct-to-LDS loads of one operand K-slice (this wave's share: 4 KB).
// gbase is wave-uniform; lds_slice is the LDS address of the slice.
__device__ inline void dma_slice(const TileCoords& tc, const char* gbase, const uint32_t (&off)[4],
                                 char* lds_slice) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    __builtin_amdgcn_global_load_lds(CCE_GLOBAL_PTR(gbase + off[j]),
                                     CCE_LDS_PTR(lds_slice + (tc.wave * 4 + j) * 1024), 16, 0, 0);
  }
}

// One 64-deep stage of MFMA work.  `stage_addr` is the LDS address of the stage.
// Fragments are double-buffered in registers: the reads of step ks+1 are in
// flight while the 8 MFMAs of step ks execute.
__device__ inline void mma_stage(const TileCoords& tc, uint32_t stage_addr, f32x16 (&acc)[kRB][kCB]) {
  bf16x8 p[2][kRB], q[2][kCB];
#define CCE_READ_FRAGS(buf, ks)                                              \
  {                                                                          \
    uint32_t pa = stage_addr + tc.p_off[ks], qa = stage_addr + tc.q_off[ks]; \
    p[buf][0] = lds_read_b128<0>(pa);                                        \
    p[buf][1] = lds_read_b128<4096>(pa);                                     \
    p[buf][2] = lds_read_b128<8192>(pa);                                     \
    p[buf][3] = lds_read_b128<12288>(pa);                                    \
    q[buf][0] = lds_read_b128<0>(qa);                                        \
    q[buf][1] = lds_read_b128<4096>(qa);                                     \
  }
  CCE_READ_FRAGS(0, 0)
  lds_wait(p[0], q[0]);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int cur = ks & 1, nxt = cur ^ 1;
    if (ks < 3) CCE_READ_FRAGS(nxt, ks + 1)
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb)
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[cur][rb], q[cur][cb], acc[rb][cb], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (ks < 3) lds_wait(p[nxt], q[nxt]);
  }
#undef CCE_READ_FRAGS
}

// Sweep P tiles t0 .. t1-1 (tile t = rows [256 t, 256 t + 256) of P, clamped to
// p_rows) against one fixed 256-row Q tile, with the K loop running seamlessly
// from one tile into the next: the first stage of tile t+1 is already in flight
// while the last stage of tile t is multiplied.  After the last stage of each
// tile, on_tile(t) consumes the accumulators and must leave them zeroed.
// One barrier per 64-deep stage: it publishes the stage that just landed and
// retires the stage the next loads overwrite.
template <class OnTile>
__device__ inline void sweep_tiles(const TileCoords& tc, char* lds, const char* P, int p_rows, int64_t ld_bytes,
                                   int t0, int t1, const char* gQ, const uint32_t (&offQ)[4], int KT,
                                   f32x16 (&acc)[kRB][kCB], OnTile on_tile) {
  if (t0 >= t1) return;
  const uint32_t lds_base = lds_addr(lds);
  uint32_t offP[4];
  const char* gP = P + (int64_t)t0 * kTileR * ld_bytes;
  dma_offsets(tc, min(kTileR, p_rows - t0 * kTileR), ld_bytes, offP);
  dma_slice(tc, gP, offP, lds);
  dma_slice(tc, gQ, offQ, lds + kSliceBytes);
  int stage = 0;
  for (int t = t0; t < t1; ++t) {
    for (int kt = 0; kt < KT; ++kt) {
      wait_dma();
      __builtin_amdgcn_s_barrier();
      bool more = true;
      int64_t k_next = (int64_t)(kt + 1) * (kTileK * 2);
      if (kt + 1 == KT) {
        k_next = 0;
        if (t + 1 < t1) {
          gP += (int64_t)kTileR * ld_bytes;
          dma_offsets(tc, min(kTileR, p_rows - (t + 1) * kTileR), ld_bytes, offP);
        } else {
          more = false;
        }
      }
      if (more) {
        char* nxt = lds + (stage ^ 1) * kStageBytes;
        dma_slice(tc, gP + k_next, offP, nxt);
        dma_slice(tc, gQ + k_next, offQ, nxt + kSliceBytes);
      }
      mma_stage(tc, lds_base + stage * kStageBytes, acc);
      stage ^= 1;
    }
    on_tile(t);
  }
}

// Row (0..31) inside a 32x32 block of accumulator element i of this lane.
__device__ inline int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

}  // namespace cce
