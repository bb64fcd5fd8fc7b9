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
// r is stored at chunk position c ^ ((r >> 1) & 7).  The LDS has 64 banks of 4 B
// and serves a ds_read_b128 sixteen lanes (256 B) per cycle; sixteen consecutive
// rows at one logical chunk then cover all sixteen 16-byte bank groups (row parity
// picks the 128-byte half, the swizzled chunk the position inside it), so the
// fragment reads are conflict free.  (Measured: the 32-bank swizzle c ^ (r & 7)
// costs one extra cycle per four on every read.)  Because
// the LDS destination of a direct load is fixed (lane i of the instruction
// writes bytes [16 i, 16 i + 16) of a 1 KB span), the swizzle is applied on the
// global side: lane i fetches the chunk that belongs at its position.
//
// An operand whose contracted index is NOT contiguous in memory ("K-major": rows are K
// steps, 256 output rows or columns contiguous, as E and GZ are when the contraction runs
// over tokens) is staged as 64 K-rows of 512 B and its fragments are fetched with
// ds_read_b64_tr_b16: sixteen lanes read a 4 (K) x 16 block as four 8-byte pieces per row
// and each receives four consecutive K values of one column, so two such reads make one
// MFMA operand.  Chunk c of K-row k sits at position c ^ (4 * (k & 3)), which spreads the
// four rows a 16-lane group touches over all banks.
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

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Eight consecutive K values of this lane's column from a K-major slice: two transposing
// reads, K rows IMM/512 .. +3 and +4 .. +7 relative to `addr`.
template <int IMM>
__device__ inline bf16x8 lds_read_tr(uint32_t addr) {
  u32x2 lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(IMM));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(IMM + 2048));
  u32x4 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
  return __builtin_bit_cast(bf16x8, v);
}

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
// Wait until at most N vector-memory operations of this wave are outstanding.  They retire in
// issue order, so everything issued before the last N (the direct loads of the coming stage)
// has landed while the N most recent ones (an epilogue's stores) may still be in flight.
template <int N>
__device__ inline void wait_dma_except() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

struct TileCoords {
  int lane, wave, wave_r, wave_c;
  // LDS byte offsets (relative to a stage's start) of this lane's P row and Q
  // row at each of the four 16-deep MFMA steps of a stage, swizzle included
  uint32_t p_off[4], q_off[4];
  // the same for K-major slices: byte offset of the lane's 8-byte piece in the first K-row
  // group of a stage, per 32-wide block of the wave (later K steps are immediate offsets)
  uint32_t pk_off[kRB], qk_off[kCB];
  __device__ void init() {
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wave_r = wave >> 2;
    wave_c = wave & 3;
    uint32_t p_row = (uint32_t)(wave_r * kWaveRows + (lane & 31)) * 128u;
    uint32_t q_row = (uint32_t)(wave_c * kWaveCols + (lane & 31)) * 128u + kSliceBytes;
    uint32_t x = (uint32_t)((lane >> 5) ^ ((lane >> 1) & 7));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint32_t k = ((uint32_t)(ks * 2) ^ x) * 16u;
      p_off[ks] = p_row + k;
      q_off[ks] = q_row + k;
    }
    // K-major: lane = (column c = lane & 31, K half kg = lane >> 5); as a source lane of its
    // 16-lane group it reads K-row (s >> 2) and columns 4 (s & 3) .. +3 of the group's 16
    const uint32_t s16 = (uint32_t)(lane & 15), half = (uint32_t)((lane >> 4) & 1), kg = (uint32_t)(lane >> 5);
    const uint32_t krow = 8u * kg + (s16 >> 2), swz = 4u * (s16 >> 2);
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
      uint32_t chunk = (uint32_t)(wave_r * kWaveRows + rb * 32) / 8u + 2u * half + ((s16 & 3u) >> 1);
      pk_off[rb] = krow * 512u + ((chunk ^ swz) << 4) + 8u * (s16 & 1u);
    }
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      uint32_t chunk = (uint32_t)(wave_c * kWaveCols + cb * 32) / 8u + 2u * half + ((s16 & 3u) >> 1);
      qk_off[cb] = krow * 512u + ((chunk ^ swz) << 4) + 8u * (s16 & 1u) + kSliceBytes;
    }
  }
};

// K-major operand: the lane's constants for the four 16-byte chunks it brings in per stage.
// DMA instruction ii = wave * 4 + j covers K-rows 2 ii and 2 ii + 1 (32 chunks each); lane
// i fills position i & 31 of row 2 ii + (i >> 5), i.e. logical chunk (i & 31) ^ (4 * (k & 3)).
struct KMajorLane {
  uint32_t krow0;        // K-row of j = 0 (row of j is krow0 + 2 j)
  uint32_t col[2];       // byte offset of the chunk inside the row for even / odd j
  __device__ void init(const TileCoords& tc, int chunks_valid) {
    krow0 = (uint32_t)(tc.wave * 8 + (tc.lane >> 5));
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      uint32_t k = krow0 + 2u * par;
      int c = (int)(((uint32_t)tc.lane & 31u) ^ (4u * (k & 3u)));
      if (c >= chunks_valid) c = chunks_valid - 1;     // columns past the operand's width: duplicates, discarded later
      col[par] = (uint32_t)c * 16u;
    }
  }
  // offsets (from the operand tile's origin: row 0, first column of the tile) for the stage
  // that starts at K-row k0; K-rows past k_last are clamped to it
  __device__ void offsets(int k0, int k_last, uint32_t ld_bytes, uint32_t (&off)[4]) const {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int k = k0 + (int)krow0 + 2 * j;
      k = k < k_last ? k : k_last;
      off[j] = (uint32_t)k * ld_bytes + col[j & 1];
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
    int chunk = (tc.lane & 7) ^ ((r >> 1) & 7);
    int rr = r < rows_valid ? r : rows_valid - 1;
    off[j] = (uint32_t)((int64_t)rr * ld_bytes + chunk * 16);
  }
}

// One direct-to-LDS load: this wave's j-th 1 KB span (8 rows) of a 32 KB operand
// slice.  gbase is wave-uniform; lds_slice is the slice's LDS address.
__device__ inline void dma_one(const TileCoords& tc, const char* gbase, uint32_t off, char* lds_slice, int j) {
  __builtin_amdgcn_global_load_lds(CCE_GLOBAL_PTR(gbase + off), CCE_LDS_PTR(lds_slice + (tc.wave * 4 + j) * 1024), 16,
                                   0, 0);
}

// Source of one 64-deep stage: wave-uniform base pointers of the P and Q K-slices
// plus the per-lane row/chunk offsets from dma_offsets().
struct StageSrc {
  const char* gP;
  const char* gQ;
  uint32_t offP[4], offQ[4];
};

__device__ inline void dma_stage(const TileCoords& tc, const StageSrc& src, char* lds_stage) {
#pragma unroll
  for (int j = 0; j < 4; ++j) dma_one(tc, src.gP, src.offP[j], lds_stage, j);
#pragma unroll
  for (int j = 0; j < 4; ++j) dma_one(tc, src.gQ, src.offQ[j], lds_stage + kSliceBytes, j);
}

// Issue the fragment reads of 16-deep step KS of the stage at LDS address `addr`.
template <bool PK, bool QK, int KS>
__device__ inline void read_frags(const TileCoords& tc, uint32_t addr, bf16x8 (&p)[kRB], bf16x8 (&q)[kCB]) {
  if constexpr (PK) {
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) p[rb] = lds_read_tr<KS * 16 * 512>(addr + tc.pk_off[rb]);
  } else {
    const uint32_t pa = addr + tc.p_off[KS];
    p[0] = lds_read_b128<0>(pa);
    p[1] = lds_read_b128<4096>(pa);
    p[2] = lds_read_b128<8192>(pa);
    p[3] = lds_read_b128<12288>(pa);
  }
  if constexpr (QK) {
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) q[cb] = lds_read_tr<KS * 16 * 512>(addr + tc.qk_off[cb]);
  } else {
    const uint32_t qa = addr + tc.q_off[KS];
    q[0] = lds_read_b128<0>(qa);
    q[1] = lds_read_b128<4096>(qa);
  }
}
#define CCE_READ_FRAGS(buf, addr, ks) read_frags<PK, QK, ks>(tc, addr, p[buf], q[buf]);

// Orders every MFMA that follows after the volatile asm statements that precede (the
// fragment reads just issued): without it the compiler sinks the reads below the MFMAs
// and folds the two fragment buffers into one set of registers, which leaves the LDS
// latency exposed.
__device__ inline void pin_acc(f32x16 (&acc)[kRB][kCB]) {
  asm volatile("" : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]), "+v"(acc[2][0]),
               "+v"(acc[2][1]), "+v"(acc[3][0]), "+v"(acc[3][1]));
}

#define CCE_MMA8(buf)                                                                                          \
  pin_acc(acc);                                                                                                \
  _Pragma("unroll") for (int rb = 0; rb < kRB; ++rb) _Pragma("unroll") for (int cb = 0; cb < kCB; ++cb)        \
      acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[buf][rb], q[buf][cb], acc[rb][cb], 0, 0, 0);

// Software-pipelined main loop over `nsteps` 64-deep stages, two LDS stages.
//
//   next(src)      fills the DMA source of the following stage; it is called once per
//                  stage, in stage order (a cursor that runs two stages ahead of the MFMAs).
//   step_done(i)   is called after the MFMAs of stage i have been issued; an epilogue that
//                  consumes the accumulators goes here (and must leave them zeroed).  It returns
//                  true when it has just issued at least KSTORE global stores as its last
//                  vector-memory operations: the next stage then does not wait for them.
//
// Per stage i the wave runs four 16-deep MFMA groups.  Fragments are double-buffered in
// registers: the reads for group g+1 are in flight while group g multiplies.  The single
// workgroup barrier of a stage sits between groups 2 and 3, after this wave's last LDS
// read of stage i: past it (a) every wave's loads of stage i+1 have landed, so the first
// fragments of stage i+1 are fetched under cover of group 3, and (b) stage i's buffer is
// dead, so the loads of stage i+2 are issued into it, interleaved with group 3's MFMAs so
// that their address-queue back-pressure never delays an MFMA.  Each load has one full
// stage to arrive.
// PK / QK: the P / Q operand is K-major (see the top of this file).
template <bool PK = false, bool QK = false, int KSTORE = 0, class Next, class StepDone>
__device__ inline void mma_pipeline(const TileCoords& tc, char* lds, int nsteps, f32x16 (&acc)[kRB][kCB], Next next,
                                    StepDone step_done) {
  if (nsteps <= 0) return;
  const uint32_t lds_base = lds_addr(lds);
  bf16x8 p[2][kRB], q[2][kCB];
  StageSrc src;
  next(src);
  dma_stage(tc, src, lds);
  wait_dma();
  __builtin_amdgcn_s_barrier();
  next(src);
  dma_stage(tc, src, lds + kStageBytes);
  CCE_READ_FRAGS(0, lds_base, 0)
  lds_wait(p[0], q[0]);
  int stage = 0;
  bool stores_pending = false;
  // The loop body is branch free (but for the choice of wait below): the last two iterations fetch a stage nobody multiplies
  // (next() keeps returning an in-bounds source) and prefetch fragments nobody uses.
  for (int i = 0; i < nsteps; ++i) {
    const uint32_t cur = lds_base + stage * kStageBytes;
    const uint32_t oth = lds_base + (stage ^ 1) * kStageBytes;
    CCE_READ_FRAGS(1, cur, 1)
    CCE_MMA8(0)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[1], q[1]);
    CCE_READ_FRAGS(0, cur, 2)
    CCE_MMA8(1)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[0], q[0]);
    CCE_READ_FRAGS(1, cur, 3)
    CCE_MMA8(0)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[1], q[1]);
    if (KSTORE > 0 && stores_pending) wait_dma_except<KSTORE>();
    else wait_dma();
    __builtin_amdgcn_s_barrier();
    CCE_READ_FRAGS(0, oth, 0)
    next(src);
    char* dst = lds + stage * kStageBytes;
    // group 3 with the eight loads of stage i+2 slotted between its MFMAs
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[1][rb], q[1][cb], acc[rb][cb], 0, 0, 0);
        const int m = rb * kCB + cb;
        if (m < 4) dma_one(tc, src.gP, src.offP[m], dst, m);
        else dma_one(tc, src.gQ, src.offQ[m - 4], dst + kSliceBytes, m - 4);
        __builtin_amdgcn_sched_barrier(0);
      }
    lds_wait(p[0], q[0]);
    stores_pending = step_done(i);
    stage ^= 1;
  }
  wait_dma();   // the surplus loads must have landed before the LDS is reused or released
}

// Variant with three P buffers and two Q buffers (all 160 KB of the LDS), for kernels that need
// no other LDS while the pipeline runs and whose operands are both K-contiguous.  The P loads
// of stage i+3 and the Q loads of stage i+2 are issued together (Q first) in the last quarter
// of stage i: P gets two stages to land, only the Q half of a stage is waited for one stage
// after its issue, and the four newest P loads stay in flight across the barrier, so the
// memory system is never drained.  Same contract as mma_pipeline.
constexpr int kLdsBytes3 = 5 * kSliceBytes;
template <int KSTORE = 0, class Next, class StepDone>
__device__ inline void mma_pipeline3(const TileCoords& tc, char* lds, int nsteps, f32x16 (&acc)[kRB][kCB], Next next,
                                     StepDone step_done) {
  if (nsteps <= 0) return;
  const uint32_t lds_base = lds_addr(lds);
  constexpr uint32_t q_area = 3u * kSliceBytes;      // the Q buffers follow the three P buffers
  bf16x8 p[2][kRB], q[2][kCB];
  auto issue_p = [&](const StageSrc& s, int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_one(tc, s.gP, s.offP[j], lds + buf * kSliceBytes, j);
  };
  auto issue_q = [&](const StageSrc& s, int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_one(tc, s.gQ, s.offQ[j], lds + q_area + buf * kSliceBytes, j);
  };
#define CCE_READ_FRAGS3(buf, pbi, qbi, ks)                                                       \
  {                                                                                              \
    const uint32_t pa = lds_base + (pbi) * kSliceBytes + tc.p_off[ks];                           \
    const uint32_t qa = lds_base + q_area + (qbi) * kSliceBytes + (tc.q_off[ks] - kSliceBytes);  \
    p[buf][0] = lds_read_b128<0>(pa);                                                            \
    p[buf][1] = lds_read_b128<4096>(pa);                                                         \
    p[buf][2] = lds_read_b128<8192>(pa);                                                         \
    p[buf][3] = lds_read_b128<12288>(pa);                                                        \
    q[buf][0] = lds_read_b128<0>(qa);                                                            \
    q[buf][1] = lds_read_b128<4096>(qa);                                                         \
  }
  // prologue: stage 0 complete, then P1, Q1, P2 in flight; Q2 follows in iteration 0
  StageSrc sq;
  next(sq);
  issue_p(sq, 0);
  issue_q(sq, 0);
  wait_dma();
  __builtin_amdgcn_s_barrier();
  next(sq);
  issue_p(sq, 1);
  issue_q(sq, 1);
  next(sq);            // stage 2: its Q half is still to be issued
  issue_p(sq, 2);
  CCE_READ_FRAGS3(0, 0u, 0u, 0)
  lds_wait(p[0], q[0]);
  uint32_t pb = 0, qb = 0;     // buffers of the current stage
  bool stores_pending = false;
  for (int i = 0; i < nsteps; ++i) {
    const uint32_t pn = pb == 2 ? 0 : pb + 1, qn = qb ^ 1;
    CCE_READ_FRAGS3(1, pb, qb, 1)
    CCE_MMA8(0)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[1], q[1]);
    CCE_READ_FRAGS3(0, pb, qb, 2)
    CCE_MMA8(1)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[0], q[0]);
    CCE_READ_FRAGS3(1, pb, qb, 3)
    CCE_MMA8(0)
    __builtin_amdgcn_sched_barrier(0);
    lds_wait(p[1], q[1]);
    // stage i+1 must have landed: its P (issued two stages ago) and its Q (one stage ago); the
    // four P loads issued after that Q, and an epilogue's stores after those, may stay in flight
    if (KSTORE > 0 && stores_pending) wait_dma_except<4 + KSTORE>();
    else wait_dma_except<4>();
    __builtin_amdgcn_s_barrier();
    CCE_READ_FRAGS3(0, pn, qn, 0)
    StageSrc sp;
    next(sp);            // stage i + 3
    char* dstQ = lds + q_area + qb * kSliceBytes;   // the buffers stage i has just left
    char* dstP = lds + pb * kSliceBytes;
    pin_acc(acc);
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p[1][rb], q[1][cb], acc[rb][cb], 0, 0, 0);
        const int m = rb * kCB + cb;
        if (m < 4) dma_one(tc, sq.gQ, sq.offQ[m], dstQ, m);        // Q of stage i + 2 first
        else dma_one(tc, sp.gP, sp.offP[m - 4], dstP, m - 4);      // then P of stage i + 3
        __builtin_amdgcn_sched_barrier(0);
      }
    lds_wait(p[0], q[0]);
    stores_pending = step_done(i);
    sq = sp;
    pb = pn;
    qb = qn;
  }
#undef CCE_READ_FRAGS3
  wait_dma();   // the surplus loads must have landed before the LDS is reused or released
}

// Sweep P tiles t0 .. t1-1 (tile t = rows [256 t, 256 t + 256) of P, clamped to p_rows)
// against one fixed 256-row Q tile, with the K loop running seamlessly from one tile into
// the next.  After the last stage of each tile, on_tile(t) consumes the accumulators and
// must leave them zeroed; its return value is that of mma_pipeline's step_done.  RING3 selects
// the five-slice ring (lds must then hold kLdsBytes3 bytes).  With `serpentine`, tiles with odd t
// take their 64-deep K stages in descending order: the Q slices such a tile starts with are the
// ones the tile before it has just used, still in the L2 (a third less traffic behind the L2 in
// the forward pass).  The sum over K of an element then depends on the parity of its tile.
template <int KSTORE = 0, bool RING3 = false, class OnTile>
__device__ inline void sweep_tiles(const TileCoords& tc, char* lds, const char* P, int p_rows, int64_t ld_bytes,
                                   int t0, int t1, const char* gQ, const uint32_t (&offQ)[4], int KT,
                                   f32x16 (&acc)[kRB][kCB], OnTile on_tile, bool serpentine = false) {
  if (t0 >= t1) return;
  // DMA cursor: (tile, k-step) of the next stage to fetch
  int cur_t = t0, cur_kt = 0;
  const char* gP = P + (int64_t)t0 * kTileR * ld_bytes;
  uint32_t offP[4];
  dma_offsets(tc, min(kTileR, p_rows - t0 * kTileR), ld_bytes, offP);
  int kt = 0, t = t0;   // compute cursor
  auto next = [&](StageSrc& src) {
    const int64_t koff = (int64_t)((serpentine && (cur_t & 1)) ? KT - 1 - cur_kt : cur_kt) * (kTileK * 2);
    src.gP = gP + koff;
    src.gQ = gQ + koff;
#pragma unroll
    for (int j = 0; j < 4; ++j) { src.offP[j] = offP[j]; src.offQ[j] = offQ[j]; }
    if (++cur_kt == KT) {
      if (cur_t + 1 < t1) {
        cur_kt = 0;
        ++cur_t;
        gP += (int64_t)kTileR * ld_bytes;
        dma_offsets(tc, min(kTileR, p_rows - cur_t * kTileR), ld_bytes, offP);
      } else {
        cur_kt = KT - 1;   // past the end: keep re-fetching the last slice (surplus loads)
      }
    }
  };
  auto step_done = [&](int) {
    if (++kt == KT) {
      kt = 0;
      const bool stored = on_tile(t);
      ++t;
      return stored;
    }
    return false;
  };
  if constexpr (RING3) mma_pipeline3<KSTORE>(tc, lds, (t1 - t0) * KT, acc, next, step_done);
  else mma_pipeline<false, false, KSTORE>(tc, lds, (t1 - t0) * KT, acc, next, step_done);
}

// Sweep entries e0 .. e1-1 of a list of independent 256 x 256 tiles, the K loop running
// seamlessly from one tile into the next.  src_of(e, gP, offP, gQ, offQ) fills the operand
// sources of entry e at K offset 0 (both operands K-contiguous); on_tile(e) consumes the
// accumulators after the entry's last stage and must leave them zeroed (return value as above).
template <int KSTORE = 0, class SrcOf, class OnTile>
__device__ inline void sweep_entries(const TileCoords& tc, char* lds, int e0, int e1, int KT, f32x16 (&acc)[kRB][kCB],
                                     SrcOf src_of, OnTile on_tile) {
  if (e0 >= e1) return;
  int cur_e = e0, cur_kt = 0;   // DMA cursor
  const char *gP, *gQ;
  uint32_t offP[4], offQ[4];
  src_of(cur_e, gP, offP, gQ, offQ);
  int kt = 0, e = e0;           // compute cursor
  mma_pipeline<false, false, KSTORE>(
      tc, lds, (e1 - e0) * KT, acc,
      [&](StageSrc& src) {
        const int64_t koff = (int64_t)cur_kt * (kTileK * 2);
        src.gP = gP + koff;
        src.gQ = gQ + koff;
#pragma unroll
        for (int j = 0; j < 4; ++j) { src.offP[j] = offP[j]; src.offQ[j] = offQ[j]; }
        if (++cur_kt == KT) {
          if (cur_e + 1 < e1) {
            cur_kt = 0;
            ++cur_e;
            src_of(cur_e, gP, offP, gQ, offQ);
          } else {
            cur_kt = KT - 1;   // past the end: keep re-fetching the last slice (surplus loads)
          }
        }
      },
      [&](int) {
        if (++kt == KT) {
          kt = 0;
          const bool stored = on_tile(e);
          ++e;
          return stored;
        }
        return false;
      });
}

// Row (0..31) inside a 32x32 block of accumulator element i of this lane.
__device__ inline int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

}  // namespace cce
