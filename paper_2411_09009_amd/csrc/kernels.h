// Internal launch interface between the C-ABI dispatcher and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cce {

typedef __bf16 bf16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Per-token forward partial: m2 = max_j(a_ij) * log2(e) over a vocabulary range,
// s = sum_j 2^(a_ij * log2(e) - m2) over the same range.  Both kernel families
// produce this pair and the finalize kernel merges them.
typedef float2 LsePartial;

// Placement of a dim_a x dim_b grid of work items on the chip's XCDs (each has its own
// L2).  The hardware deals workgroups to the XCDs round-robin, so workgroup wg runs on
// XCD wg % 8.  The map hands every XCD a run of `wgs_per_xcd` consecutive logical items,
// ordered as rectangles of group_a x group_b items (a fastest inside a rectangle,
// rectangles a-major), so that the workgroups resident on one XCD at a time share as
// many operand slices as possible.  group_a divides dim_a, group_b divides dim_b and
// group_a * group_b divides wgs_per_xcd.
constexpr int kXcds = 8;
struct XcdMap {
  int dim_a, dim_b, wgs_per_xcd, group_a, group_b;
};
__host__ __device__ inline XcdMap make_xcd_map(int dim_a, int dim_b) {
  XcdMap m{dim_a, dim_b, 1, 1, 1};
  const int total = dim_a * dim_b;
  m.wgs_per_xcd = (total + kXcds - 1) / kXcds;
  for (int g = 8; g >= 1; --g)
    if (dim_a % g == 0 && m.wgs_per_xcd % g == 0) { m.group_a = g; break; }
  for (int g = 32 / m.group_a; g >= 1; --g)
    if (dim_b % g == 0 && m.wgs_per_xcd % (m.group_a * g) == 0) { m.group_b = g; break; }
  return m;
}
inline unsigned xcd_map_grid(const XcdMap& m) { return (unsigned)(kXcds * m.wgs_per_xcd); }
// false: this workgroup is padding (the grid is rounded up to a multiple of 8)
__device__ inline bool xcd_map_decode(const XcdMap& m, int wg, int& a, int& b) {
  if (wg / kXcds >= m.wgs_per_xcd) return false;   // the launch may be larger than this map needs
  const int logical = (wg % kXcds) * m.wgs_per_xcd + wg / kXcds;
  if (logical >= m.dim_a * m.dim_b) return false;
  const int per_group = m.group_a * m.group_b;
  const int g = logical / per_group, w = logical % per_group;
  const int groups_a = m.dim_a / m.group_a;
  a = (g % groups_a) * m.group_a + w % m.group_a;
  b = (g / groups_a) * m.group_b + w / m.group_a;
  return a < m.dim_a && b < m.dim_b;
}

// How the (token tile, vocabulary tile) grid of the forward / recompute kernels is cut into
// workgroups: every token tile is paired with `splits` contiguous ranges of `tiles_per_split`
// vocabulary tiles, enough of them that one round of token tiles (at most `round_cap` at a
// time, so that their E tiles stay cache resident) gives every CU a workgroup.  Computed on
// the host for N tokens and, when ignored tokens were removed, again on the device for the
// number actually present (the host launches max_grid workgroups, which covers either).
struct SplitPlan {
  int n_tiles, splits, tiles_per_split;
  XcdMap map;
};
__host__ __device__ inline SplitPlan make_split_plan(int n_tokens, int v_tiles, int want_wgs, int round_cap) {
  SplitPlan p{};
  p.n_tiles = (n_tokens + 255) / 256;
  if (p.n_tiles < 1) p.n_tiles = 1;
  const int round_tiles = p.n_tiles < round_cap ? p.n_tiles : round_cap;
  int splits = want_wgs / round_tiles;   // rounded down: a round must not exceed the CUs by a few workgroups
  if (splits > v_tiles) splits = v_tiles;
  if (splits < 1) splits = 1;
  p.tiles_per_split = (v_tiles + splits - 1) / splits;
  p.splits = (v_tiles + p.tiles_per_split - 1) / p.tiles_per_split;
  p.map = make_xcd_map(p.n_tiles, p.splits);
  return p;
}
// workgroups to launch so that the plan of any token count up to n_tokens fits
inline unsigned split_plan_max_grid(int n_tokens, int v_tiles, int want_wgs, int round_cap) {
  const int n_tiles = (n_tokens + 255) / 256;
  int64_t most = (int64_t)want_wgs + (n_tiles < round_cap ? n_tiles : round_cap);     // up to round_cap token tiles
  const int64_t big = (int64_t)n_tiles * ((want_wgs + round_cap - 1) / round_cap);     // more than that
  if (n_tiles > round_cap && big > most) most = big;
  if (most > (int64_t)n_tiles * v_tiles) most = (int64_t)n_tiles * v_tiles;
  return (unsigned)((most + kXcds - 1) / kXcds * kXcds + kXcds);
}
// rows of the per-split partial buffer that plan can address (stride = tokens rounded up to 256)
inline size_t split_plan_max_partial_rows(int n_tokens, int v_tiles, int want_wgs, int round_cap) {
  return (size_t)split_plan_max_grid(n_tokens, v_tiles, want_wgs, round_cap) * 256;
}

// Small batches leave the dE product with fewer (token tile, D tile) pairs than CUs; it then cuts each
// slab's contraction into this many parts with a running sum each (added up when dE is stored).
// Host and device: with ignored tokens removed the kernels plan again for the tokens present.
__host__ __device__ inline int dE_ksplit_for(int64_t n_tokens, int64_t D) {
  const int64_t tiles = ((n_tokens + 255) / 256) * ((D + 255) / 256);
  if (tiles <= 0) return 1;
  int64_t k = (256 + tiles / 2) / tiles;
  if (k < 1) k = 1;
  if (k > 8) k = 8;
  return (int)k;
}
// Parts and part stride (elements) of the dE running sums when `n_tokens` of the `N` tokens the workspace
// was sized for are present: the parts planned for n_tokens, as many of them as fit the space of the
// ksplit_N parts of N rows, each part n_tokens rounded up to 256 rows.
struct DEParts {
  int parts;
  int64_t stride;
};
__host__ __device__ inline DEParts dE_parts_present(int64_t n_tokens, int64_t N, int64_t D, int ksplit_N) {
  DEParts p;
  const int64_t rows = (n_tokens + 255) / 256 * 256;
  int64_t k = dE_ksplit_for(n_tokens, D);
  const int64_t fit = rows > 0 ? ((int64_t)ksplit_N * N) / rows : 1;
  if (k > fit) k = fit;
  if (k < 1) k = 1;
  p.parts = (int)k;
  p.stride = rows * D;
  if (k == 1 && rows > N) p.stride = N * D;   // a single part never needs the padding rows
  return p;
}

// ---- forward, MFMA path ------------------------------------------------------
struct FwdMfmaParams {
  const bf16* E;        // [N, D]
  const bf16* C;        // [V, D]
  int N, D, V;
  float softcap;        // 0 = none
  LsePartial* partial;  // [splits, partial_stride]
  int v_tiles;          // ceil(V / 256)
  SplitPlan plan;       // for N tokens (a = token tile, b = vocabulary split)
  int want_wgs, round_cap;   // the plan's inputs, for the device-side plan
  unsigned grid;        // workgroups to launch
  const int* n_dev;        // optional device count of tokens actually present in E (ignored tokens removed):
                           // the kernel then plans for that many tokens and the partial stride is that
                           // count rounded up to 256
  unsigned long long* bad_targets;   // optional counter the finalize kernel adds to: workgroup 0 clears it here
  uint16_t* block_max;     // optional [ceil(V / 128), block_max_stride] bf16 bits: for every token the largest
                           // (soft-capped) logit within each 128-wide vocabulary block, rounded up; nullptr = off
  int block_max_stride;    // N rounded up to 256
};
hipError_t launch_fwd_lse_mfma(const FwdMfmaParams& p, hipStream_t stream);

// ---- forward, plain kernels (float or bf16 storage, fp32 FMA) -----------------
struct FwdPlainParams {
  const void* E;
  const void* C;
  int dtype;            // CCE_BF16 / CCE_F32
  int N, D, V;
  float softcap;
  LsePartial* partial;  // [splits, N]
  int splits, tiles_per_split;   // 64-wide vocabulary tiles
  unsigned long long* bad_targets;   // optional counter the finalize kernel adds to: workgroup (0, 0) clears it here
};
hipError_t launch_fwd_lse_plain(const FwdPlainParams& p, hipStream_t stream);

// ---- finalize: merge partials, indexed dot product, loss (Alg. 1 + Eq. 4) -----
struct FinalizeParams {
  const void* E;
  const void* C;
  int dtype;
  const int64_t* targets;
  int N, D, V;
  float softcap;
  int64_t ignore_index;
  const LsePartial* partial;   // [splits, N], or as planned on the device when n_dev is set
  int splits;
  int v_tiles, want_wgs, round_cap;   // MFMA path with n_dev: inputs of the device-side plan
  float* out_loss;
  float* out_lse;
  // ignored tokens removed: E and partial hold *n_dev tokens, token k being the caller's token idx[k]
  // (targets and the outputs keep the caller's indexing); nullptr = all N tokens in place
  const int* n_dev;
  const int* idx;
  // optional: number of targets that are neither ignore_index nor inside [0, V) (they are treated as
  // ignored); cleared by the forward kernel that precedes this one.  nullptr when ignored tokens were
  // removed: the compaction kernel has then counted them already.
  unsigned long long* bad_targets;
};
hipError_t launch_finalize(const FinalizeParams& p, hipStream_t stream);

// Counters kept at the start of the forward workspace.
struct ForwardStats {
  unsigned long long bad_targets;   // targets that are neither ignore_index nor inside [0, V)
};

// ---- backward -----------------------------------------------------------------
// Filter counters kept at the start of the backward workspace.
struct FilterStats {
  unsigned long long blocks_total;
  unsigned long long blocks_kept;
};

// One vocabulary slab [v0, v0 + vs) of the backward pass; vs is the slab's padded
// width (a multiple of the path's tile width), columns >= V hold zeros.
struct BwdCommon {
  const void* E;
  const void* C;
  int dtype;
  const int64_t* targets;
  const float* lse;
  const float* dloss;
  int N, D, V;
  float softcap;
  int64_t ignore_index;
  float eps;            // 0 = no filtering
  int filter_dE, filter_dC;
  FilterStats* stats;
  // ignored tokens removed (Appendix B): E holds *n_dev tokens, token k being the caller's token
  // idx[k]; targets, lse and dloss keep the caller's indexing.  nullptr = all N tokens in place.
  const int* n_dev;
  const int* idx;
};

// MFMA path buffers (bf16).  Np = N rounded up to 256.
struct BwdMfmaSlab {
  int v0, vs, Np;
  bf16* GZ;             // [Np, vs]  dloss * G * a'   (token-major; zero for tokens >= N and columns >= V)
  float* dEacc;         // [ksplit, N, D] fp32; with acc_mode != 0: bf16 [ksplit, N, D] running sums followed by
                        // bf16 [ksplit, N, D] compensation terms (the same bytes)
  int acc_mode;         // 0: fp32 accumulator; 1: bf16 running sum; 2: bf16 running sum + Kahan compensation
  int ksplit;           // parts the dE product cuts a slab's K steps into (>= 1), one accumulator each
  int64_t dE_part_stride;   // N * D
                        // (with BwdCommon::n_dev both are planned again on the device: dE_parts_present)
  uint32_t* flags_nv;   // [Np/256, vs/64]  block (256 tokens x 64 vocab) has a significant entry
  uint32_t* flags_vn;   // [vs/256, Np/64]  block (64 tokens x 256 vocab) has a significant entry
  int first;            // first slab of the call: dEacc is overwritten instead of added to
  const bf16* Crows;    // row v0 of the classifier as this slab sees it: C + v0 * D, or the slab's
                        // gathered copy when the vocabulary is walked in sorted order
  const int* perm;      // sorted position -> original vocabulary index (rows of dC are written
                        // through it); nullptr = identity
  // optional work list of the recompute kernel (nullptr = every tile of the slab):
  // tile_list[i] = token tile << 16 | slab-local vocabulary tile, token-tile major; *tile_count entries
  const uint32_t* tile_list;
  const uint32_t* tile_count;
};

// ---- tiles the gradient filter cannot skip (from the forward's block-maximum record) ----
struct TileListParams {
  const uint16_t* block_max;   // [ceil(V / 128), stride] bf16 bits, see FwdMfmaParams
  int stride;
  const int64_t* targets;
  const float* lse;
  int N, V;
  int64_t ignore_index;
  float log_eps;               // log(filter_eps) minus a rounding margin
  int n_tiles, v_tiles;        // ceil(N / 256), ceil(V / 256)
  int slab_tiles;              // vocabulary tiles per slab
  int slabs;
  const int* n_dev;            // ignored tokens removed: see BwdCommon
  const int* idx;
  uint8_t* tile_flag;          // [n_tiles, v_tiles] scratch
  uint32_t* tile_list;         // [slabs, n_tiles * slab_tiles] out
  uint32_t* tile_count;        // [slabs] out
};
hipError_t launch_tile_lists(const TileListParams& p, hipStream_t stream);
// cus: compute units of the device (one workgroup, or one share of the work list, per CU)
hipError_t launch_bwd_recompute_mfma(const BwdCommon& c, const BwdMfmaSlab& s, int cus, hipStream_t stream);
// Filter flags of the MFMA path: every slab has its own region of `region_words` words
// ([Np/256, vs/64] then [vs/256, Np/64]); all are cleared once before the first slab and
// counted once after the last.
hipError_t launch_zero_flags(uint32_t* flags, int64_t words, hipStream_t stream);
hipError_t launch_count_flags(const uint32_t* flags, int64_t region_words, int slabs, int n_tiles, int vs, int V,
                              FilterStats* stats, const int* n_dev, hipStream_t stream);
hipError_t launch_bwd_dE_mfma(const BwdCommon& c, const BwdMfmaSlab& s, hipStream_t stream);
hipError_t launch_bwd_dC_mfma(const BwdCommon& c, const BwdMfmaSlab& s, void* out_dC, hipStream_t stream);

// Plain path buffers (GZ kept in fp32, token-major only).
struct BwdPlainSlab {
  int v0, vs;           // vs multiple of 64
  float* GZ;            // [N, vs]
  float* dEacc;         // [N, D]
  uint8_t* flags;       // [ceil(N/64), vs/64]
  int first;
};
hipError_t launch_bwd_gz_plain(const BwdCommon& c, const BwdPlainSlab& s, hipStream_t stream);
hipError_t launch_bwd_dE_plain(const BwdCommon& c, const BwdPlainSlab& s, hipStream_t stream);
hipError_t launch_bwd_dC_plain(const BwdCommon& c, const BwdPlainSlab& s, void* out_dC, hipStream_t stream);

// ---- vocabulary sorting (Section 4.3) ------------------------------------------
struct VocabSortParams {
  const bf16* E;            // [N, D]
  const bf16* C;            // [V, D]
  const int64_t* targets;   // [N]
  int N, D, V;
  int64_t ignore_index;
  float* partial;           // [vocab_sort_partial_bytes(D)] column sums of row blocks of E
  float* mean;              // [D] mean token embedding
  float* key;               // [V] mean logit of every vocabulary entry
  float* key_sorted;        // [V]
  int* index;               // [V] 0 .. V-1
  int* perm;                // [V] out: original index at each sorted position (descending key)
  int* inverse;             // [V] out: sorted position of each original index
  int64_t* targets_sorted;  // [N] out: targets as sorted positions (ignored / out-of-range -> ignore_index)
  void* temp;               // radix-sort scratch
  size_t temp_bytes;
};
size_t vocab_sort_temp_bytes(int64_t V);
// what the radix sort really asks for (a size query: nothing is launched)
hipError_t vocab_sort_temp_needed(int64_t V, size_t* bytes);
size_t vocab_sort_partial_bytes(int64_t D);
hipError_t launch_vocab_sort(const VocabSortParams& p, hipStream_t stream);
// out[r][:] = C[perm[p0 + r]][:], r < rows (D a multiple of 8)
hipError_t launch_gather_rows(const bf16* C, const int* perm, int p0, int rows, int D, bf16* out, hipStream_t stream);

// Sum of the `parts` accumulators dEacc (fp32 [parts, N, D]) -> out_dE in the storage dtype.  With idx /
// n_dev (ignored tokens removed) row k goes to row idx[k] of out_dE for k < *n_dev and every other row is zeroed.
// acc_bf16: the accumulators hold bf16 running sums (BwdMfmaSlab::acc_mode != 0) instead of fp32.
hipError_t launch_store_dE(const float* dEacc, int parts, void* out_dE, int dtype, int64_t N, int64_t D,
                           const int* idx, const int* n_dev, bool acc_bf16, hipStream_t stream);
// (with idx / n_dev, `parts` is the count planned for N tokens; the kernel uses dE_parts_present)

// ---- removing ignored tokens (Appendix B) ---------------------------------------
// idx[k] = index of the k-th token whose target is valid (in order), *count = their number;
// *bad_targets (optional) = number of targets that are neither ignore_index nor inside [0, V)
hipError_t launch_compact_tokens(const int64_t* targets, int N, int V, int64_t ignore_index, int* idx, int* count,
                                 unsigned long long* bad_targets, hipStream_t stream);
// out[k][:] = E[idx[k]][:] for k < *count (bf16, D a multiple of 8)
hipError_t launch_gather_tokens(const bf16* E, const int* idx, const int* count, int N, int D, bf16* out,
                                hipStream_t stream);
hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t stream);
hipError_t launch_clear_stats(FilterStats* stats, hipStream_t stream);

}  // namespace cce
