// C ABI of the library (see include/cce.h): argument checks, path selection,
// workspace carve-up and kernel sequencing.  No arithmetic of the method lives
// here; every step of the path runs in the HIP kernels this file launches.
#include "cce.h"
#include "kernels.h"

#include <hip/hip_runtime.h>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>

namespace {

using namespace cce;

thread_local char g_hip_error[256] = "no HIP error recorded";
thread_local char g_noalloc_error[256] = "problem too large for the static scratch of cce_forward_noalloc";

int hip_fail(hipError_t e, const char* what) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
  return CCE_EHIP;
}
#define CCE_HIP(call)                                 \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return hip_fail(e_, #call); \
  } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int kMaxDevices = 64;
constexpr int64_t kMfmaSlabCols = 6144;  // recommended backward slab width (vocabulary entries), MFMA path
constexpr int64_t kPlainSlabCols = 4096;
constexpr int kMaxFilteredKSteps = 2048;
constexpr int kSlabBuffers = 2;          // vocabulary slabs in flight in the MFMA backward pass
constexpr int64_t kWideSlabFactor = 4;   // CCE_OP_BACKWARD_WIDE: slab width over the recommended one

int cu_count() {
  static std::atomic<int> cached[kMaxDevices];   // zero-initialised; 0 = not asked yet
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);   // every thread computes the same value
  }
  return n;
}

// Workspace lent to the plain entry points (cce_set_workspace): one registration per device.
// The library never allocates, frees or synchronises; without a registration the plain calls
// return CCE_EWORKSPACE.
struct LentWorkspace {
  void* ptr = nullptr;
  size_t bytes = 0;
};
LentWorkspace g_lent[kMaxDevices];
std::mutex g_lent_mutex;

int lent_workspace(LentWorkspace* out) {
  int dev = 0;
  CCE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CCE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_lent_mutex);
  *out = g_lent[dev];
  return out->ptr ? CCE_OK : CCE_EWORKSPACE;
}

// Helper streams of the MFMA backward pass: the two gradient products of a vocabulary
// slab run beside each other and beside the recompute of the next slab, so that the
// partly filled last round of one kernel's workgroups is topped up by the others.
// One set per device, created on first use; a call holds the device's mutex while it
// enqueues, so the events are never recorded by two calls at once (a wait refers to
// the record that precedes it in program order).
constexpr int kEventRing = 4;
struct Helpers {
  std::mutex mutex;
  bool ready = false;
  hipStream_t product[3] = {};        // [0], [2] dC products of even / odd slabs, [1] dE products
  hipEvent_t started = nullptr;
  hipEvent_t recomputed[kEventRing] = {};
  hipEvent_t dC_done[kEventRing] = {};
  hipEvent_t dE_done[kEventRing] = {};
  hipEvent_t joined[3] = {};          // one per product stream: everything enqueued on it so far
};
Helpers g_helpers[kMaxDevices];

int helpers_for_device(Helpers** out) {
  int dev = 0;
  CCE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CCE_EUNSUPPORTED;
  Helpers& h = g_helpers[dev];
  std::lock_guard<std::mutex> lock(h.mutex);
  if (!h.ready) {
    for (auto& st : h.product) CCE_HIP(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    CCE_HIP(hipEventCreateWithFlags(&h.started, hipEventDisableTiming));
    for (int i = 0; i < kEventRing; ++i) {
      CCE_HIP(hipEventCreateWithFlags(&h.recomputed[i], hipEventDisableTiming));
      CCE_HIP(hipEventCreateWithFlags(&h.dC_done[i], hipEventDisableTiming));
      CCE_HIP(hipEventCreateWithFlags(&h.dE_done[i], hipEventDisableTiming));
    }
    for (auto& ev : h.joined) CCE_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    h.ready = true;
  }
  *out = &h;
  return CCE_OK;
}

// Scratch of cce_forward_noalloc: device memory that exists as long as the library is loaded, so
// that the call needs no allocation at all.  The name below is a host-side stand-in, not a
// device address: host code uses the address hipGetSymbolAddress returns for the current device
// (every GPU holds its own copy), looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void* g_scratch_ptr[kMaxDevices];   // per device, nullptr = not looked up yet
std::mutex g_scratch_mutex;

int static_scratch(void** out) {
  int dev = 0;
  CCE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CCE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    CCE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));   // address on the current device
    if (!ptr) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CCE_OK;
}

bool use_mfma(int64_t D, const cce_opts* o) {
  return o->dtype == CCE_BF16 && !(o->flags & CCE_PLAIN_KERNELS) && D % 64 == 0;
}

size_t block_max_bytes(int64_t N, int64_t V) {
  return (size_t)((V + 127) / 128) * (size_t)round_up(N, 256) * sizeof(uint16_t);
}

int check_common(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                 float softcap, const cce_opts* o) {
  if (!o) return CCE_EINVAL;
  if (o->dtype != CCE_BF16 && o->dtype != CCE_F32) return CCE_EUNSUPPORTED;
  if (o->flags & ~(uint32_t)(CCE_FILTER_DE | CCE_FILTER_DC | CCE_VOCAB_SORT | CCE_PLAIN_KERNELS | CCE_SKIP_TILES |
                            CCE_COMPACT_IGNORED | CCE_SINGLE_STREAM | CCE_ACCUM_BF16 | CCE_ACCUM_KAHAN)) return CCE_EUNSUPPORTED;
  if (!E || !C || !targets) return CCE_EINVAL;
  if (N <= 0 || D <= 0 || V <= 0) return CCE_EINVAL;
  if (N > (int64_t)0x7fff0000 || V > (int64_t)0x7fff0000 || D > (1 << 22)) return CCE_EINVAL;
  if (!(softcap >= 0.f) || std::isinf(softcap)) return CCE_EINVAL;   // rejects NaN and negatives
  if (!(o->filter_eps >= 0.f) || !(o->filter_eps < 1.f)) return CCE_EINVAL;
  if (!aligned(E, 16) || !aligned(C, 16) || !aligned(targets, 8)) return CCE_EINVAL;
  if (o->workspace && !aligned(o->workspace, 256)) return CCE_EINVAL;
  if ((o->flags & CCE_SKIP_TILES) && o->block_max) {
    if (!aligned(o->block_max, 256)) return CCE_EINVAL;
    // the record is addressed with 32-bit element offsets
    if ((uint64_t)((V + 127) / 128) * (uint64_t)round_up(N, 256) >= ((uint64_t)1 << 31)) return CCE_EUNSUPPORTED;
    if (o->block_max_bytes < block_max_bytes(N, V)) return CCE_EWORKSPACE;
  }
  return CCE_OK;
}

// ------------------------------------------------------------------ forward plan
struct FwdPlan {
  bool mfma;
  int splits, tiles_per_split;   // plain path
  int n_tiles, v_tiles;
  SplitPlan plan;                // MFMA path, for N tokens
  int want_wgs, round_cap;
  unsigned grid;
  size_t off_partial, partial_bytes;
  // ignored tokens removed (CCE_COMPACT_IGNORED, MFMA path): index list, count, compacted copy of E
  bool compact;
  size_t off_idx, off_count, off_Ec;
  size_t total_bytes;
};

FwdPlan plan_forward(int64_t N, int64_t D, int64_t V, const cce_opts* o) {
  FwdPlan p{};
  p.mfma = use_mfma(D, o);
  const int tile = p.mfma ? 256 : 64;
  const int cus = cu_count();
  p.n_tiles = (int)((N + tile - 1) / tile);
  p.v_tiles = (int)((V + tile - 1) / tile);
  p.compact = p.mfma && (o->flags & CCE_COMPACT_IGNORED);
  if (p.mfma) {
    // enough vocabulary splits that one round of token tiles (at most 32 at a time, so that
    // the E tiles in flight stay cache resident) fills every CU
    p.want_wgs = cus;
    p.round_cap = 32;
    p.plan = make_split_plan((int)N, p.v_tiles, p.want_wgs, p.round_cap);
    p.splits = p.plan.splits;
    p.tiles_per_split = p.plan.tiles_per_split;
    p.grid = p.compact ? split_plan_max_grid((int)N, p.v_tiles, p.want_wgs, p.round_cap) : xcd_map_grid(p.plan.map);
  } else {
    int splits = (4 * cus + p.n_tiles - 1) / p.n_tiles;
    if (splits > p.v_tiles) splits = p.v_tiles;
    if (splits < 1) splits = 1;
    p.tiles_per_split = (p.v_tiles + splits - 1) / splits;
    p.splits = (p.v_tiles + p.tiles_per_split - 1) / p.tiles_per_split;
  }
  p.off_partial = 256;   // the workspace starts with the forward's counters (ForwardStats)
  size_t rows = (size_t)p.splits * (size_t)N;
  if (p.compact) {
    // the device-side plan for fewer tokens uses more splits of fewer rows
    const size_t most = split_plan_max_partial_rows((int)N, p.v_tiles, p.want_wgs, p.round_cap);
    if (most > rows) rows = most;
  }
  p.partial_bytes = align_up(rows * sizeof(LsePartial), 256);
  p.total_bytes = p.off_partial + p.partial_bytes;
  if (p.compact) {
    p.off_idx = p.total_bytes;   p.total_bytes += align_up((size_t)N * 4, 256);
    p.off_count = p.total_bytes; p.total_bytes += 256;
    p.off_Ec = p.total_bytes;    p.total_bytes += align_up((size_t)round_up(N, 256) * D * 2, 256);
  }
  return p;
}

// ------------------------------------------------------------------ backward plan
int dE_ksplit(int64_t N, int64_t D) { return dE_ksplit_for(N, D); }


struct BwdPlan {
  bool mfma;
  int64_t Np, vs;          // padded token count, slab width
  size_t off_flags[kSlabBuffers], off_dEacc, off_GZ[kSlabBuffers];   // GZ: one per slab in flight (MFMA path);
                                                                       // flags: [0] only, one region per slab on the MFMA path
  size_t flag_region_words;
  // vocabulary sorting (MFMA path only)
  size_t off_partial, off_mean, off_key, off_key_sorted, off_index, off_perm, off_inverse, off_targets, off_Cs[kSlabBuffers],
      off_sort_temp;
  size_t sort_temp_bytes;
  // work lists of the recompute kernel (CCE_SKIP_TILES)
  size_t off_tile_flag, off_tile_list, off_tile_count;
  // ignored tokens removed (CCE_COMPACT_IGNORED)
  size_t off_idx, off_count, off_Ec;
  size_t total_bytes;
};

BwdPlan layout_backward(bool mfma, int64_t N, int64_t D, int64_t V, int64_t vs, bool sort, bool lists,
                        bool compact) {
  BwdPlan p{};
  p.mfma = mfma;
  p.vs = vs;
  size_t off = 256;   // FilterStats
  if (mfma) {
    p.Np = round_up(N, 256);
    p.off_dEacc = off;
    off += align_up((size_t)dE_ksplit(N, D) * (size_t)N * D * 4, 256);
    {
      const size_t slabs = (size_t)((round_up(V, 256) + vs - 1) / vs);
      p.flag_region_words = (size_t)(p.Np / 256) * (vs / 64) + (size_t)(vs / 256) * (p.Np / 64);
      p.off_flags[0] = off;
      off += align_up(slabs * p.flag_region_words * 4, 256);
    }
    for (int b = 0; b < kSlabBuffers; ++b) {
      p.off_GZ[b] = off;
      off += align_up((size_t)p.Np * vs * 2, 256);
    }
    if (sort) {
      p.off_partial = off;  off += align_up(vocab_sort_partial_bytes(D), 256);
      p.off_mean = off;     off += align_up((size_t)D * 4, 256);
      p.off_key = off;      off += align_up((size_t)V * 4, 256);
      p.off_key_sorted = off; off += align_up((size_t)V * 4, 256);
      p.off_index = off;    off += align_up((size_t)V * 4, 256);
      p.off_perm = off;     off += align_up((size_t)V * 4, 256);
      p.off_inverse = off;  off += align_up((size_t)V * 4, 256);
      p.off_targets = off;  off += align_up((size_t)N * 8, 256);
      for (int b = 0; b < kSlabBuffers; ++b) { p.off_Cs[b] = off; off += align_up((size_t)vs * D * 2, 256); }
      p.sort_temp_bytes = vocab_sort_temp_bytes(V);
      p.off_sort_temp = off; off += align_up(p.sort_temp_bytes, 256);
    }
    if (lists) {
      const size_t n_tiles = (size_t)(p.Np / 256), v_tiles = (size_t)((V + 255) / 256), slab_tiles = (size_t)(vs / 256);
      const size_t slabs = (v_tiles + slab_tiles - 1) / slab_tiles;
      p.off_tile_flag = off;  off += align_up(n_tiles * v_tiles, 256);
      p.off_tile_list = off;  off += align_up(slabs * n_tiles * slab_tiles * 4, 256);
      p.off_tile_count = off; off += align_up(slabs * 4, 256);
    }
    if (compact) {
      p.off_idx = off;   off += align_up((size_t)N * 4, 256);
      p.off_count = off; off += 256;
      p.off_Ec = off;    off += align_up((size_t)p.Np * D * 2, 256);
    }
  } else {
    p.Np = N;
    p.off_flags[0] = off;
    off += align_up((size_t)((N + 63) / 64) * (vs / 64), 256);
    p.off_dEacc = off;
    off += align_up((size_t)N * D * 4, 256);
    p.off_GZ[0] = off;
    off += align_up((size_t)N * vs * 4, 256);
  }
  p.total_bytes = off;
  return p;
}

int64_t slab_tile(bool mfma) { return mfma ? 256 : 64; }

// Small batches: the slab widens as the batch shrinks (the GZ slab keeps its size) so that the
// recompute still has a tile for every CU.
int64_t recommended_slab(bool mfma, int64_t N, int64_t V) {
  int64_t full = round_up(V, slab_tile(mfma));
  int64_t rec = mfma ? kMfmaSlabCols : kPlainSlabCols;
  if (mfma) {
    int64_t widen = 8192 / round_up(N, 256);
    if (widen > 8) widen = 8;
    if (widen > 1) rec *= widen;
  }
  return full < rec ? full : rec;
}

// Widest slab a larger workspace buys (CCE_OP_BACKWARD_WIDE).  Every slab costs one launch of each
// kernel and one read-modify-write pass over the dE accumulator whatever it contains, which is what
// a filtered pass mostly consists of; fewer, wider slabs cut exactly that.  Bounded by the 32-bit
// element offsets of the recompute kernel and by the step list a filtered dE product keeps in LDS.
int64_t widest_slab(bool mfma, int64_t N, int64_t V) {
  const int64_t rec = recommended_slab(mfma, N, V);
  if (!mfma) return rec;
  int64_t wide = rec * kWideSlabFactor;
  const int64_t by_offsets = (((int64_t)1 << 30) / round_up(N, 256)) / 256 * 256;
  const int64_t by_steps = (int64_t)kMaxFilteredKSteps * 64;
  if (wide > by_offsets) wide = by_offsets;
  if (wide > by_steps) wide = by_steps;
  const int64_t full = round_up(V, 256);
  if (wide > full) wide = full;
  return wide > rec ? wide : rec;
}

// widest slab (multiple of the tile width, at most the widest one above) that fits `bytes`
int64_t fit_slab(bool mfma, int64_t N, int64_t D, int64_t V, size_t bytes, bool sort, bool lists, bool compact) {
  const int64_t t = slab_tile(mfma);
  int64_t lo = 0, hi = widest_slab(mfma, N, V) / t;   // in tiles
  if (mfma) {
    // the recompute kernel addresses the slab with 32-bit element offsets
    const int64_t cap = (((int64_t)1 << 30) / round_up(N, 256)) / t;
    if (hi > cap) hi = cap;
  }
  while (lo < hi) {
    int64_t mid = (lo + hi + 1) / 2;
    if (layout_backward(mfma, N, D, V, mid * t, sort, lists, compact).total_bytes <= bytes) lo = mid; else hi = mid - 1;
  }
  return lo * t;
}

}  // namespace

// =============================================================================
extern "C" {

void cce_default_opts(int dtype, cce_opts* opts) {
  if (!opts) return;
  memset(opts, 0, sizeof(*opts));
  opts->dtype = dtype;
  if (dtype == CCE_BF16) {
    opts->flags = CCE_FILTER_DE | CCE_FILTER_DC;
    opts->filter_eps = 0x1p-12f;
  }
}

const char* cce_strerror(int status) {
  switch (status) {
    case CCE_OK: return "success";
    case CCE_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, bad softcap or eps)";
    case CCE_EWORKSPACE: return "workspace missing or too small (see cce_workspace_bytes)";
    case CCE_EUNSUPPORTED: return "unsupported dtype, flag combination, or a size beyond the kernels' 32-bit offsets";
    case CCE_EHIP: return g_hip_error;
    case CCE_ESCRATCH: return g_noalloc_error;
    default: return "unknown status";
  }
}

size_t cce_workspace_bytes(int op, int64_t N, int64_t D, int64_t V, const cce_opts* opts) {
  if (!opts || N <= 0 || D <= 0 || V <= 0) return 0;
  if (opts->dtype != CCE_BF16 && opts->dtype != CCE_F32) return 0;
  const bool mfma = use_mfma(D, opts);
  const bool sort = mfma && (opts->flags & CCE_VOCAB_SORT);
  const bool lists = mfma && !sort && (opts->flags & CCE_SKIP_TILES);
  const bool compact = mfma && (opts->flags & CCE_COMPACT_IGNORED);
  switch (op) {
    case CCE_OP_FORWARD: return plan_forward(N, D, V, opts).total_bytes;
    case CCE_OP_BACKWARD:
      return layout_backward(mfma, N, D, V, recommended_slab(mfma, N, V), sort, lists, compact).total_bytes;
    case CCE_OP_BACKWARD_MIN: return layout_backward(mfma, N, D, V, slab_tile(mfma), sort, lists, compact).total_bytes;
    case CCE_OP_BACKWARD_WIDE:
      return layout_backward(mfma, N, D, V, widest_slab(mfma, N, V), sort, lists, compact).total_bytes;
    default: return 0;
  }
}

size_t cce_block_max_bytes(int64_t N, int64_t V) {
  if (N <= 0 || V <= 0) return 0;
  return block_max_bytes(N, V);
}

void cce_filter_block(int64_t N, int64_t D, int64_t V, const cce_opts* opts, int* block_rows, int* block_cols) {
  (void)N;
  (void)V;
  const bool mfma = opts && use_mfma(D, opts);
  // MFMA path: dE skips (256 tokens x 64 vocab) blocks, dC skips (64 x 256); the
  // common refinement 64 x 64 is what both tests see as "kept together".
  if (block_rows) *block_rows = mfma ? 256 : 64;
  if (block_cols) *block_cols = mfma ? 64 : 64;
}

int cce_forward_ex(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                   float softcap, int64_t ignore_index, float* out_loss, float* out_lse, const cce_opts* opts) {
  int st = check_common(E, C, targets, N, D, V, softcap, opts);
  if (st != CCE_OK) return st;
  if (!out_loss || !out_lse) return CCE_EINVAL;
  const FwdPlan plan = plan_forward(N, D, V, opts);
  if (!opts->workspace || opts->workspace_bytes < plan.total_bytes) return CCE_EWORKSPACE;
  hipStream_t stream = (hipStream_t)opts->stream;
  ForwardStats* fstats = (ForwardStats*)opts->workspace;
  LsePartial* partial = (LsePartial*)((char*)opts->workspace + plan.off_partial);
  const int* n_dev = nullptr;
  const int* idx = nullptr;
  if (plan.compact) {
    if ((uint64_t)N * (uint64_t)D * 2 >= ((uint64_t)1 << 32)) return CCE_EUNSUPPORTED;
    char* ws = (char*)opts->workspace;
    int* idx_w = (int*)(ws + plan.off_idx);
    int* count_w = (int*)(ws + plan.off_count);
    bf16* Ec = (bf16*)(ws + plan.off_Ec);
    CCE_HIP(launch_compact_tokens(targets, (int)N, (int)V, ignore_index, idx_w, count_w, &fstats->bad_targets, stream));
    CCE_HIP(launch_gather_tokens((const bf16*)E, idx_w, count_w, (int)N, (int)D, Ec, stream));
    // ignored tokens: loss 0 (and lse 0, documented as unspecified)
    CCE_HIP(launch_fill_f32(out_loss, N, 0.f, stream));
    CCE_HIP(launch_fill_f32(out_lse, N, 0.f, stream));
    E = Ec;
    n_dev = count_w;
    idx = idx_w;
  }

  if (plan.mfma) {
    FwdMfmaParams p{};
    p.E = (const bf16*)E;
    p.n_dev = n_dev;
    p.C = (const bf16*)C;
    p.N = (int)N; p.D = (int)D; p.V = (int)V;
    p.softcap = softcap;
    p.partial = partial;
    p.v_tiles = plan.v_tiles;
    p.plan = plan.plan;
    p.want_wgs = plan.want_wgs; p.round_cap = plan.round_cap;
    p.grid = plan.grid;
    p.bad_targets = plan.compact ? nullptr : &fstats->bad_targets;
    if ((opts->flags & CCE_SKIP_TILES) && opts->block_max) {
      p.block_max = (uint16_t*)opts->block_max;
      p.block_max_stride = (int)round_up(N, 256);
    }
    CCE_HIP(launch_fwd_lse_mfma(p, stream));
  } else {
    FwdPlainParams p{};
    p.E = E; p.C = C; p.dtype = opts->dtype;
    p.N = (int)N; p.D = (int)D; p.V = (int)V;
    p.softcap = softcap;
    p.partial = partial;
    p.splits = plan.splits; p.tiles_per_split = plan.tiles_per_split;
    p.bad_targets = &fstats->bad_targets;
    CCE_HIP(launch_fwd_lse_plain(p, stream));
  }
  FinalizeParams f{};
  f.E = E; f.C = C; f.dtype = opts->dtype; f.targets = targets;
  f.N = (int)N; f.D = (int)D; f.V = (int)V;
  f.softcap = softcap; f.ignore_index = ignore_index;
  f.partial = partial; f.splits = plan.splits;
  f.out_loss = out_loss; f.out_lse = out_lse;
  f.n_dev = n_dev; f.idx = idx;
  f.bad_targets = plan.compact ? nullptr : &fstats->bad_targets;
  f.v_tiles = plan.v_tiles; f.want_wgs = plan.want_wgs; f.round_cap = plan.round_cap;
  CCE_HIP(launch_finalize(f, stream));
  return CCE_OK;
}

}  // extern "C"

namespace {

// Everything the MFMA backward enqueues, slab after slab.  `forked[i]` is set as soon as work has
// been put on helper stream i, so that the caller can join exactly those streams back into the
// caller's stream whether this returns success or a failure half way.
int enqueue_backward_mfma(const BwdCommon& c0, const BwdPlan& plan, Helpers* h, const void* C, const int64_t* targets,
                          const float* lse, int64_t N, int64_t D, int64_t V, int64_t vs, bool sort, bool lists_layout,
                          bool compact, const void* E, void* out_dC, const cce_opts* opts, char* ws,
                          hipStream_t stream, bool (&forked)[3], int* ksplit_out, const int** n_dev_out,
                          const int** idx_out) {
  BwdCommon c = c0;
  const int64_t ignore_index = c.ignore_index;
  BwdMfmaSlab s{};
  s.Np = (int)plan.Np;
  s.dEacc = (float*)(ws + plan.off_dEacc);
  s.ksplit = dE_ksplit(N, D);
  s.dE_part_stride = N * D;
  s.acc_mode = (opts->flags & CCE_ACCUM_KAHAN) ? 2 : (opts->flags & CCE_ACCUM_BF16) ? 1 : 0;
  *ksplit_out = s.ksplit;
  const bool serial = (opts->flags & CCE_SINGLE_STREAM) != 0;
  // a filtered contraction keeps its list of 64-wide steps in LDS; longer ones (N > 131072) run unfiltered
  if (plan.Np / 64 > kMaxFilteredKSteps) c.filter_dC = 0;
  CCE_HIP(launch_clear_stats(c.stats, stream));
  // helper work may not start before the caller's earlier work on `stream` (which may produce C)
  if (!serial) CCE_HIP(hipEventRecord(h->started, stream));
  if (compact) {
    int* idx_w = (int*)(ws + plan.off_idx);
    int* count_w = (int*)(ws + plan.off_count);
    bf16* Ec = (bf16*)(ws + plan.off_Ec);
    CCE_HIP(launch_compact_tokens(targets, (int)N, (int)V, ignore_index, idx_w, count_w, nullptr, stream));
    CCE_HIP(launch_gather_tokens((const bf16*)E, idx_w, count_w, (int)N, (int)D, Ec, stream));
    c.E = Ec;              // the vocabulary sort below keeps using the caller's E (its key is a batch mean)
    c.n_dev = count_w;
    c.idx = idx_w;
    *n_dev_out = count_w;
    *idx_out = idx_w;
  }
  if (sort) {
    VocabSortParams v{};
    v.E = (const bf16*)E; v.C = (const bf16*)C; v.targets = targets;
    v.N = (int)N; v.D = (int)D; v.V = (int)V; v.ignore_index = ignore_index;
    v.partial = (float*)(ws + plan.off_partial);
    v.mean = (float*)(ws + plan.off_mean);
    v.key = (float*)(ws + plan.off_key);
    v.key_sorted = (float*)(ws + plan.off_key_sorted);
    v.index = (int*)(ws + plan.off_index);
    v.perm = (int*)(ws + plan.off_perm);
    v.inverse = (int*)(ws + plan.off_inverse);
    v.targets_sorted = (int64_t*)(ws + plan.off_targets);
    v.temp = ws + plan.off_sort_temp;
    v.temp_bytes = plan.sort_temp_bytes;
    CCE_HIP(launch_vocab_sort(v, stream));   // the scratch size was checked before the first launch
    c.targets = v.targets_sorted;    // from here on the vocabulary is indexed by sorted position
    s.perm = v.perm;
  }
  const bool use_lists = lists_layout && opts->block_max && c.filter_dE && c.filter_dC && c.eps > 0.f;
  const int64_t slab_tiles = vs / 256;
  if (use_lists) {
    TileListParams t{};
    t.block_max = (const uint16_t*)opts->block_max;
    t.stride = (int)plan.Np;
    t.targets = targets; t.lse = lse;
    t.n_dev = c.n_dev; t.idx = c.idx;
    t.N = (int)N; t.V = (int)V; t.ignore_index = ignore_index;
    t.log_eps = logf(c.eps) - 0.02f;   // margin for the fp32 rounding of lse and of the recorded maxima
    t.n_tiles = (int)(plan.Np / 256); t.v_tiles = (int)((V + 255) / 256);
    t.slab_tiles = (int)slab_tiles;
    t.slabs = (int)((t.v_tiles + slab_tiles - 1) / slab_tiles);
    t.tile_flag = (uint8_t*)(ws + plan.off_tile_flag);
    t.tile_list = (uint32_t*)(ws + plan.off_tile_list);
    t.tile_count = (uint32_t*)(ws + plan.off_tile_count);
    CCE_HIP(launch_tile_lists(t, stream));
  }
  const int64_t n_slabs = (round_up(V, 256) + vs - 1) / vs;
  uint32_t* flags_all = (uint32_t*)(ws + plan.off_flags[0]);
  CCE_HIP(launch_zero_flags(flags_all, n_slabs * (int64_t)plan.flag_region_words, stream));
  const int cus = cu_count();
  int64_t slab = 0;
  for (int64_t v0 = 0; v0 < V; v0 += vs, ++slab) {
    const int b = (int)(slab % kSlabBuffers), e = (int)(slab % kEventRing);
    const int64_t vs_this = (round_up(V - v0, 256) < vs) ? round_up(V - v0, 256) : vs;
    s.v0 = (int)v0;
    s.vs = (int)vs_this;
    s.first = v0 == 0;
    s.GZ = (bf16*)(ws + plan.off_GZ[b]);
    s.flags_nv = flags_all + slab * (int64_t)plan.flag_region_words;
    s.flags_vn = s.flags_nv + (plan.Np / 256) * (vs_this / 64);
    if (!serial && slab >= kSlabBuffers) {
      // this slab's buffers were last read by the products of slab - kSlabBuffers
      const int e2 = (int)((slab - kSlabBuffers) % kEventRing);
      CCE_HIP(hipStreamWaitEvent(stream, h->dC_done[e2], 0));
      CCE_HIP(hipStreamWaitEvent(stream, h->dE_done[e2], 0));
    }
    const int64_t rows_valid = (V - v0 < vs_this) ? V - v0 : vs_this;
    s.Crows = (const bf16*)C + v0 * D;
    if (use_lists) {
      s.tile_list = (const uint32_t*)(ws + plan.off_tile_list) + slab * (plan.Np / 256) * slab_tiles;
      s.tile_count = (const uint32_t*)(ws + plan.off_tile_count) + slab;
    }
    if (sort) {
      // the slab's rows of C, gathered in sorted order (its buffer was last read by the
      // recompute and the dE product of the slab that used it before, both waited for above)
      bf16* Cs = (bf16*)(ws + plan.off_Cs[b]);
      CCE_HIP(launch_gather_rows((const bf16*)C, s.perm, (int)v0, (int)rows_valid, (int)D, Cs, stream));
      s.Crows = Cs;
    }
    CCE_HIP(launch_bwd_recompute_mfma(c, s, cus, stream));
    if (serial) {
      CCE_HIP(launch_bwd_dC_mfma(c, s, out_dC, stream));
      CCE_HIP(launch_bwd_dE_mfma(c, s, stream));
      continue;
    }
    CCE_HIP(hipEventRecord(h->recomputed[e], stream));
    // dC products of consecutive slabs write disjoint rows: they alternate between two
    // streams so that the last, partly filled round of one overlaps the next one's start
    const int dC_i = (slab & 1) ? 2 : 0;
    hipStream_t dC_stream = h->product[dC_i], dE_stream = h->product[1];
    // a helper stream's first work of the call waits for the caller's earlier work on `stream`
    if (!forked[dC_i]) CCE_HIP(hipStreamWaitEvent(dC_stream, h->started, 0));
    forked[dC_i] = true;
    CCE_HIP(hipStreamWaitEvent(dC_stream, h->recomputed[e], 0));
    CCE_HIP(launch_bwd_dC_mfma(c, s, out_dC, dC_stream));
    CCE_HIP(hipEventRecord(h->dC_done[e], dC_stream));
    // dEacc is read-modify-written slab after slab: stream order keeps that sequence
    if (!forked[1]) CCE_HIP(hipStreamWaitEvent(dE_stream, h->started, 0));
    forked[1] = true;
    CCE_HIP(hipStreamWaitEvent(dE_stream, h->recomputed[e], 0));
    CCE_HIP(launch_bwd_dE_mfma(c, s, dE_stream));
    CCE_HIP(hipEventRecord(h->dE_done[e], dE_stream));
  }
  return CCE_OK;
}

}  // namespace

extern "C" {

int cce_backward_ex(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                    float softcap, int64_t ignore_index, const float* lse, const float* dLoss, void* out_dE,
                    void* out_dC, const cce_opts* opts) {
  int st = check_common(E, C, targets, N, D, V, softcap, opts);
  if (st != CCE_OK) return st;
  if (!lse || !dLoss || !out_dE || !out_dC) return CCE_EINVAL;
  if (!aligned(out_dE, 16) || !aligned(out_dC, 16)) return CCE_EINVAL;
  const bool mfma = use_mfma(D, opts);
  const bool sort = (opts->flags & CCE_VOCAB_SORT) != 0;
  if (sort && !mfma) return CCE_EUNSUPPORTED;   // vocabulary sorting exists on the bf16 MFMA path only
  const bool acc_bf16 = (opts->flags & (CCE_ACCUM_BF16 | CCE_ACCUM_KAHAN)) != 0;
  if (acc_bf16 && !mfma) return CCE_EUNSUPPORTED;   // so do the bf16 accumulation variants
  // the MFMA gradient products address E with 32-bit byte offsets (whatever the workspace)
  if (mfma && (uint64_t)N * (uint64_t)D * 2 >= ((uint64_t)1 << 32)) return CCE_EUNSUPPORTED;
  if (!opts->workspace) return CCE_EWORKSPACE;
  // the workspace is laid out for work lists whenever the flag asks for them (as sized by
  // cce_workspace_bytes); they are used only when nothing but filtered products reads GZ
  const bool lists_layout = mfma && !sort && (opts->flags & CCE_SKIP_TILES);
  const bool compact = mfma && (opts->flags & CCE_COMPACT_IGNORED);
  const int64_t vs = fit_slab(mfma, N, D, V, opts->workspace_bytes, sort, lists_layout, compact);
  if (vs <= 0) return CCE_EWORKSPACE;
  const BwdPlan plan = layout_backward(mfma, N, D, V, vs, sort, lists_layout, compact);
  hipStream_t stream = (hipStream_t)opts->stream;
  char* ws = (char*)opts->workspace;

  BwdCommon c{};
  c.E = E; c.C = C; c.dtype = opts->dtype; c.targets = targets; c.lse = lse; c.dloss = dLoss;
  c.N = (int)N; c.D = (int)D; c.V = (int)V;
  c.softcap = softcap; c.ignore_index = ignore_index;
  c.eps = opts->filter_eps;
  c.filter_dE = (opts->flags & CCE_FILTER_DE) ? 1 : 0;
  c.filter_dC = (opts->flags & CCE_FILTER_DC) ? 1 : 0;
  c.stats = (FilterStats*)ws;
  float* dEacc = (float*)(ws + plan.off_dEacc);

  if (mfma) {
    // ---- everything that can refuse the call, before the first launch
    // ... and a slab of C likewise
    if ((uint64_t)vs * (uint64_t)D * 2 >= ((uint64_t)1 << 32)) return CCE_EUNSUPPORTED;
    // a work-list entry packs the token tile and the slab-local vocabulary tile into 16 bits each,
    // and the tile-flag kernel puts the token tiles into grid.y
    if (lists_layout && (plan.Np / 256 > 65535 || vs / 256 > 65535)) return CCE_EUNSUPPORTED;
    if (sort) {
      size_t need = 0;
      CCE_HIP(vocab_sort_temp_needed(V, &need));
      if (need > plan.sort_temp_bytes) return CCE_EWORKSPACE;
    }
    Helpers* h = nullptr;
    st = helpers_for_device(&h);
    if (st != CCE_OK) return st;
    std::lock_guard<std::mutex> lock(h->mutex);
    bool forked[3] = {false, false, false};
    int ksplit = 1;
    const int* n_dev = nullptr;
    const int* idx = nullptr;
    st = enqueue_backward_mfma(c, plan, h, C, targets, lse, N, D, V, vs, sort, lists_layout, compact, E, out_dC, opts, ws,
                               stream, forked, &ksplit, &n_dev, &idx);
    // join every helper stream that got work back into the caller's stream, also after a failure half
    // way (a capture must not be left with unjoined streams)
    for (int i = 0; i < 3; ++i) {
      if (!forked[i]) continue;
      hipError_t e1 = hipEventRecord(h->joined[i], h->product[i]);
      hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(stream, h->joined[i], 0) : e1;
      if (e2 != hipSuccess && st == CCE_OK) st = hip_fail(e2, "joining a helper stream");
    }
    if (st != CCE_OK) return st;   // outputs are undefined after a failure past the first launch
    const int64_t n_slabs = (round_up(V, 256) + vs - 1) / vs;
    CCE_HIP(launch_count_flags((const uint32_t*)(ws + plan.off_flags[0]), (int64_t)plan.flag_region_words, (int)n_slabs,
                               (int)(plan.Np / 256), (int)vs, (int)V, c.stats, n_dev, stream));
    CCE_HIP(launch_store_dE(dEacc, ksplit, out_dE, opts->dtype, N, D, idx, n_dev, acc_bf16, stream));
    return CCE_OK;
  }
  CCE_HIP(launch_clear_stats(c.stats, stream));
  BwdPlainSlab s{};
  s.GZ = (float*)(ws + plan.off_GZ[0]);
  s.dEacc = dEacc;
  s.flags = (uint8_t*)(ws + plan.off_flags[0]);
  for (int64_t v0 = 0; v0 < V; v0 += vs) {
    const int64_t vs_this = (round_up(V - v0, 64) < vs) ? round_up(V - v0, 64) : vs;
    s.v0 = (int)v0;
    s.vs = (int)vs_this;
    s.first = v0 == 0;
    CCE_HIP(launch_bwd_gz_plain(c, s, stream));
    CCE_HIP(launch_bwd_dC_plain(c, s, out_dC, stream));
    CCE_HIP(launch_bwd_dE_plain(c, s, stream));
  }
  CCE_HIP(launch_store_dE(dEacc, 1, out_dE, opts->dtype, N, D, nullptr, nullptr, false, stream));
  return CCE_OK;
}

int cce_set_workspace(void* workspace, size_t workspace_bytes) {
  if ((workspace == nullptr) != (workspace_bytes == 0)) return CCE_EINVAL;
  if (workspace && !aligned(workspace, 256)) return CCE_EINVAL;
  int dev = 0;
  CCE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CCE_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_lent_mutex);
  g_lent[dev].ptr = workspace;
  g_lent[dev].bytes = workspace_bytes;
  return CCE_OK;
}

int cce_forward(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                float softcap, int64_t ignore_index, float* out_loss, float* out_lse) {
  cce_opts o;
  cce_default_opts(CCE_BF16, &o);
  int st = check_common(E, C, targets, N, D, V, softcap, &o);
  if (st != CCE_OK) return st;
  LentWorkspace w;
  st = lent_workspace(&w);
  if (st != CCE_OK) return st;
  o.workspace = w.ptr;
  o.workspace_bytes = w.bytes;      // cce_forward_ex checks it against the exact requirement
  return cce_forward_ex(E, C, targets, N, D, V, softcap, ignore_index, out_loss, out_lse, &o);
}

int cce_forward_noalloc(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                        float softcap, int64_t ignore_index, float* out_loss, float* out_lse, const cce_opts* opts) {
  // every check of cce_forward_ex that does not concern the workspace, before anything else
  int st = check_common(E, C, targets, N, D, V, softcap, opts);
  if (st != CCE_OK) return st;
  if (!out_loss || !out_lse) return CCE_EINVAL;
  const size_t need = plan_forward(N, D, V, opts).total_bytes;
  if (need > kStaticScratchBytes) {
    snprintf(g_noalloc_error, sizeof(g_noalloc_error),
             "cce_forward_noalloc: this call needs %zu bytes of scratch, the library's static array holds %zu "
             "(use cce_forward_ex with a caller workspace)", need, kStaticScratchBytes);
    return CCE_ESCRATCH;
  }
  cce_opts o = *opts;
  st = static_scratch(&o.workspace);
  if (st != CCE_OK) return st;
  o.workspace_bytes = kStaticScratchBytes;
  // The forward kernels write every (split, token) partial the finalize kernel reads, and the first of them
  // clears the out-of-range-target counter at the head of the scratch: what an earlier call left in the
  // array is never read.
  return cce_forward_ex(E, C, targets, N, D, V, softcap, ignore_index, out_loss, out_lse, &o);
}

size_t cce_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int cce_backward(const void* E, const void* C, const int64_t* targets, int64_t N, int64_t D, int64_t V,
                 float softcap, int64_t ignore_index, const float* lse, const float* dLoss, void* out_dE,
                 void* out_dC) {
  cce_opts o;
  cce_default_opts(CCE_BF16, &o);
  int st = check_common(E, C, targets, N, D, V, softcap, &o);
  if (st != CCE_OK) return st;
  LentWorkspace w;
  st = lent_workspace(&w);
  if (st != CCE_OK) return st;
  o.workspace = w.ptr;
  o.workspace_bytes = w.bytes;      // cce_backward_ex uses the widest slab that fits it
  return cce_backward_ex(E, C, targets, N, D, V, softcap, ignore_index, lse, dLoss, out_dE, out_dC, &o);
}

int cce_forward_target_stats(const void* workspace, void* stream, uint64_t* out_of_range) {
  if (!out_of_range) return CCE_EINVAL;
  if (!workspace) {
    // the workspace lent to the plain entry points
    LentWorkspace w;
    int st = lent_workspace(&w);
    if (st != CCE_OK) return st;
    workspace = w.ptr;
  }
  ForwardStats host{};
  CCE_HIP(hipMemcpyAsync(&host, workspace, sizeof(host), hipMemcpyDeviceToHost, (hipStream_t)stream));
  CCE_HIP(hipStreamSynchronize((hipStream_t)stream));
  *out_of_range = host.bad_targets;
  return CCE_OK;
}

int cce_backward_filter_stats(const void* workspace, void* stream, uint64_t* blocks_total, uint64_t* blocks_kept) {
  if (!blocks_total || !blocks_kept) return CCE_EINVAL;
  if (!workspace) {
    // the workspace lent to the plain entry points
    LentWorkspace w;
    int st = lent_workspace(&w);
    if (st != CCE_OK) return st;
    workspace = w.ptr;
  }
  FilterStats host{};
  CCE_HIP(hipMemcpyAsync(&host, workspace, sizeof(host), hipMemcpyDeviceToHost, (hipStream_t)stream));
  CCE_HIP(hipStreamSynchronize((hipStream_t)stream));
  *blocks_total = host.blocks_total;
  *blocks_kept = host.blocks_kept;
  return CCE_OK;
}

}  // extern "C"
