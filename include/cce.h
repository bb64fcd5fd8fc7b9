/*
 * cce.h - C ABI of the MI355X (gfx950) fused linear cross-entropy library.
 *
 * The library computes the per-token cross-entropy of a linear classifier
 * without ever writing the N x |V| logit matrix to device memory
 * (paper Section 3, Eq. 4:  l_i = C_{x_i}^T E_i - log sum_j exp(C_j^T E_i);
 * this library returns the negative of l_i, the usual NLL).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device.  The
 *     caller owns every buffer; the library only reads inputs and writes the
 *     outputs / the workspace named in the call.
 *   - E is [N, D] and C is [V, D], row-major, contiguous (leading dimension D):
 *     the paper's D x N / D x |V| matrices, whose columns are the tokens / the
 *     vocabulary entries (Appendix A), stored with that index outermost.
 *     Element type: bfloat16 (CCE_BF16) or float (CCE_F32); E, C, out_dE and
 *     out_dC share it.  Pointers must be 16-byte aligned.
 *   - targets is int64 [N].  A token is "ignored" when its target equals
 *     ignore_index or lies outside [0, V): it gets loss 0, contributes nothing
 *     to dE / dC, and its dLoss entry is not read (Appendix B: ignored tokens
 *     change neither loss nor gradient).  Targets outside [0, V) other than
 *     ignore_index are counted (cce_forward_target_stats).
 *   - softcap == 0 disables logit soft-capping; softcap > 0 replaces every
 *     logit z by softcap * tanh(z / softcap) (the soft-capping named in
 *     Table A2; formula is this library's reading).  Negative or NaN: CCE_EINVAL.
 *   - Calls are asynchronous on a HIP stream (opts->stream, or the null stream
 *     for the plain entry points) and never synchronise it.  Work that the
 *     library spreads over helper streams is joined back into that stream
 *     before the call returns.
 *   - The library never allocates, frees or synchronises device memory: all
 *     scratch is the caller's (opts->workspace, or the buffer lent with
 *     cce_set_workspace for the plain entry points).  Per device it creates
 *     three helper streams and a few events on the first backward call.
 *   - Return value: CCE_OK (0) or a negative cce_status.  On CCE_EINVAL,
 *     CCE_EUNSUPPORTED, CCE_EWORKSPACE and CCE_ESCRATCH nothing has been
 *     launched and no output has been written.  After CCE_EHIP (a launch or
 *     runtime call failed part-way) the outputs are undefined; helper streams
 *     that had been given work are still joined back into the caller's stream.
 *   - Results are bitwise reproducible from call to call: no atomics and no
 *     lock-ordered reductions are used (the paper's Alg. 2 / Alg. 4 use
 *     spin-locks; Section 4.2 itself notes alternatives may be preferable).
 */
#ifndef CCE_H_
#define CCE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cce_status {
  CCE_OK = 0,
  CCE_EINVAL = -1,       /* null / misaligned pointer, non-positive size, bad softcap or eps */
  CCE_EWORKSPACE = -2,   /* opts->workspace missing or smaller than the minimum */
  CCE_EUNSUPPORTED = -3, /* unknown dtype or flag, or a size beyond the kernels' 32-bit offsets
                            (backward on the MFMA path: N * D * 2 bytes must stay below 4 GiB) */
  CCE_EHIP = -4,         /* a HIP runtime call failed; see cce_strerror */
  CCE_ESCRATCH = -5      /* cce_forward_noalloc: the problem needs more scratch than the library's static
                            array holds (cce_noalloc_scratch_bytes); cce_strerror gives both figures */
} cce_status;

enum { CCE_BF16 = 0, CCE_F32 = 1 };

/* cce_opts.flags */
enum {
  CCE_FILTER_DE = 1u << 0,   /* apply gradient filtering to dE (Section 4.3) */
  CCE_FILTER_DC = 1u << 1,   /* apply gradient filtering to dC; clearing only this bit is the
                                paper's "CCE-Kahan-FullC" choice, clearing only FILTER_DE "FullE".
                                MFMA path with N > 131072 tokens: dC is computed unfiltered whatever this
                                bit says (a filtered contraction over tokens keeps its list of kept
                                64-token steps in LDS, 2048 entries); still within every tolerance, since
                                the filter only ever drops terms */
  CCE_VOCAB_SORT = 1u << 2,  /* backward only: walk the vocabulary in descending order of each entry's
                                mean logit over the batch (Section 4.3, "Vocabulary sorting"), so that
                                entries with non-negligible softmax mass share filter blocks.  The mean
                                is taken before the soft-cap, where it equals <C_j, mean_i E_i>.  Changes
                                which blocks the filter skips, never the unfiltered result (beyond the
                                fp32 summation order of dE).  bf16 MFMA path only (CCE_EUNSUPPORTED
                                otherwise); costs O(|V|) extra workspace plus two slab-sized copies of C
                                rows.  The forward pass ignores the flag. */
  CCE_PLAIN_KERNELS = 1u << 3, /* run the plain fp32-FMA kernels instead of the MFMA ones (always used
                                for CCE_F32 and for shapes the MFMA kernels do not take) */
  CCE_COMPACT_IGNORED = 1u << 5, /* remove ignored tokens before the work (Appendix B): the kernels run on a
                                compacted copy of the rows of E whose target is valid, so the cost scales
                                with the number of valid tokens.  Loss, dE and dC are unchanged (loss and dE
                                rows of ignored tokens are 0); out_lse of ignored tokens is then unspecified.
                                Forward and backward are independent in this (either may set it; with
                                CCE_SKIP_TILES both must agree).  bf16 MFMA path only, ignored otherwise.
                                Costs one copy of E in the workspace. */
  CCE_SINGLE_STREAM = 1u << 6, /* backward: enqueue every kernel on the caller's stream.  By default the MFMA
                                backward spreads a slab's recompute and its two gradient products over
                                helper streams (joined back before the call returns); this flag gives the
                                plain sequence, slower, e.g. for per-kernel profiling. */
  CCE_ACCUM_BF16 = 1u << 7,  /* backward: keep dE's running sum over vocabulary slabs in bf16 in device memory, rounded
                                after every slab, instead of fp32.  This is the paper's own choice for its sums in
                                global memory ("the final gradient floating point type", Section 5) and is offered to
                                measure what it costs in accuracy: the error grows with the number of slabs.  dC is
                                not affected (each of its rows is complete after one pass, there is no sum in device
                                memory).  bf16 MFMA path only (CCE_EUNSUPPORTED otherwise).  Same workspace size. */
  CCE_ACCUM_KAHAN = 1u << 8, /* backward: as CCE_ACCUM_BF16 (implied) with Kahan-compensated summation, the paper's
                                "CCE-Kahan" (Section 5): a second bf16 array holds the rounding error of the running
                                sum and is subtracted from the next slab's contribution.  Both arrays together take
                                the bytes of the fp32 accumulator they replace. */
  CCE_SKIP_TILES = 1u << 4    /* forward: also record, in opts->block_max, the largest logit of every token
                                within each 128-wide vocabulary block; backward (with both CCE_FILTER_* set
                                and filter_eps > 0): do not even recompute the logit tiles in which that
                                record shows no softmax entry can reach filter_eps and which hold no target.
                                With CCE_COMPACT_IGNORED the record is indexed by compacted token, so
                                forward and backward must then both set (or both clear) that flag.
                                The gradients are bit-identical to the filtered backward without the flag
                                (only tiles whose blocks the filter drops anyway are left out); Alg. 3 / 4
                                recompute every tile first and test afterwards.  bf16 MFMA path only; ignored
                                together with CCE_VOCAB_SORT (the record is in forward vocabulary order).
                                Costs 2 * |V| / 128 bytes per token (cce_block_max_bytes). */
};

/* cce_workspace_bytes(op, ...) */
enum {
  CCE_OP_FORWARD = 0,        /* exact requirement of cce_forward_ex */
  CCE_OP_BACKWARD = 1,       /* recommended size for cce_backward_ex: the narrowest slabs at which the
                                unfiltered pass runs at full speed */
  CCE_OP_BACKWARD_MIN = 2,   /* smallest size cce_backward_ex accepts (narrowest slab) */
  CCE_OP_BACKWARD_WIDE = 3   /* largest size cce_backward_ex makes use of: slabs four times as wide.  Each
                                slab costs one launch per kernel and one pass over the fp32 dE accumulator
                                whatever the filter leaves of it, so a filtered pass gets faster with fewer,
                                wider slabs; an unfiltered one does not */
};

typedef struct cce_opts {
  int dtype;              /* CCE_BF16 or CCE_F32 */
  uint32_t flags;         /* any of the CCE_* flag bits above */
  float filter_eps;       /* gradient-filter threshold on |softmax - onehot|; 0 disables filtering.
                             The paper's value for bf16 is 2^-12 (Section 4.3). */
  void* workspace;        /* device scratch, 256-byte aligned, owned by the caller */
  size_t workspace_bytes;
  void* stream;           /* hipStream_t; NULL = null stream */
  void* block_max;        /* CCE_SKIP_TILES: device buffer of cce_block_max_bytes(N, V) bytes, 256-byte
                             aligned, owned by the caller; written by the forward call, read by the
                             backward call on the same inputs.  NULL = the flag has no effect. */
  size_t block_max_bytes;
} cce_opts;

/* Fills *opts with the defaults the plain entry points use for `dtype`:
 * bf16: FILTER_DE | FILTER_DC, filter_eps = 2^-12;  f32: no filtering (eps = 0).
 * workspace = NULL, stream = NULL. */
void cce_default_opts(int dtype, cce_opts* opts);

/*
 * Forward (Alg. 1 indexed matmul + Alg. 2 linear-log-sum-exp, Eq. 4).
 *   out_lse [N] float:  log sum_j exp(a_ij) for EVERY row, ignored or not.
 *   out_loss[N] float:  out_lse_i - a_{i,x_i} for valid tokens, 0 for ignored ones.
 * Extra device memory: the workspace only, O(N) floats; the logits live in
 * registers / LDS.  (CCE_COMPACT_IGNORED adds a copy of E, CCE_SKIP_TILES the
 * caller's block_max record.)
 *
 * cce_forward: bf16 inputs, default options, null stream, scratch taken from the
 * buffer lent with cce_set_workspace (CCE_EWORKSPACE when none is registered on
 * the current device or it is smaller than cce_workspace_bytes(CCE_OP_FORWARD)).
 */
int cce_forward(const void* E, const void* C, const int64_t* targets,
                int64_t N, int64_t D, int64_t V,
                float softcap, int64_t ignore_index,
                float* out_loss, float* out_lse);

int cce_forward_ex(const void* E, const void* C, const int64_t* targets,
                   int64_t N, int64_t D, int64_t V,
                   float softcap, int64_t ignore_index,
                   float* out_loss, float* out_lse, const cce_opts* opts);

/*
 * Forward for callers that cannot allocate device memory and have no workspace to lend: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as cce_forward_ex (bit-identical), except that
 * opts->workspace / workspace_bytes are ignored: the scratch (the per-split (max, sum) pairs)
 * lives in a static device array inside the library, cce_noalloc_scratch_bytes() = 8 MiB per
 * GPU the library runs on, held until the process ends.  The call allocates and frees
 * nothing, on the device or through any library.  A problem whose forward workspace
 * (cce_workspace_bytes(CCE_OP_FORWARD, ...)) exceeds the array is refused with CCE_ESCRATCH
 * before anything is launched: at the 8 vocabulary splits of a large batch that is N >= 131072
 * tokens, and any call with CCE_COMPACT_IGNORED whose copy of E does not fit.
 * Every call on one GPU shares that GPU's array, which keeps the previous call's contents
 * (never read: each call writes all the partials it merges, and its forward kernel clears the
 * one counter that must start at zero).  Calls that overlap on one GPU
 * (different streams, different threads) race on it; calls on one stream are safe.
 */
int cce_forward_noalloc(const void* E, const void* C, const int64_t* targets,
                        int64_t N, int64_t D, int64_t V,
                        float softcap, int64_t ignore_index,
                        float* out_loss, float* out_lse, const cce_opts* opts);

/* Size in bytes of the static scratch array behind cce_forward_noalloc. */
size_t cce_noalloc_scratch_bytes(void);

/*
 * Backward (Alg. 4, the merged linear-cross-entropy backward; gradient formula
 * of Section 4.3):  with S = exp(a - lse), G = S - onehot(x) (0 for ignored rows),
 *   out_dE[N, D] = sum_j dLoss_i G_ij a'_ij C_j,   out_dC[V, D] = sum_i dLoss_i G_ij a'_ij E_i,
 * a'_ij = 1 - (a_ij / softcap)^2 with soft-capping, else 1.
 *   lse   [N] float: out_lse of the forward call on the same inputs.
 *   dLoss [N] float: upstream gradient of out_loss.
 * Both outputs are OVERWRITTEN (not accumulated into), in the dtype of E / C,
 * accumulated in fp32 and rounded once.
 * Gradient filtering (Section 4.3): a block of G whose entries are all below
 * filter_eps in magnitude is left out of the products that have their
 * CCE_FILTER_* bit set.  Block shape is an implementation choice
 * (cce_filter_block reports it).
 * Extra device memory: the workspace: two slabs of the gradient-of-logits matrix
 * (bf16, N x slab width), fp32 [N, D] accumulator(s) and 4 bytes of filter flag per
 * 256 x 64 and 64 x 256 block of logits - the only part that grows with |V|.
 * Any workspace of at least cce_workspace_bytes(CCE_OP_BACKWARD_MIN) bytes is accepted; the
 * call uses the widest slab that fits it, up to that of CCE_OP_BACKWARD_WIDE.
 * Work that the call spreads over the library's helper streams is joined back into
 * opts->stream before it returns; the whole call can be captured into a HIP graph.
 *
 * cce_backward: bf16, null stream, filtering on at 2^-12, scratch taken from the buffer
 * lent with cce_set_workspace (any size from CCE_OP_BACKWARD_MIN up; CCE_EWORKSPACE
 * when none is registered on the current device or it is smaller than that).
 */
int cce_backward(const void* E, const void* C, const int64_t* targets,
                 int64_t N, int64_t D, int64_t V,
                 float softcap, int64_t ignore_index,
                 const float* lse, const float* dLoss,
                 void* out_dE, void* out_dC);

int cce_backward_ex(const void* E, const void* C, const int64_t* targets,
                    int64_t N, int64_t D, int64_t V,
                    float softcap, int64_t ignore_index,
                    const float* lse, const float* dLoss,
                    void* out_dE, void* out_dC, const cce_opts* opts);

/*
 * Lends the plain entry points (cce_forward, cce_backward) their scratch on the CURRENT device:
 * `workspace` is device memory of `workspace_bytes` bytes, 256-byte aligned, owned by the caller,
 * who keeps it alive and unused by anything else until it registers another buffer or NULL / 0
 * (which withdraws it).  Forward and backward calls share it, so calls that use it must not
 * overlap (one stream, or ordered by the caller).  cce_workspace_bytes(CCE_OP_BACKWARD, ...) of the
 * largest problem covers both.  The plain signatures carry no workspace argument and the
 * library does not allocate: this call is how memory reaches them.  Host-side only (nothing is
 * launched).  Returns CCE_OK, CCE_EINVAL (misaligned, or pointer / size inconsistent) or CCE_EHIP.
 */
int cce_set_workspace(void* workspace, size_t workspace_bytes);

/* Workspace size in bytes for `op` (CCE_OP_*) at this shape and these options
 * (dtype and flags are read; workspace fields are not).  0 on invalid arguments. */
size_t cce_workspace_bytes(int op, int64_t N, int64_t D, int64_t V, const cce_opts* opts);

/* Size in bytes of the block-maximum record of CCE_SKIP_TILES; 0 on invalid arguments. */
size_t cce_block_max_bytes(int64_t N, int64_t V);

/* Rows (tokens) x columns (vocabulary entries) of the block the gradient filter
 * tests as a unit, for the kernels `opts` selects at this shape. */
void cce_filter_block(int64_t N, int64_t D, int64_t V, const cce_opts* opts,
                      int* block_rows, int* block_cols);

/* Number of targets of the last forward call that used this workspace (NULL: the buffer lent
 * with cce_set_workspace) which were neither ignore_index nor inside [0, V).  Such targets are
 * treated as ignored (no access out of bounds, loss 0, no gradient); this call is how a caller
 * learns of them: the paper is silent on invalid labels, and a device-side count read after the
 * fact keeps the hot path free of synchronisation.  Synchronises `stream` (a reporting call).
 * Not available for cce_forward_noalloc, whose scratch is not addressable by the caller. */
int cce_forward_target_stats(const void* workspace, void* stream, uint64_t* out_of_range);

/* Host-side counters of the last cce_backward(_ex) call that used this
 * workspace (NULL: the buffer lent with cce_set_workspace): number of filter blocks
 * visited and number kept.  Synchronises
 * `stream` (this is a reporting call, not part of the hot path).
 * Returns CCE_OK or a negative status. */
int cce_backward_filter_stats(const void* workspace, void* stream,
                              uint64_t* blocks_total, uint64_t* blocks_kept);

/* Static, NUL-terminated description of a status code; for CCE_EHIP the text of
 * the last failing HIP call on this thread. */
const char* cce_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CCE_H_ */
