"""MI355X-native fused linear cross-entropy (Cut Cross-Entropy hot path).

The product is the C-ABI shared library built from csrc/ (declared in
include/cce.h).  This package is its thin ctypes binding: it marshals torch
device tensors into the C calls and nothing else.  There is no CPU or eager
fallback: if the library has not been built, load() raises.
"""
from .binding import (  # noqa: F401
    CCE_BF16, CCE_F32,
    CCE_FILTER_DE, CCE_FILTER_DC, CCE_VOCAB_SORT, CCE_PLAIN_KERNELS, CCE_SKIP_TILES, CCE_COMPACT_IGNORED, CCE_SINGLE_STREAM,
    CCE_ACCUM_BF16, CCE_ACCUM_KAHAN,
    CCE_OP_FORWARD, CCE_OP_BACKWARD, CCE_OP_BACKWARD_MIN, CCE_OP_BACKWARD_WIDE,
    CceError, CceOpts, LIB_PATH,
    load, cce_default_opts, cce_workspace_bytes, cce_block_max_bytes, cce_filter_block, cce_strerror,
    cce_forward, cce_forward_ex, cce_forward_noalloc, cce_noalloc_scratch_bytes, cce_backward, cce_backward_ex, cce_backward_filter_stats, cce_forward_target_stats,
    make_opts, cce_set_workspace,
)
