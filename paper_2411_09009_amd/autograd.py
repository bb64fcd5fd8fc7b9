"""torch.autograd front end of the library: ``linear_cross_entropy(e, c, targets, ...)``.

The interface of the paper's Section 4: embeddings E, classifier C and targets x in, the
cross-entropy loss out, gradients of E and C by back-propagation.  Everything the method
computes runs inside libcce.so (cce_forward_ex / cce_backward_ex); this module only keeps
what the backward call needs (E, C, x, LSE), owns the workspaces, and applies the caller's
reduction to the per-token loss the library returns.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import torch

from . import binding as B

_workspaces: Dict[Tuple[int, int, str], torch.Tensor] = {}


def _workspace(device: torch.device, kind: str, nbytes: int) -> torch.Tensor:
    """One buffer per (device, stream, use), grown on demand.  Work on one stream is ordered, so
    consecutive calls may share it; calls on different streams get buffers of their own."""
    key = (device.index if device.index is not None else torch.cuda.current_device(),
           torch.cuda.current_stream(device).cuda_stream, kind)
    buf = _workspaces.get(key)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = buf
    return buf


class _LinearCrossEntropy(torch.autograd.Function):
    @staticmethod
    def forward(ctx, e, c, targets, softcap, ignore_index, flags, filter_eps, wide):
        if e.dtype != c.dtype:
            raise TypeError("e and c must have one dtype")
        e2 = e.reshape(-1, e.shape[-1]).contiguous()
        c2 = c.contiguous()
        t2 = targets.reshape(-1).contiguous()
        N, D = e2.shape
        V = c2.shape[0]
        dtype = B.CCE_BF16 if e2.dtype == torch.bfloat16 else B.CCE_F32
        o = B.make_opts(dtype, flags=flags, filter_eps=filter_eps)
        ws = _workspace(e2.device, "fwd", B.cce_workspace_bytes(B.CCE_OP_FORWARD, N, D, V, o))
        block_max = None
        if o.flags & B.CCE_SKIP_TILES:
            # read again by the backward call: not shared between calls
            block_max = torch.empty(B.cce_block_max_bytes(N, V), dtype=torch.uint8, device=e2.device)
        o = B.make_opts(dtype, flags=flags, filter_eps=filter_eps, workspace=ws, block_max=block_max)
        loss, lse = B.cce_forward_ex(e2, c2, t2, float(softcap), int(ignore_index), o)
        ctx.save_for_backward(e2, c2, t2, lse)
        ctx.block_max = block_max
        ctx.args = (float(softcap), int(ignore_index), dtype, o.flags, o.filter_eps, bool(wide))
        ctx.e_shape = e.shape
        lse_out = lse.view(targets.shape)
        ctx.mark_non_differentiable(lse_out)
        return loss.view(targets.shape), lse_out

    @staticmethod
    def backward(ctx, grad_loss, _grad_lse):
        e2, c2, t2, lse = ctx.saved_tensors
        softcap, ignore_index, dtype, flags, eps, wide = ctx.args
        N, D = e2.shape
        V = c2.shape[0]
        o = B.make_opts(dtype, flags=flags, filter_eps=eps)
        op = B.CCE_OP_BACKWARD_WIDE if wide else B.CCE_OP_BACKWARD
        ws = _workspace(e2.device, "bwd", B.cce_workspace_bytes(op, N, D, V, o))
        o = B.make_opts(dtype, flags=flags, filter_eps=eps, workspace=ws, block_max=ctx.block_max)
        dloss = grad_loss.reshape(-1).to(torch.float32).contiguous()
        dE, dC = B.cce_backward_ex(e2, c2, t2, lse, dloss, softcap, ignore_index, o)
        return dE.view(ctx.e_shape), dC, None, None, None, None, None, None


def linear_cross_entropy(e: torch.Tensor, c: torch.Tensor, targets: torch.Tensor, softcap: float = 0.0,
                         ignore_index: int = -100, reduction: str = "mean", filter_eps: Optional[float] = None,
                         filter_dE: bool = True, filter_dC: bool = True, vocab_sort: bool = False,
                         skip_tiles: bool = False, compact_ignored: bool = False, wide_workspace: bool = False,
                         return_lse: bool = False):
    """Cross-entropy of the logits ``e @ c.T`` against ``targets`` without materialising them.

    e [..., D] and c [V, D] are bfloat16 (MFMA kernels; filtering on at 2^-12 unless filter_eps
    says otherwise) or float32 (plain kernels, no filtering); targets [...] int64 with
    ``ignore_index`` marking tokens that take no part.  reduction: "none" (per-token loss, float32),
    "sum", or "mean" over the tokens that take part.  The keyword switches map one to one onto the
    CCE_* flags of include/cce.h; filter_dE / filter_dC cleared give the paper's FullE / FullC
    variants (Section 5.3).
    """
    if reduction not in ("none", "sum", "mean"):
        raise ValueError("reduction must be 'none', 'sum' or 'mean'")
    bf16 = e.dtype == torch.bfloat16
    flags = 0
    if bf16:
        flags |= (B.CCE_FILTER_DE if filter_dE else 0) | (B.CCE_FILTER_DC if filter_dC else 0)
        flags |= B.CCE_VOCAB_SORT if vocab_sort else 0
        flags |= B.CCE_SKIP_TILES if skip_tiles else 0
        flags |= B.CCE_COMPACT_IGNORED if compact_ignored else 0
    if filter_eps is None:
        filter_eps = 2.0 ** -12 if bf16 else 0.0
    loss, lse = _LinearCrossEntropy.apply(e, c, targets, softcap, ignore_index, flags, filter_eps, wide_workspace)
    if reduction == "sum":
        loss = loss.sum()
    elif reduction == "mean":
        valid = (targets != ignore_index) & (targets >= 0) & (targets < c.shape[0])
        loss = loss.sum() / valid.sum().clamp_min(1)
    return (loss, lse) if return_lse else loss
