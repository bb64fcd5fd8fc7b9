"""ctypes binding of libcce.so: same names as include/cce.h, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libcce.so")

CCE_BF16, CCE_F32 = 0, 1
CCE_FILTER_DE, CCE_FILTER_DC, CCE_VOCAB_SORT, CCE_PLAIN_KERNELS, CCE_SKIP_TILES, CCE_COMPACT_IGNORED, CCE_SINGLE_STREAM = 1, 2, 4, 8, 16, 32, 64
CCE_ACCUM_BF16, CCE_ACCUM_KAHAN = 128, 256
CCE_OP_FORWARD, CCE_OP_BACKWARD, CCE_OP_BACKWARD_MIN, CCE_OP_BACKWARD_WIDE = 0, 1, 2, 3


class CceOpts(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int),
        ("flags", ctypes.c_uint32),
        ("filter_eps", ctypes.c_float),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("block_max", ctypes.c_void_p),
        ("block_max_bytes", ctypes.c_size_t),
    ]


class CceError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("cce status %d: %s" % (status, text))
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load libcce.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2411_09009_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    po = ctypes.POINTER(CceOpts)
    lib.cce_default_opts.argtypes = [ctypes.c_int, po]
    lib.cce_default_opts.restype = None
    lib.cce_strerror.argtypes = [ctypes.c_int]
    lib.cce_strerror.restype = ctypes.c_char_p
    lib.cce_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64, po]
    lib.cce_workspace_bytes.restype = sz
    lib.cce_block_max_bytes.argtypes = [i64, i64]
    lib.cce_block_max_bytes.restype = sz
    lib.cce_filter_block.argtypes = [i64, i64, i64, po, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.cce_filter_block.restype = None
    fwd = [vp, vp, vp, i64, i64, i64, f32, i64, vp, vp]
    bwd = [vp, vp, vp, i64, i64, i64, f32, i64, vp, vp, vp, vp]
    lib.cce_forward.argtypes = fwd
    lib.cce_forward_ex.argtypes = fwd + [po]
    lib.cce_forward_noalloc.argtypes = fwd + [po]
    lib.cce_forward_noalloc.restype = ctypes.c_int
    lib.cce_noalloc_scratch_bytes.argtypes = []
    lib.cce_noalloc_scratch_bytes.restype = sz
    lib.cce_backward.argtypes = bwd
    lib.cce_backward_ex.argtypes = bwd + [po]
    for f in (lib.cce_forward, lib.cce_forward_ex, lib.cce_backward, lib.cce_backward_ex):
        f.restype = ctypes.c_int
    lib.cce_backward_filter_stats.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
    lib.cce_backward_filter_stats.restype = ctypes.c_int
    lib.cce_forward_target_stats.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.cce_forward_target_stats.restype = ctypes.c_int
    lib.cce_set_workspace.argtypes = [vp, sz]
    lib.cce_set_workspace.restype = ctypes.c_int
    _lib = lib
    return lib


def cce_strerror(status: int) -> str:
    return load().cce_strerror(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise CceError(status, cce_strerror(status))


def cce_default_opts(dtype: int) -> CceOpts:
    o = CceOpts()
    load().cce_default_opts(int(dtype), ctypes.byref(o))
    return o


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return CCE_BF16
    if t.dtype == torch.float32:
        return CCE_F32
    raise TypeError("E / C must be bfloat16 or float32, got %s" % t.dtype)


def make_opts(dtype: int, flags: Optional[int] = None, filter_eps: Optional[float] = None,
              workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None,
              block_max: Optional[torch.Tensor] = None) -> CceOpts:
    """Defaults of the plain entry points, overridden by the arguments given."""
    o = cce_default_opts(dtype)
    if flags is not None:
        o.flags = int(flags)
    if filter_eps is not None:
        o.filter_eps = float(filter_eps)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    if block_max is not None:
        o.block_max = block_max.data_ptr()
        o.block_max_bytes = block_max.numel() * block_max.element_size()
    o.stream = torch.cuda.current_stream().cuda_stream if stream is None else int(stream)
    return o


_lent = {}   # device index -> the tensor lent to the plain entry points (kept alive here)


def cce_set_workspace(workspace: Optional[torch.Tensor]) -> None:
    """Lends `workspace` (a device tensor; None withdraws it) to cce_forward / cce_backward on its device."""
    if workspace is None:
        _check(load().cce_set_workspace(None, 0))
        _lent.pop(torch.cuda.current_device(), None)
        return
    with torch.cuda.device(workspace.device):
        _check(load().cce_set_workspace(workspace.data_ptr(), workspace.numel() * workspace.element_size()))
        _lent[workspace.device.index] = workspace


def cce_workspace_bytes(op: int, N: int, D: int, V: int, opts: CceOpts) -> int:
    return int(load().cce_workspace_bytes(int(op), int(N), int(D), int(V), ctypes.byref(opts)))


def cce_block_max_bytes(N: int, V: int) -> int:
    return int(load().cce_block_max_bytes(int(N), int(V)))


def cce_filter_block(N: int, D: int, V: int, opts: CceOpts) -> Tuple[int, int]:
    r, c = ctypes.c_int(0), ctypes.c_int(0)
    load().cce_filter_block(int(N), int(D), int(V), ctypes.byref(opts), ctypes.byref(r), ctypes.byref(c))
    return r.value, c.value


def _shapes(E: torch.Tensor, C: torch.Tensor, targets: torch.Tensor):
    if not (E.is_cuda and C.is_cuda and targets.is_cuda):
        raise ValueError("E, C and targets must be device tensors")
    if not (E.is_contiguous() and C.is_contiguous() and targets.is_contiguous()):
        raise ValueError("E, C and targets must be contiguous")
    if E.dim() != 2 or C.dim() != 2 or E.shape[1] != C.shape[1] or targets.shape != (E.shape[0],):
        raise ValueError("expected E [N, D], C [V, D], targets [N]")
    if targets.dtype != torch.int64 or E.dtype != C.dtype:
        raise TypeError("targets must be int64 and E, C of one dtype")
    return E.shape[0], E.shape[1], C.shape[0]


def cce_forward(E, C, targets, softcap: float = 0.0, ignore_index: int = -100, out_loss=None, out_lse=None):
    """Plain entry point: bf16, null stream, scratch from the buffer lent with cce_set_workspace."""
    N, D, V = _shapes(E, C, targets)
    if E.dtype != torch.bfloat16:
        raise TypeError("cce_forward takes bfloat16; use cce_forward_ex for float32")
    out_loss = torch.empty(N, dtype=torch.float32, device=E.device) if out_loss is None else out_loss
    out_lse = torch.empty(N, dtype=torch.float32, device=E.device) if out_lse is None else out_lse
    _check(load().cce_forward(E.data_ptr(), C.data_ptr(), targets.data_ptr(), N, D, V, float(softcap),
                              int(ignore_index), out_loss.data_ptr(), out_lse.data_ptr()))
    return out_loss, out_lse


def cce_forward_ex(E, C, targets, softcap: float, ignore_index: int, opts: CceOpts, out_loss=None, out_lse=None):
    N, D, V = _shapes(E, C, targets)
    out_loss = torch.empty(N, dtype=torch.float32, device=E.device) if out_loss is None else out_loss
    out_lse = torch.empty(N, dtype=torch.float32, device=E.device) if out_lse is None else out_lse
    _check(load().cce_forward_ex(E.data_ptr(), C.data_ptr(), targets.data_ptr(), N, D, V, float(softcap),
                                 int(ignore_index), out_loss.data_ptr(), out_lse.data_ptr(), ctypes.byref(opts)))
    return out_loss, out_lse


def cce_forward_noalloc(E, C, targets, softcap: float, ignore_index: int, opts: CceOpts, out_loss, out_lse):
    """Forward on the library's static scratch.  The outputs are required arguments: this wrapper
    allocates nothing either."""
    N, D, V = _shapes(E, C, targets)
    _check(load().cce_forward_noalloc(E.data_ptr(), C.data_ptr(), targets.data_ptr(), N, D, V, float(softcap),
                                      int(ignore_index), out_loss.data_ptr(), out_lse.data_ptr(), ctypes.byref(opts)))
    return out_loss, out_lse


def cce_noalloc_scratch_bytes() -> int:
    return int(load().cce_noalloc_scratch_bytes())


def _bwd_args(E, C, targets, lse, dloss, out_dE, out_dC):
    N, D, V = _shapes(E, C, targets)
    for name, t in (("lse", lse), ("dLoss", dloss)):
        if t.dtype != torch.float32 or t.shape != (N,) or not t.is_cuda or not t.is_contiguous():
            raise ValueError("%s must be a contiguous float32 device tensor of shape [N]" % name)
    out_dE = torch.empty_like(E) if out_dE is None else out_dE
    out_dC = torch.empty_like(C) if out_dC is None else out_dC
    return N, D, V, out_dE, out_dC


def cce_backward(E, C, targets, lse, dloss, softcap: float = 0.0, ignore_index: int = -100, out_dE=None, out_dC=None):
    """Plain entry point: bf16, null stream, filtering on at 2^-12, scratch from the lent buffer."""
    N, D, V, out_dE, out_dC = _bwd_args(E, C, targets, lse, dloss, out_dE, out_dC)
    if E.dtype != torch.bfloat16:
        raise TypeError("cce_backward takes bfloat16; use cce_backward_ex for float32")
    _check(load().cce_backward(E.data_ptr(), C.data_ptr(), targets.data_ptr(), N, D, V, float(softcap),
                               int(ignore_index), lse.data_ptr(), dloss.data_ptr(), out_dE.data_ptr(),
                               out_dC.data_ptr()))
    return out_dE, out_dC


def cce_backward_ex(E, C, targets, lse, dloss, softcap: float, ignore_index: int, opts: CceOpts,
                    out_dE=None, out_dC=None):
    N, D, V, out_dE, out_dC = _bwd_args(E, C, targets, lse, dloss, out_dE, out_dC)
    _check(load().cce_backward_ex(E.data_ptr(), C.data_ptr(), targets.data_ptr(), N, D, V, float(softcap),
                                  int(ignore_index), lse.data_ptr(), dloss.data_ptr(), out_dE.data_ptr(),
                                  out_dC.data_ptr(), ctypes.byref(opts)))
    return out_dE, out_dC


def cce_backward_filter_stats(workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None) -> Tuple[int, int]:
    total, kept = ctypes.c_uint64(0), ctypes.c_uint64(0)
    ws = None if workspace is None else workspace.data_ptr()
    st = torch.cuda.current_stream().cuda_stream if stream is None else int(stream)
    _check(load().cce_backward_filter_stats(ws, st, ctypes.byref(total), ctypes.byref(kept)))
    return total.value, kept.value


def cce_forward_target_stats(workspace: Optional[torch.Tensor] = None, stream: Optional[int] = None) -> int:
    n = ctypes.c_uint64(0)
    ws = None if workspace is None else workspace.data_ptr()
    st = torch.cuda.current_stream().cuda_stream if stream is None else int(stream)
    _check(load().cce_forward_target_stats(ws, st, ctypes.byref(n)))
    return n.value
