"""Helpers shared by the GPU parity tests: move a seeded workload to the device, call the
library through its binding with guarded buffers, and compare against the fp64 oracle.

Every workspace, block-maximum record and output handed to the library here sits between two
guard regions filled with a sentinel byte; the guards are verified after each call, so a kernel
that writes outside a buffer it was given fails the test that ran it (host-side check only:
the kernels themselves always run to completion)."""
import numpy as np
import torch

import paper_2411_09009_amd as L

GUARD_BYTES = 4096          # a multiple of the 256-byte alignment the library asks for
SENTINEL = 0xA5


class Guarded:
    """A device buffer of `nbytes` with a sentinel-filled guard region on either side."""

    def __init__(self, nbytes, fill=None):
        nbytes = max(int(nbytes), 256)
        self.raw = torch.full((nbytes + 2 * GUARD_BYTES,), SENTINEL, dtype=torch.uint8, device="cuda:0")
        assert self.raw.data_ptr() % 256 == 0
        self.buf = self.raw[GUARD_BYTES:GUARD_BYTES + nbytes]
        if fill is not None:
            self.buf.fill_(fill)

    def view(self, dtype, shape):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        return self.buf[:n].view(dtype).view(*shape)

    def check(self, what=""):
        lo, hi = self.raw[:GUARD_BYTES], self.raw[GUARD_BYTES + self.buf.numel():]
        ok = bool((lo == SENTINEL).all()) and bool((hi == SENTINEL).all())
        assert ok, "guard region around %s was overwritten" % what


def to_device(w):
    dev = torch.device("cuda:0")
    if w.dtype == "bf16":
        E = torch.from_numpy(w.E.view(np.int16)).to(dev).view(torch.bfloat16)
        C = torch.from_numpy(w.C.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        E = torch.from_numpy(w.E).to(dev)
        C = torch.from_numpy(w.C).to(dev)
    t = torch.from_numpy(w.targets).to(dev)
    return E, C, t


def dtype_code(w):
    return L.CCE_BF16 if w.dtype == "bf16" else L.CCE_F32


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0")


def run_forward(w, E, C, t, flags=None, softcap=None, block_max=None):
    cap = w.softcap if softcap is None else softcap
    N, D, V = E.shape[0], E.shape[1], C.shape[0]
    o = L.make_opts(dtype_code(w), flags=flags)
    ws = Guarded(L.cce_workspace_bytes(L.CCE_OP_FORWARD, N, D, V, o))
    g_loss, g_lse = Guarded(N * 4), Guarded(N * 4)
    loss, lse = g_loss.view(torch.float32, (N,)), g_lse.view(torch.float32, (N,))
    o = L.make_opts(dtype_code(w), flags=flags, workspace=ws.buf, block_max=block_max)
    L.cce_forward_ex(E, C, t, cap, w.ignore_index, o, out_loss=loss, out_lse=lse)
    torch.cuda.synchronize()
    for g, what in ((ws, "the forward workspace"), (g_loss, "out_loss"), (g_lse, "out_lse")):
        g.check(what)
    return loss.clone(), lse.clone()


def run_backward(w, E, C, t, lse, dloss, flags=None, eps=None, ws_bytes=None, softcap=None, op=None, block_max=None):
    cap = w.softcap if softcap is None else softcap
    N, D, V = E.shape[0], E.shape[1], C.shape[0]
    o = L.make_opts(dtype_code(w), flags=flags, filter_eps=eps)
    if ws_bytes is None:
        ws_bytes = L.cce_workspace_bytes(L.CCE_OP_BACKWARD if op is None else op, N, D, V, o)
    ws = Guarded(ws_bytes)
    esz = E.element_size()
    g_dE, g_dC = Guarded(N * D * esz), Guarded(V * D * esz)
    dE, dC = g_dE.view(E.dtype, (N, D)), g_dC.view(C.dtype, (V, D))
    o = L.make_opts(dtype_code(w), flags=flags, filter_eps=eps, workspace=ws.buf, block_max=block_max)
    L.cce_backward_ex(E, C, t, lse, dloss, cap, w.ignore_index, o, out_dE=dE, out_dC=dC)
    torch.cuda.synchronize()
    stats = L.cce_backward_filter_stats(ws.buf)
    for g, what in ((ws, "the backward workspace"), (g_dE, "out_dE"), (g_dC, "out_dC")):
        g.check(what)
    return dE, dC, stats


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def max_row_err(got, ref):
    """Largest per-row error  max_r ||got_r - ref_r|| / max(||ref_r||, median_r ||ref_r||).

    A whole-matrix Frobenius norm is carried by the few rows with large gradients (the rows of dC that
    are somebody's target); this one gives every row its own say, with the median row norm as the floor
    for rows that are (nearly) zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rn = np.linalg.norm(ref, axis=1)
    floor = float(np.median(rn))
    if floor == 0.0:
        floor = float(rn.max()) if rn.max() > 0 else 1.0
    return float(np.max(np.linalg.norm(got - ref, axis=1) / np.maximum(rn, floor)))


def max_rel(got, ref, floor=1.0):
    """max |got - ref| / max(|ref|, floor): relative error with a floor for values near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
