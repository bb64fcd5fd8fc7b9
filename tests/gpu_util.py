"""Helpers shared by the GPU parity tests: move a seeded workload to the device and
compare against the fp64 oracle."""
import numpy as np
import torch

import paper_2411_09009_amd as L


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
    o = L.make_opts(dtype_code(w), flags=flags)
    ws = workspace(L.cce_workspace_bytes(L.CCE_OP_FORWARD, w.N, w.D, w.V, o))
    o = L.make_opts(dtype_code(w), flags=flags, workspace=ws, block_max=block_max)
    loss, lse = L.cce_forward_ex(E, C, t, cap, w.ignore_index, o)
    torch.cuda.synchronize()
    return loss, lse


def run_backward(w, E, C, t, lse, dloss, flags=None, eps=None, ws_bytes=None, softcap=None, op=None, block_max=None):
    cap = w.softcap if softcap is None else softcap
    o = L.make_opts(dtype_code(w), flags=flags, filter_eps=eps)
    if ws_bytes is None:
        ws_bytes = L.cce_workspace_bytes(L.CCE_OP_BACKWARD if op is None else op, w.N, w.D, w.V, o)
    ws = workspace(ws_bytes)
    o = L.make_opts(dtype_code(w), flags=flags, filter_eps=eps, workspace=ws, block_max=block_max)
    dE, dC = L.cce_backward_ex(E, C, t, lse, dloss, cap, w.ignore_index, o)
    torch.cuda.synchronize()
    stats = L.cce_backward_filter_stats(ws)
    return dE, dC, stats


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def max_rel(got, ref, floor=1.0):
    """max |got - ref| / max(|ref|, floor): relative error with a floor for values near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
