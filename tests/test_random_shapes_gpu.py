"""Seeded sweep over shapes, options and workspace sizes: every case runs forward and backward
through the C ABI and is compared with the fp64 oracle like the hand-picked cases of
test_parity_gpu.py.  The point is the combinations nobody thought of: sizes on and around the
tile edges (1, 63..65, 255..257, ...), both kernel families (bf16 MFMA; plain kernels for bf16
with D not a multiple of 64 and for float32), every subset of the option flags, the three workspace
sizes, soft-cap off / below / above the fixed-maximum limit, nearly everything ignored.

Tolerances (bf16; float32: 1e-5 and 1e-4): loss / LSE 1e-3, gradients 1e-2 relative Frobenius
against the exact gradient, plus
the element-wise filter's own error when a filter is on (the block filter drops a subset of
what the element-wise one drops)."""
import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from oracle import cce_oracle as O
from workloads import make

from gpu_util import f64, max_rel, max_row_err, rel_fro, run_backward, run_forward, to_device

pytestmark = pytest.mark.gpu

NAMES = ["gemma2_2b", "small_vocab", "llama3_8b", "stress_peaked", "tiny"]      # tiny: float32 inputs
CASES = 96


def draw(k):
    rng = np.random.default_rng(1000 + k)
    D = int(rng.choice([64, 128, 192, 256, 320, 512, 40, 72]))       # 40, 72: bf16 on the plain kernels
    N = int(rng.choice([1, 7, 64, 255, 256, 257, 300, 511, 513, 700, 1025, 1500, 2300, 4200]))
    V = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 1537, 4096, 6145, 7000, 12289, 20000, 30011]))
    while N * D * V > 4e9:          # keeps the oracle at about a second per case
        if V > 1000:
            V //= 2
        else:
            N //= 2
    name = NAMES[int(rng.integers(len(NAMES)))]
    cap = float(rng.choice([-1.0, 0.0, 5.0, 30.0, 50.0]))     # -1: the configuration's own
    ign = float(rng.choice([0.0, 0.02, 0.5, 0.97]))
    flags = 0
    for bit, p in ((L.CCE_FILTER_DE, 0.8), (L.CCE_FILTER_DC, 0.8), (L.CCE_VOCAB_SORT, 0.3), (L.CCE_SKIP_TILES, 0.4),
                   (L.CCE_COMPACT_IGNORED, 0.4), (L.CCE_SINGLE_STREAM, 0.2), (L.CCE_ACCUM_KAHAN, 0.15)):
        if rng.random() < p:
            flags |= bit
    op = int(rng.choice([L.CCE_OP_BACKWARD, L.CCE_OP_BACKWARD_MIN, L.CCE_OP_BACKWARD_WIDE]))
    eps = float(rng.choice([0.0, 2.0 ** -12]))
    if name == "tiny" or D % 64:
        flags &= ~(L.CCE_VOCAB_SORT | L.CCE_ACCUM_KAHAN)   # the sorted walk and the bf16 sums exist on the MFMA path only
    if name == "tiny":
        eps = 0.0                           # the filter threshold is a bf16 notion (Section 4.3)
    return name, N, D, V, cap, ign, flags, op, eps


@pytest.mark.parametrize("k", range(CASES))
def test_random_case_matches_oracle(cce, k):
    name, N, D, V, cap, ign, flags, op, eps = draw(k)
    print("case %d: %s N=%d D=%d V=%d cap=%g ignored=%g flags=%d op=%d eps=%g" % (k, name, N, D, V, cap, ign, flags, op, eps),
          flush=True)
    w = make(name, N=N, D=D, V=V, ignore_frac=ign, seed=k, **({} if cap < 0 else {"softcap": cap}))
    E, C, t = to_device(w)
    bm = None
    if flags & L.CCE_SKIP_TILES:
        bm = torch.empty(max(L.cce_block_max_bytes(N, V), 256), dtype=torch.uint8, device="cuda")
    loss, lse = run_forward(w, E, C, t, flags=flags, block_max=bm)
    E64, C64 = w.E64(), w.C64()
    r_loss, r_lse = O.forward(E64, C64, w.targets, w.softcap, w.ignore_index)
    valid = w.targets != w.ignore_index
    tol_loss = 1e-3 if w.dtype == "bf16" else 1e-5
    if flags & L.CCE_COMPACT_IGNORED:     # LSE of removed tokens is unspecified
        assert not valid.any() or max_rel(f64(lse)[valid], r_lse[valid]) <= tol_loss
        lse = torch.where(torch.from_numpy(valid).cuda(), lse, torch.zeros_like(lse))
    else:
        assert max_rel(f64(lse), r_lse) <= tol_loss
    assert max_rel(f64(loss), r_loss) <= tol_loss

    lam = (np.random.default_rng(k).standard_normal(N) / N).astype(np.float32)
    dE, dC, _ = run_backward(w, E, C, t, lse, torch.from_numpy(lam).cuda(), flags=flags, eps=eps, op=op, block_max=bm)
    lam64 = lam.astype(np.float64)
    rdE, rdC = O.backward(E64, C64, w.targets, r_lse, lam64, w.softcap, w.ignore_index)
    tolE = tolC = 1e-2 if w.dtype == "bf16" else 1e-4
    if eps > 0 and flags & (L.CCE_FILTER_DE | L.CCE_FILTER_DC):
        fdE, fdC = O.backward(E64, C64, w.targets, r_lse, lam64, w.softcap, w.ignore_index, eps=eps, filter_mode="element")
        tolE += rel_fro(fdE, rdE)
        tolC += rel_fro(fdC, rdC)
    assert torch.isfinite(dE.float()).all() and torch.isfinite(dC.float()).all()
    assert rel_fro(f64(dE), rdE) <= tolE and rel_fro(f64(dC), rdC) <= tolC
    if not (eps > 0 and flags & (L.CCE_FILTER_DE | L.CCE_FILTER_DC)):
        # exact path: every row on its own, relative to max(its norm, the median row norm)
        tol_row = 1e-2 if w.dtype == "bf16" else 1e-4
        assert max_row_err(f64(dE), rdE) <= tol_row and max_row_err(f64(dC), rdC) <= tol_row
