"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(explicit workspaces of the recommended size, bf16 MFMA kernels).

The fp64 oracle cannot be re-run at these sizes inside a test, so its outputs were
written once by tests/golden/make_golden.py (which calls only oracle/ and the seeded
generator): LSE and loss for every token, and complete rows of dE and dC for sampled
tokens / vocabulary entries (first, last, the row before a ragged tile edge, the most
frequent targets, a never-targeted entry, an ignored token, random ones).  A row of dE
or dC is an exact restriction of the full gradient, so these are element-by-element
comparisons of sampled outputs.  Properties that hold at any size cover the rest.

Tolerances as in test_parity_gpu.py: loss / LSE max relative error <= 1e-3, sampled
gradient rows relative Frobenius error <= 1e-2.  The block-filtered backward is compared
with the unfiltered oracle and with the oracle's element-wise filter: it drops a subset of
what the element-wise filter drops, so its error may not exceed that one's by more than
the dense kernel's own rounding error.
"""
import os

import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from workloads import make

from gpu_util import f64, max_rel, rel_fro, run_backward, run_forward, to_device

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FULL = ["small_vocab", "gemma2_2b", "llama3_8b", "stress", "stress_peaked"]
TOL_LOSS = 1e-3
TOL_GRAD = 1e-2


def rows_of(t, rows):
    return f64(t[torch.from_numpy(np.asarray(rows)).to(t.device)])


@pytest.mark.parametrize("name", FULL)
def test_full_size_matches_stored_oracle(cce, name):
    path = os.path.join(GOLDEN, name + ".npz")
    assert os.path.exists(path), "stored oracle values missing: run tests/golden/make_golden.py " + name
    g = np.load(path)
    print("generating %s" % name, flush=True)
    w = make(name)
    assert (w.N, w.D, w.V) == (int(g["N"]), int(g["D"]), int(g["V"]))
    # the generator reproduced the exact inputs the oracle saw
    assert int(np.uint64(w.E.astype(np.uint64).sum())) == int(g["e_sum"])
    assert int(np.uint64(w.C.astype(np.uint64).sum())) == int(g["c_sum"])
    assert int(w.targets.sum()) == int(g["t_sum"])

    E, C, t = to_device(w)
    print("forward %s N=%d D=%d V=%d" % (name, w.N, w.D, w.V), flush=True)
    loss, lse = run_forward(w, E, C, t)
    e_lse = max_rel(f64(lse), g["lse"].astype(np.float64))
    e_loss = max_rel(f64(loss), g["loss"].astype(np.float64))
    print("  lse err %.2e  loss err %.2e" % (e_lse, e_loss), flush=True)
    assert e_lse <= TOL_LOSS and e_loss <= TOL_LOSS
    ign = w.targets == w.ignore_index
    assert np.all(f64(loss)[ign] == 0.0)

    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    er, vr = g["dE_rows"], g["dC_rows"]
    ref_dE, ref_dC = g["dE"].astype(np.float64), g["dC"].astype(np.float64)

    print("backward (unfiltered) %s" % name, flush=True)
    dE, dC, stats = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    eE, eC = rel_fro(rows_of(dE, er), ref_dE), rel_fro(rows_of(dC, vr), ref_dC)
    print("  dE rows err %.2e  dC rows err %.2e" % (eE, eC), flush=True)
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    assert stats[0] == stats[1] > 0
    # properties at full size
    if ign.any():
        assert torch.all(dE[torch.from_numpy(np.nonzero(ign)[0]).cuda()] == 0)
    assert torch.isfinite(dE.float()).all() and torch.isfinite(dC.float()).all()
    if w.softcap == 0:
        # without a cap the rows of G sum to zero, hence sum_j dC_j = sum_i lam_i (sum_j G_ij) E_i = 0
        col = dC.double().sum(0)
        scale = dC.double().abs().sum(0)
        assert float((col.abs() / scale.clamp_min(1e-30)).max()) <= 4e-3   # bf16 output rounding is 2^-9 relative

    print("backward (filtered, eps 2^-12) %s" % name, flush=True)
    dEf, dCf, stats_f = run_backward(w, E, C, t, lse, dloss)
    fE, fC = rel_fro(rows_of(dEf, er), ref_dE), rel_fro(rows_of(dCf, vr), ref_dC)
    elemE = rel_fro(g["dE_f"].astype(np.float64), ref_dE)
    elemC = rel_fro(g["dC_f"].astype(np.float64), ref_dC)
    print("  filtered: dE rows err %.2e (element-wise filter %.2e)  dC rows err %.2e (%.2e)  blocks kept %d / %d"
          % (fE, elemE, fC, elemC, stats_f[1], stats_f[0]), flush=True)
    assert fE <= elemE + eE + 1e-3 and fC <= elemC + eC + 1e-3
    assert 0 < stats_f[1] <= stats_f[0]

    print("backward (filtered, wide slabs) %s" % name, flush=True)
    dEw, dCw, stats_w = run_backward(w, E, C, t, lse, dloss, op=L.CCE_OP_BACKWARD_WIDE)
    wE, wC = rel_fro(rows_of(dEw, er), ref_dE), rel_fro(rows_of(dCw, vr), ref_dC)
    print("  wide:     dE rows err %.2e  dC rows err %.2e" % (wE, wC), flush=True)
    assert wE <= elemE + eE + 1e-3 and wC <= elemC + eC + 1e-3
    assert stats_w == stats_f and torch.equal(dCw, dCf)
    del dEw, dCw

    print("backward (filtered, vocabulary sorted) %s" % name, flush=True)
    flags = L.CCE_FILTER_DE | L.CCE_FILTER_DC | L.CCE_VOCAB_SORT
    dEs, dCs, stats_s = run_backward(w, E, C, t, lse, dloss, flags=flags)
    sE, sC = rel_fro(rows_of(dEs, er), ref_dE), rel_fro(rows_of(dCs, vr), ref_dC)
    print("  sorted:   dE rows err %.2e  dC rows err %.2e  blocks kept %d / %d" % (sE, sC, stats_s[1], stats_s[0]),
          flush=True)
    assert sE <= elemE + eE + 1e-3 and sC <= elemC + eC + 1e-3
    assert stats_s[0] == stats_f[0] and 0 < stats_s[1] <= stats_s[0]

    print("backward (filtered, tiles skipped from the forward's block maxima) %s" % name, flush=True)
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    bm = torch.empty(L.cce_block_max_bytes(w.N, w.V), dtype=torch.uint8, device="cuda")
    loss2, lse2 = run_forward(w, E, C, t, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(lse2, lse) and torch.equal(loss2, loss)
    dEk, dCk, stats_k = run_backward(w, E, C, t, lse, dloss, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(dEk, dEf) and torch.equal(dCk, dCf) and stats_k == stats_f

    if ign.any():
        print("ignored tokens removed (Appendix B) %s" % name, flush=True)
        cf = both | L.CCE_COMPACT_IGNORED
        loss3, lse3 = run_forward(w, E, C, t, flags=cf)
        assert torch.equal(loss3, loss)
        dEc, dCc, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, flags=cf)
        assert torch.equal(dEc, dE)
        cC = rel_fro(rows_of(dCc, vr), ref_dC)
        print("  compacted: dC rows err %.2e" % cC, flush=True)
        assert cC <= TOL_GRAD
