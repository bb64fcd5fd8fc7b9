"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(explicit workspaces of the recommended size, bf16 MFMA kernels).

What the fp64 oracle supplies at these sizes:
  * stored (tests/golden/<config>.npz, written by tests/golden/make_golden.py, which calls only
    oracle/ and the seeded generator): LSE and loss of EVERY token; 16 complete rows of dE and dC with
    and without the element-wise filter; and, for >= 1024 sampled tokens and >= 1024 sampled vocabulary
    entries, 16 entries of each row of dE / dC together with the norm of the complete row;
  * computed here, on the host, by the oracle itself from those stored LSEs: complete rows of dE
    for >= 1024 sampled tokens and complete rows of dC for >= 1024 sampled vocabulary entries.  A
    row of dE needs only its own token and all of C; a row of dC needs only its own logit column
    once the LSE of every token is known: both are exact restrictions of the full gradient, a few
    seconds of fp64 each (stored in full they would be 20 - 80 MB per configuration), and checked here
    against the stored entries and norms before the kernels are compared with them.
    The samples (tests/golden/sampling.py) hold both sides of every 256-token tile edge (dE) and of every multiple of 2048 in
    the vocabulary (dC): every slab edge of the recommended (6144 k) and of the wide (16384 k,
    24576 k) slab width, so that each slab of either width has at least its first and its last row
    checked; the ragged last tile's edges; the most frequent and never-used targets; ignored tokens;
    the boosted rows of the peaked variant; random ones.
  * for the largest configuration, a complete oracle backward on a sub-batch (first N' tokens, full D
    and |V|, ragged last token tile), where every one of the |V| rows of dC is compared.
Properties that hold at any size cover the rest (shift invariance, sum_j dC_j = 0, zero rows).

Tolerances as in test_parity_gpu.py: loss / LSE max relative error <= 1e-3; gradient rows relative
Frobenius error <= 1e-2 and, row by row, ||delta row|| <= 1e-2 max(||row||, median row norm).  The
block-filtered backward is compared with the unfiltered oracle and with the oracle's element-wise
filter: it drops a subset of what the element-wise filter drops, so its error may not exceed that
one's by more than the dense kernel's own rounding error.  On these synthetic inputs the softmax of
the Gemma-shaped configuration is so flat that every entry is below 2^-12: the filter (the paper's,
at the paper's threshold) then removes the whole softmax term and the filtered dE is 1.9e-2 from the
exact gradient (the oracle's element-wise filter: 2.0e-2).  That is outside the 1e-2 asked of the
exact path; it is asserted below as what it is.
"""
import os
import time

import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from oracle import cce_oracle as O
from workloads import make

from gpu_util import f64, max_rel, max_row_err, rel_fro, run_backward, run_forward, to_device
from golden.sampling import sample_columns, sample_tokens, sample_vocab

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
FULL = ["small_vocab", "gemma2_2b", "llama3_8b", "stress", "stress_peaked"]
# Table A3 shapes beyond the five configurations, and a small batch at the Gemma shape (the split-K regime)
MORE_SHAPES = ["gemma2_9b", "qwen25_7b", "gemma2_2b_n1024"]
TOL_LOSS = 1e-3
TOL_GRAD = 1e-2
TOL_ROW = 1e-2
# distance of the default-filtered dE rows from the EXACT gradient (see the module docstring)
FILTERED_DE_BOUND = {"gemma2_2b": 2.5e-2, "gemma2_9b": 2.5e-2, "gemma2_2b_n1024": 2.5e-2}


def rows_of(t, rows):
    return f64(t[torch.from_numpy(np.asarray(rows)).to(t.device)])


def load_golden(name, w):
    path = os.path.join(GOLDEN, name + ".npz")
    assert os.path.exists(path), "stored oracle values missing: run tests/golden/make_golden.py " + name
    g = np.load(path)
    assert (w.N, w.D, w.V) == (int(g["N"]), int(g["D"]), int(g["V"]))
    # the generator reproduced the exact inputs the oracle saw
    assert int(np.uint64(w.E.astype(np.uint64).sum())) == int(g["e_sum"])
    assert int(np.uint64(w.C.astype(np.uint64).sum())) == int(g["c_sum"])
    assert int(w.targets.sum()) == int(g["t_sum"])
    return g


def check_sampled_rows(name, w, g, dE, dC, what):
    """>= 1024 rows of dE and of dC: first the kernels against the stored oracle entries (16 columns of every
    sampled row), then against complete rows the oracle computes now from the stored LSEs, which are themselves
    checked against the stored entries and row norms."""
    t0 = time.time()
    tok, voc, cols = sample_tokens(w), sample_vocab(w), sample_columns(w)
    assert np.array_equal(tok, g["tok_rows"]) and np.array_equal(voc, g["voc_rows"]) and np.array_equal(cols, g["cols"])
    got_dE, got_dC = rows_of(dE, tok), rows_of(dC, voc)
    sE, sC = g["dE_sub"].astype(np.float64), g["dC_sub"].astype(np.float64)
    eE_s, eC_s = rel_fro(got_dE[:, cols], sE), rel_fro(got_dC[:, cols], sC)
    assert eE_s <= TOL_GRAD and eC_s <= TOL_GRAD
    # every sampled row on its own, scaled by the stored norm of the complete row (16 of D entries are seen)
    scale = np.sqrt(len(cols) / w.D)
    for got, sub, norm in ((got_dE, sE, g["dE_norm"]), (got_dC, sC, g["dC_norm"])):
        floor = float(np.median(norm)) or 1.0
        worst = np.max(np.linalg.norm(got[:, cols] - sub, axis=1) / (np.maximum(norm, floor) * scale))
        assert worst <= 3 * TOL_ROW, worst                  # 16 entries stand for a row: looser than the complete rows below
    lse = g["lse"].astype(np.float64)
    lam = w.mean_dloss().astype(np.float64)
    C64 = w.C64()
    ref_dE = O.backward_dE_rows(w.E64(tok), C64, w.targets[tok], lse[tok], lam[tok], np.arange(len(tok)),
                                w.softcap, w.ignore_index)
    ref_dC = O.backward_dC_rows(w.E64(), C64, w.targets, lse, lam, voc, w.softcap, w.ignore_index)
    del C64
    # the rows computed here are the ones the committed script stored entries and norms of
    assert np.allclose(ref_dE[:, cols], sE, rtol=1e-5, atol=1e-12) and np.allclose(ref_dC[:, cols], sC, rtol=1e-5, atol=1e-12)
    assert np.allclose(np.linalg.norm(ref_dE, axis=1), g["dE_norm"], rtol=1e-9, atol=1e-15)
    assert np.allclose(np.linalg.norm(ref_dC, axis=1), g["dC_norm"], rtol=1e-9, atol=1e-15)
    eE, eC = rel_fro(got_dE, ref_dE), rel_fro(got_dC, ref_dC)
    rE, rC = max_row_err(got_dE, ref_dE), max_row_err(got_dC, ref_dC)
    print("  %s: %d dE rows err %.2e (worst row %.2e; stored entries %.2e)  %d dC rows err %.2e (worst row %.2e; stored entries %.2e)"
          "  [oracle %.0f s]" % (what, len(tok), eE, rE, eE_s, len(voc), eC, rC, eC_s, time.time() - t0), flush=True)
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    assert rE <= TOL_ROW and rC <= TOL_ROW
    return tok, voc, ref_dE, ref_dC


def check_invariants_without_cap(w, E, C, t, dloss):
    """Full-size properties of the uncapped loss (Section 3: Eq. 4 depends on logit differences only).

    Adding the same amount s_i k to every logit of token i leaves its loss unchanged and moves its LSE by
    s_i k.  The shift is made with exactly representable inputs: 64 more columns of D, all zero except one
    that holds s_i in E and k in every row of C.  And since rows of G sum to zero, sum_j dC_j = 0."""
    N, V = E.shape[0], C.shape[0]
    loss0, lse0 = run_forward(w, E, C, t, softcap=0.0)
    s = torch.randint(-8, 9, (N,), device="cuda").to(torch.bfloat16)
    k = 4.0
    Ex = torch.zeros(N, 64, dtype=torch.bfloat16, device="cuda")
    Ex[:, 0] = s
    Cx = torch.zeros(V, 64, dtype=torch.bfloat16, device="cuda")
    Cx[:, 0] = k
    E2, C2 = torch.cat([E, Ex], dim=1).contiguous(), torch.cat([C, Cx], dim=1).contiguous()
    del Ex, Cx
    loss1, lse1 = run_forward(w, E2, C2, t, softcap=0.0)
    shift = s.float() * k
    d_lse = float(((lse1 - lse0 - shift).abs() / lse0.abs().clamp_min(1.0)).max())
    d_loss = float(((loss1 - loss0).abs() / loss0.abs().clamp_min(1.0)).max())
    print("  shift invariance: lse moved by s*k within %.2e, loss unchanged within %.2e" % (d_lse, d_loss), flush=True)
    assert d_lse <= TOL_LOSS and d_loss <= TOL_LOSS
    dE2, dC2, _ = run_backward(w, E2, C2, t, lse1, dloss, eps=0.0, softcap=0.0)
    del E2, C2
    col = dC2.double().sum(0)
    scale = dC2.double().abs().sum(0)
    worst = float((col.abs() / scale.clamp_min(1e-30)).max())
    print("  sum_j dC_j = 0 within %.2e of sum_j |dC_j|" % worst, flush=True)
    assert worst <= 4e-3                                # bf16 output rounding is 2^-9 relative per element
    # the added columns of dE: dE_i[extra] = k sum_j gz_ij = 0 up to the bf16 rounding of the target's entry of GZ
    # (about -dloss_i, relative error up to 2^-9); the 63 all-zero columns of C give exact zeros
    assert float(dE2[:, -64].float().abs().max()) <= k * float(dloss.abs().max()) * 2.0 ** -8
    assert torch.all(dE2[:, -63:] == 0)
    return loss0, lse0


@pytest.mark.parametrize("name", FULL)
def test_full_size_matches_stored_oracle(cce, name):
    print("generating %s" % name, flush=True)
    w = make(name)
    g = load_golden(name, w)

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
    print("  stored rows: dE err %.2e  dC err %.2e" % (eE, eC), flush=True)
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    assert stats[0] == stats[1] > 0
    tok, voc, live_dE, live_dC = check_sampled_rows(name, w, g, dE, dC, "recommended slabs")
    # properties at full size
    if ign.any():
        assert torch.all(dE[torch.from_numpy(np.nonzero(ign)[0]).cuda()] == 0)
    assert torch.isfinite(dE.float()).all() and torch.isfinite(dC.float()).all()
    if w.softcap == 0:
        # without a cap the rows of G sum to zero, hence sum_j dC_j = sum_i lam_i (sum_j G_ij) E_i = 0
        col = dC.double().sum(0)
        scale = dC.double().abs().sum(0)
        assert float((col.abs() / scale.clamp_min(1e-30)).max()) <= 4e-3   # bf16 output rounding is 2^-9 relative

    print("backward (unfiltered, wide slabs) %s" % name, flush=True)
    dEw0, dCw0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=L.CCE_OP_BACKWARD_WIDE)
    assert torch.equal(dCw0, dC)                        # a row of dC is final within its slab, whatever the width
    wE = rel_fro(rows_of(dEw0, tok), live_dE)
    rE = max_row_err(rows_of(dEw0, tok), live_dE)
    print("  wide slabs: %d dE rows err %.2e (worst row %.2e)" % (len(tok), wE, rE), flush=True)
    assert wE <= TOL_GRAD and rE <= TOL_ROW
    del dEw0, dCw0, live_dE, live_dC

    print("backward (filtered, eps 2^-12) %s" % name, flush=True)
    dEf, dCf, stats_f = run_backward(w, E, C, t, lse, dloss)
    fE, fC = rel_fro(rows_of(dEf, er), ref_dE), rel_fro(rows_of(dCf, vr), ref_dC)
    elemE = rel_fro(g["dE_f"].astype(np.float64), ref_dE)
    elemC = rel_fro(g["dC_f"].astype(np.float64), ref_dC)
    print("  filtered: dE rows err %.2e (element-wise filter %.2e)  dC rows err %.2e (%.2e)  blocks kept %d / %d"
          % (fE, elemE, fC, elemC, stats_f[1], stats_f[0]), flush=True)
    assert fE <= elemE + eE + 1e-3 and fC <= elemC + eC + 1e-3
    assert fE <= FILTERED_DE_BOUND.get(name, TOL_GRAD) and fC <= TOL_GRAD
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
    del dEs, dCs

    print("backward (filtered, tiles skipped from the forward's block maxima) %s" % name, flush=True)
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    bm = torch.empty(L.cce_block_max_bytes(w.N, w.V), dtype=torch.uint8, device="cuda")
    loss2, lse2 = run_forward(w, E, C, t, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(lse2, lse) and torch.equal(loss2, loss)
    dEk, dCk, stats_k = run_backward(w, E, C, t, lse, dloss, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(dEk, dEf) and torch.equal(dCk, dCf) and stats_k == stats_f
    del dEk, dCk, dEf, dCf, bm

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
        del dEc, dCc
    del dE, dC

    if name == "gemma2_2b":
        print("accumulation variants of dE's sum over the %d slabs (Section 5) %s" % ((w.V + 6143) // 6144, name), flush=True)
        both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
        for label, fl in (("bf16 running sum", L.CCE_ACCUM_BF16), ("bf16 + Kahan", L.CCE_ACCUM_KAHAN)):
            dEa, dCa, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, flags=both | fl)
            aE = rel_fro(rows_of(dEa, er), ref_dE)
            print("  %s: stored dE rows err %.2e (fp32 accumulator %.2e)" % (label, aE, eE), flush=True)
            assert aE <= (TOL_GRAD if fl == L.CCE_ACCUM_KAHAN else 3 * TOL_GRAD)
            if fl == L.CCE_ACCUM_KAHAN:
                assert aE <= 1.5 * eE + 1e-3
            assert rel_fro(rows_of(dCa, vr), ref_dC) == eC          # dC is untouched by the flag
            del dEa, dCa

    if name in ("gemma2_2b", "stress"):
        print("uncapped twin of %s: shift invariance and sum_j dC_j = 0 at full size" % name, flush=True)
        check_invariants_without_cap(w, E, C, t, dloss)


@pytest.mark.parametrize("name", MORE_SHAPES)
def test_more_model_shapes_match_the_oracle(cce, name):
    """Other shapes of the paper's Table A3 (Gemma-2 9B: D = 3584; Qwen-2.5 7B: |V| = 152064) and a small
    batch at the Gemma-2 2B shape (N = 1024: wider slabs, the dE product's contraction split in parts)."""
    print("generating %s" % name, flush=True)
    w = make(name)
    g = load_golden(name, w)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    e_lse = max_rel(f64(lse), g["lse"].astype(np.float64))
    e_loss = max_rel(f64(loss), g["loss"].astype(np.float64))
    print("  %s N=%d D=%d V=%d: lse err %.2e  loss err %.2e" % (name, w.N, w.D, w.V, e_lse, e_loss), flush=True)
    assert e_lse <= TOL_LOSS and e_loss <= TOL_LOSS
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE, dC, stats = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    assert stats[0] == stats[1] > 0
    check_sampled_rows(name, w, g, dE, dC, "dense")
    er, vr = g["dE_rows"], g["dC_rows"]
    ref_dE, ref_dC = g["dE"].astype(np.float64), g["dC"].astype(np.float64)
    eE, eC = rel_fro(rows_of(dE, er), ref_dE), rel_fro(rows_of(dC, vr), ref_dC)
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    dEf, dCf, stats_f = run_backward(w, E, C, t, lse, dloss)
    fE, fC = rel_fro(rows_of(dEf, er), ref_dE), rel_fro(rows_of(dCf, vr), ref_dC)
    elemE = rel_fro(g["dE_f"].astype(np.float64), ref_dE)
    elemC = rel_fro(g["dC_f"].astype(np.float64), ref_dC)
    print("  filtered: dE rows err %.2e (element-wise filter %.2e)  dC rows err %.2e (%.2e)  blocks kept %d / %d"
          % (fE, elemE, fC, elemC, stats_f[1], stats_f[0]), flush=True)
    assert fE <= elemE + eE + 1e-3 and fC <= elemC + eC + 1e-3
    assert fE <= FILTERED_DE_BOUND.get(name, TOL_GRAD) and fC <= TOL_GRAD


def test_largest_configuration_sub_batch_against_the_complete_oracle(cce):
    """Config 5 (D = 5120, |V| = 131072): on the first N' tokens (N' not a multiple of the tile width) the
    oracle runs the whole backward, so every row of dC and of dE is compared, not a sample."""
    import dataclasses
    n_sub = 3000
    print("generating stress_peaked", flush=True)
    full = make("stress_peaked")
    w = dataclasses.replace(full, N=n_sub, E=full.E[:n_sub].copy(), targets=full.targets[:n_sub].copy())
    del full
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    lam = w.mean_dloss()
    dE, dC, _ = run_backward(w, E, C, t, lse, torch.from_numpy(lam).cuda(), eps=0.0)
    t0 = time.time()
    E64, C64 = w.E64(), w.C64()
    ref_loss, ref_lse = O.forward(E64, C64, w.targets, w.softcap, w.ignore_index)
    print("  oracle forward %.0f s" % (time.time() - t0), flush=True)
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS
    rdE, rdC = O.backward(E64, C64, w.targets, ref_lse, lam.astype(np.float64), w.softcap, w.ignore_index)
    print("  oracle backward done at %.0f s" % (time.time() - t0), flush=True)
    del E64, C64
    got_dC = f64(dC)
    eE, eC = rel_fro(f64(dE), rdE), rel_fro(got_dC, rdC)
    rE, rC = max_row_err(f64(dE), rdE), max_row_err(got_dC, rdC)
    print("  N'=%d: dE err %.2e (worst row %.2e), all %d rows of dC err %.2e (worst row %.2e)"
          % (n_sub, eE, rE, w.V, eC, rC), flush=True)
    assert eE <= TOL_GRAD and eC <= TOL_GRAD and rE <= TOL_ROW and rC <= TOL_ROW
