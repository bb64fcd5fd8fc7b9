"""Pins for the fp64 oracle: closed forms, library routines, finite differences,
brute force and invariants.  None of these call the HIP path.

Each pin is chosen so that a plausible mistake in the oracle (dropped term,
wrong sign or index, transposed operand, cap applied in the wrong place)
fails at least one of them; test_planted_mistakes_are_caught checks that."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import cce_oracle as O
from workloads import make

IGN = -100


def rand_problem(seed, N=12, D=7, V=19, scale=1.0, ignore=(1, 5)):
    rng = np.random.default_rng(seed)
    E = rng.standard_normal((N, D)) * scale
    C = rng.standard_normal((V, D)) * scale
    x = rng.integers(0, V, N)
    for i in ignore:
        if i < N:
            x[i] = IGN
    lam = rng.standard_normal(N)
    return E, C, x, lam


# ----------------------------------------------------------------- forward pins
@pytest.mark.parametrize("cap", [0.0, 30.0])
def test_zero_classifier_gives_log_V(cap):
    E, C, x, _ = rand_problem(0, N=9, D=5, V=37)
    loss, lse = O.forward(E, np.zeros_like(C), x, cap, IGN)
    ok = x != IGN
    assert np.allclose(lse, math.log(37), rtol=0, atol=1e-14)
    assert np.allclose(loss[ok], math.log(37), rtol=0, atol=1e-14)
    assert np.all(loss[~ok] == 0.0)
    loss2, lse2 = O.forward(np.zeros_like(E), C, x, cap, IGN)
    assert np.allclose(lse2, math.log(37), atol=1e-14) and np.allclose(loss2[ok], math.log(37), atol=1e-14)


def test_single_class_and_two_class_closed_forms():
    E, C, x, _ = rand_problem(1, V=1, ignore=())
    x[:] = 0
    loss, lse = O.forward(E, C, x, 0.0, IGN)
    assert np.allclose(loss, 0.0, atol=1e-14)
    assert np.allclose(lse, E @ C[0], atol=1e-13)
    E, C, x, _ = rand_problem(2, V=2, ignore=())
    loss, _ = O.forward(E, C, x, 0.0, IGN)
    z = E @ C.T
    other = z[np.arange(len(x)), 1 - x]
    tgt = z[np.arange(len(x)), x]
    assert np.allclose(loss, np.logaddexp(0.0, other - tgt), atol=1e-13)   # softplus


@pytest.mark.parametrize("cap", [0.0, 2.5])
@pytest.mark.parametrize("scale", [1.0, 6.0])
def test_against_scipy_and_torch_library_routines(cap, scale):
    E, C, x, _ = rand_problem(3, N=33, D=11, V=57, scale=scale, ignore=(0, 7, 32))
    loss, lse = O.forward(E, C, x, cap, IGN, row_chunk=8)
    Z = torch.tensor(E) @ torch.tensor(C).T
    A = cap * torch.tanh(Z / cap) if cap > 0 else Z
    ref = torch.nn.functional.cross_entropy(A, torch.tensor(x), reduction="none", ignore_index=IGN)
    assert np.allclose(loss, ref.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(lse, scipy.special.logsumexp(A.numpy(), axis=1), rtol=1e-13, atol=1e-13)


def test_lse_bounds_and_softcap_bound():
    E, C, x, _ = rand_problem(4, N=20, D=9, V=50, scale=3.0)
    for cap in (0.0, 4.0):
        A = O.logits(E, C, cap)
        _, lse = O.forward(E, C, x, cap, IGN)
        assert np.all(lse >= A.max(1) - 1e-12) and np.all(lse <= A.max(1) + math.log(50) + 1e-12)
        if cap:
            assert np.all(np.abs(A) <= cap) and np.all(lse <= cap + math.log(50))


def test_shift_invariance_without_cap():
    E, C, x, _ = rand_problem(5)
    u = np.random.default_rng(9).standard_normal(C.shape[1])
    l0, s0 = O.forward(E, C, x, 0.0, IGN)
    l1, s1 = O.forward(E, C + u, x, 0.0, IGN)
    assert np.allclose(l0, l1, atol=1e-11)
    assert np.allclose(s1 - s0, E @ u, atol=1e-11)


def test_large_logits_do_not_overflow():
    E, C, x, _ = rand_problem(6, scale=40.0, ignore=())
    loss, lse = O.forward(E, C, x, 0.0, IGN)
    assert np.all(np.isfinite(loss)) and np.all(np.isfinite(lse))
    # exact: brute force in extended precision via python floats / math.fsum on shifted values
    Z = E @ C.T
    for i in range(3):
        m = max(Z[i])
        ref = m + math.log(math.fsum(math.exp(z - m) for z in Z[i]))
        assert abs(lse[i] - ref) <= 1e-12 * abs(ref)


def test_out_of_range_target_is_treated_as_ignored():
    E, C, x, lam = rand_problem(7, ignore=())
    x2 = x.copy()
    x2[3] = C.shape[0] + 4
    x3 = x.copy()
    x3[3] = IGN
    la, sa = O.forward(E, C, x2, 0.0, IGN)
    lb, sb = O.forward(E, C, x3, 0.0, IGN)
    assert np.array_equal(la, lb) and np.array_equal(sa, sb)


# ---------------------------------------------------------------- backward pins
def total_loss(E, C, x, lam, cap):
    loss, _ = O.forward(E, C, x, cap, IGN)
    ok = x != IGN
    return float(np.sum(lam[ok] * loss[ok]))


@pytest.mark.parametrize("cap", [0.0, 1.7])
def test_gradients_match_central_finite_differences(cap):
    E, C, x, lam = rand_problem(10, N=6, D=5, V=11, ignore=(2,))
    _, lse = O.forward(E, C, x, cap, IGN)
    dE, dC = O.backward(E, C, x, lse, lam, cap, IGN)
    h = 1e-6
    fdE = np.zeros_like(E)
    for i in range(E.shape[0]):
        for d in range(E.shape[1]):
            Ep, Em = E.copy(), E.copy()
            Ep[i, d] += h
            Em[i, d] -= h
            fdE[i, d] = (total_loss(Ep, C, x, lam, cap) - total_loss(Em, C, x, lam, cap)) / (2 * h)
    fdC = np.zeros_like(C)
    for j in range(C.shape[0]):
        for d in range(C.shape[1]):
            Cp, Cm = C.copy(), C.copy()
            Cp[j, d] += h
            Cm[j, d] -= h
            fdC[j, d] = (total_loss(E, Cp, x, lam, cap) - total_loss(E, Cm, x, lam, cap)) / (2 * h)
    assert np.linalg.norm(dE - fdE) <= 1e-7 * max(np.linalg.norm(fdE), 1.0)
    assert np.linalg.norm(dC - fdC) <= 1e-7 * max(np.linalg.norm(fdC), 1.0)
    assert np.all(dE[2] == 0.0)   # ignored token: no gradient


@pytest.mark.parametrize("cap", [0.0, 3.0])
def test_gradients_match_torch_autograd(cap):
    E, C, x, lam = rand_problem(11, N=40, D=13, V=70, scale=2.0, ignore=(0, 9, 39))
    lam[9] = np.nan   # ignored rows' upstream gradient must not be read
    _, lse = O.forward(E, C, x, cap, IGN)
    dE, dC = O.backward(E, C, x, lse, lam, cap, IGN, row_chunk=16)
    Et = torch.tensor(E, requires_grad=True)
    Ct = torch.tensor(C, requires_grad=True)
    Z = Et @ Ct.T
    A = cap * torch.tanh(Z / cap) if cap > 0 else Z
    per_tok = torch.nn.functional.cross_entropy(A, torch.tensor(x), reduction="none", ignore_index=IGN)
    lam_t = torch.tensor(np.where(x != IGN, lam, 0.0))
    (per_tok * lam_t).sum().backward()
    assert np.allclose(dE, Et.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(dC, Ct.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_zero_classifier_gradient_closed_form():
    E, C, x, lam = rand_problem(12, N=10, D=4, V=6, ignore=(3,))
    C0 = np.zeros_like(C)
    _, lse = O.forward(E, C0, x, 0.0, IGN)
    dE, dC = O.backward(E, C0, x, lse, lam, 0.0, IGN)
    assert np.allclose(dE, 0.0, atol=1e-15)
    V = C.shape[0]
    ref = np.zeros_like(C)
    for j in range(V):
        for i in range(len(x)):
            if x[i] == IGN:
                continue
            ref[j] += lam[i] * (1.0 / V - (1.0 if x[i] == j else 0.0)) * E[i]
    assert np.allclose(dC, ref, atol=1e-13)


def test_structure_of_G_and_uncapped_identities():
    E, C, x, lam = rand_problem(13, N=15, D=6, V=23, scale=2.0, ignore=(4,))
    _, lse = O.forward(E, C, x, 0.0, IGN)
    A = O.logits(E, C)
    ok = O.valid_mask(x, C.shape[0], IGN)
    G = O.softmax_minus_onehot(A, lse, x, ok)
    assert np.allclose(G[ok].sum(1), 0.0, atol=1e-13)          # softmax rows sum to one
    assert np.all(G[~ok] == 0.0)
    assert np.all(G[ok, x[ok]] < 0) and np.count_nonzero(G < 0) == ok.sum()
    dE, dC = O.backward(E, C, x, lse, lam, 0.0, IGN)
    assert np.allclose(dC.sum(0), 0.0, atol=1e-12)             # sum_j dC_j = 0 without cap
    S = scipy.special.softmax(A, axis=1)
    for i in np.nonzero(ok)[0]:
        assert np.allclose(dE[i], lam[i] * (S[i] @ C - C[x[i]]), atol=1e-12)


def test_linearity_in_upstream_gradient_and_vocab_permutation():
    E, C, x, lam = rand_problem(14, N=14, D=6, V=21, ignore=(2,))
    cap = 2.0
    _, lse = O.forward(E, C, x, cap, IGN)
    dE1, dC1 = O.backward(E, C, x, lse, lam, cap, IGN)
    dE2, dC2 = O.backward(E, C, x, lse, 3.0 * lam, cap, IGN)
    assert np.allclose(dE2, 3 * dE1, atol=1e-13) and np.allclose(dC2, 3 * dC1, atol=1e-13)
    perm = np.random.default_rng(3).permutation(C.shape[0])      # new row r holds old row perm[r]
    inv = np.argsort(perm)
    xp = np.where(x == IGN, IGN, inv[np.clip(x, 0, None)])
    lp, sp = O.forward(E, C[perm], xp, cap, IGN)
    l0, s0 = O.forward(E, C, x, cap, IGN)
    assert np.allclose(lp, l0, atol=1e-13) and np.allclose(sp, s0, atol=1e-13)
    dEp, dCp = O.backward(E, C[perm], xp, sp, lam, cap, IGN)
    assert np.allclose(dEp, dE1, atol=1e-13) and np.allclose(dCp, dC1[perm], atol=1e-13)


def test_row_and_column_restricted_backward_agree_with_full():
    E, C, x, lam = rand_problem(15, N=30, D=8, V=41, scale=2.0, ignore=(1, 5))
    for cap in (0.0, 2.0):
        _, lse = O.forward(E, C, x, cap, IGN)
        dE, dC = O.backward(E, C, x, lse, lam, cap, IGN)
        rows = np.array([0, 1, 7, 29])
        J = np.array([0, 3, int(x[0]), 40])
        assert np.allclose(O.backward_dE_rows(E, C, x, lse, lam, rows, cap, IGN), dE[rows], atol=1e-13)
        assert np.allclose(O.backward_dC_rows(E, C, x, lse, lam, J, cap, IGN), dC[J], atol=1e-13)
        eps = 0.01
        dEf, dCf = O.backward(E, C, x, lse, lam, cap, IGN, eps=eps, filter_mode="element")
        assert np.allclose(O.backward_dE_rows(E, C, x, lse, lam, rows, cap, IGN, eps=eps), dEf[rows], atol=1e-13)
        assert np.allclose(O.backward_dC_rows(E, C, x, lse, lam, J, cap, IGN, eps=eps), dCf[J], atol=1e-13)


# --------------------------------------------------------------- filtering pins
def test_filter_eps_zero_is_identity_and_element_error_bound():
    E, C, x, lam = rand_problem(16, N=24, D=8, V=300, scale=1.5, ignore=(3,))
    _, lse = O.forward(E, C, x, 0.0, IGN)
    dE, dC = O.backward(E, C, x, lse, lam, 0.0, IGN)
    dE0, dC0 = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=0.0)
    assert np.array_equal(dE, dE0) and np.array_equal(dC, dC0)
    eps = 2e-3
    dEf, dCf = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="element")
    A = O.logits(E, C)
    ok = O.valid_mask(x, C.shape[0], IGN)
    G = O.softmax_minus_onehot(A, lse, x, ok)
    dropped = np.where(np.abs(G) < eps, np.abs(G), 0.0).sum(1)
    assert dropped.max() > 0           # the filter did something
    bound = np.abs(lam) * dropped * np.linalg.norm(C, axis=1).max()
    err = np.linalg.norm(dEf - dE, axis=1)
    assert np.all(err[ok] <= bound[ok] + 1e-15)
    assert np.all(err[~ok] == 0)


def test_block_filter_sandwich():
    E, C, x, lam = rand_problem(17, N=32, D=8, V=256, scale=2.5, ignore=())
    _, lse = O.forward(E, C, x, 0.0, IGN)
    eps = 1e-3
    full = O.backward(E, C, x, lse, lam, 0.0, IGN)
    elem = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="element")
    blk = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="block", block=(8, 16), row_chunk=16)
    blk_one = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="block", block=(8, 16), row_chunk=1024)
    assert np.allclose(blk[0], blk_one[0], atol=1e-14) and np.allclose(blk[1], blk_one[1], atol=1e-14)
    # brute-force block filter
    A = O.logits(E, C)
    G = O.softmax_minus_onehot(A, lse, x, np.ones(len(x), bool))
    Gb = G.copy()
    skipped = 0
    for i0 in range(0, 32, 8):
        for j0 in range(0, 256, 16):
            if np.all(np.abs(G[i0:i0 + 8, j0:j0 + 16]) < eps):
                Gb[i0:i0 + 8, j0:j0 + 16] = 0
                skipped += 1
    assert 0 < skipped < 4 * 16
    assert np.allclose(blk[0], (Gb * lam[:, None]) @ C, atol=1e-13)
    assert np.allclose(blk[1], (Gb * lam[:, None]).T @ E, atol=1e-13)
    # every block-skipped entry is also element-skipped: block error <= element error (per row, in L1 of dropped mass)
    d_blk = np.abs(G - Gb).sum()
    d_el = np.abs(G - np.where(np.abs(G) < eps, 0, G)).sum()
    assert d_blk <= d_el + 1e-15
    # FullC / FullE variants: filter only one of the two gradients
    onlyE = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="element", filter_dC=False)
    assert np.array_equal(onlyE[0], elem[0]) and np.array_equal(onlyE[1], full[1])
    onlyC = O.backward(E, C, x, lse, lam, 0.0, IGN, eps=eps, filter_mode="element", filter_dE=False)
    assert np.array_equal(onlyC[0], full[0]) and np.array_equal(onlyC[1], elem[1])


def _constructed_counts():
    """A problem whose number of softmax entries >= 2^-12 is known exactly for every row.

    E_i is a unit vector e_{r(i)} and column r of C holds log(50) in its first k_r rows and 0 below, so row i
    of the logits has k_r entries log(50) and V - k_r zeros: softmax 50 / (50 k + V - k) for the former and
    1 / (50 k + V - k) for the latter.  With V = 5000 the former are far above 2^-12 (0.0084 at k = 20) and
    the latter below it (at most 1 / 5049 = 0.000198 < 0.000244), so the count is k_r."""
    V, ks = 5000, [1, 2, 7, 20]
    C = np.zeros((V, len(ks)))
    for r, k in enumerate(ks):
        C[:k, r] = math.log(50.0)
    pattern = [0, 3, 1, 2, 2, 0, 3]
    E = np.eye(len(ks))[pattern]
    expect = np.array([ks[r] for r in pattern])
    return E, C, expect


def test_significant_entries_per_row_on_a_constructed_case_and_by_brute_force():
    """Section 4.3: at most 1 / eps = 4096 softmax entries per token reach eps = 2^-12."""
    E, C, expect = _constructed_counts()
    x = np.zeros(len(E), dtype=np.int64)
    _, lse = O.forward(E, C, x, 0.0, IGN)
    cnt = O.significant_entries_per_row(E, C, lse, row_chunk=3)          # several chunks and a ragged last one
    assert np.array_equal(cnt, expect)
    # another threshold moves the count as the closed form says: every entry is >= 1 / 6000
    assert np.array_equal(O.significant_entries_per_row(E, C, lse, eps=1.0 / 6000), np.full(len(E), 5000))
    # with a cap the logits become cap * tanh(log(50) / cap): still k entries far above the rest
    _, lse_c = O.forward(E, C, x, 2.0, IGN)
    assert np.array_equal(O.significant_entries_per_row(E, C, lse_c, softcap=2.0), expect)
    # brute force with scalar arithmetic on a small random problem (math.exp, plain loops)
    Er, Cr, xr, _ = rand_problem(18, N=9, D=6, V=300, scale=1.4, ignore=())
    eps = 1.0 / 256
    _, lse_r = O.forward(Er, Cr, xr, 0.0, IGN)
    brute = []
    for i in range(9):
        z = [sum(Er[i, d] * Cr[j, d] for d in range(6)) for j in range(300)]
        tot = math.fsum(math.exp(v) for v in z)
        brute.append(sum(1 for v in z if math.exp(v) / tot >= eps))
    got = O.significant_entries_per_row(Er, Cr, lse_r, eps=eps)
    assert np.array_equal(got, np.array(brute)) and 0 < got.min() and got.max() < 300
    assert got.max() <= 256                                              # the 1 / eps bound
    # uniform softmax over 6000 classes: every entry 1/6000 < 2^-12, none significant
    cnt0 = O.significant_entries_per_row(Er, np.zeros((6000, 6)), np.full(9, math.log(6000)))
    assert np.all(cnt0 == 0)
    # and the bound of the paper at its own threshold on a wide random problem
    Ew, Cw, xw, _ = rand_problem(19, N=16, D=8, V=6000, scale=0.3, ignore=())
    _, lse_w = O.forward(Ew, Cw, xw, 0.0, IGN)
    assert O.significant_entries_per_row(Ew, Cw, lse_w).max() <= 4096


def test_planted_mistakes_in_the_entry_counter_are_caught(monkeypatch):
    E, C, expect = _constructed_counts()
    x = np.zeros(len(E), dtype=np.int64)
    _, lse = O.forward(E, C, x, 0.0, IGN)

    def pin_passes():
        return bool(np.array_equal(O.significant_entries_per_row(E, C, lse, row_chunk=3), expect))

    assert pin_passes()
    orig_logits = O.logits
    orig_count = np.count_nonzero
    monkeypatch.setattr(O.np, "count_nonzero", lambda a, axis=None: orig_count(a, axis=axis) - 1)      # off by one
    assert not pin_passes()
    monkeypatch.setattr(O.np, "count_nonzero", orig_count)
    monkeypatch.setattr(O.np, "count_nonzero", lambda a, axis=None: orig_count(a, axis=axis) * 0)      # returns zeros
    assert not pin_passes()
    monkeypatch.setattr(O.np, "count_nonzero", orig_count)
    monkeypatch.setattr(O, "logits", lambda E_, C_, cap=0.0: -orig_logits(E_, C_, cap))                # wrong sign
    assert not pin_passes()
    monkeypatch.setattr(O, "logits", orig_logits)
    assert pin_passes()


# ------------------------------------------------- sums kept in bf16 (Section 5, "CCE" vs "CCE-Kahan")
def test_round_to_bf16_against_ties_a_bit_level_rounding_and_torch():
    # spacing in [1, 2) is 2^-7: exact ties go to the even mantissa
    assert O.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert O.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7      # just above the tie
    assert O.round_to_bf16(-257.0) == -256.0 and O.round_to_bf16(259.0) == 260.0 and O.round_to_bf16(0.0) == 0.0
    rng = np.random.default_rng(31)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    from workloads import f32_to_bf16_bits
    from workloads.configs import bf16_bits_to_f64
    assert np.array_equal(O.round_to_bf16(x.astype(np.float64)), bf16_bits_to_f64(f32_to_bf16_bits(x)))
    assert np.array_equal(O.round_to_bf16(x.astype(np.float64)), torch.tensor(x).to(torch.bfloat16).double().numpy())


def test_accumulate_rounded_stalls_without_compensation_and_recovers_with_it():
    ones = [np.ones(3)] * 300
    assert np.array_equal(O.accumulate_rounded(ones, "exact"), np.full(3, 300.0))
    # 256 + 1 is a tie between 256 and 258 and goes to 256: the bf16 running sum stops growing there
    assert np.array_equal(O.accumulate_rounded(ones, "bf16"), np.full(3, 256.0))
    # Kahan's compensation carries the lost units over: the result stays within one spacing (2) of the true sum
    k = O.accumulate_rounded(ones, "kahan")
    assert np.all(np.abs(k - 300.0) <= 2.0) and np.array_equal(k, O.round_to_bf16(k))
    # a hand-checked sequence: 256, then three times 1
    seq = [np.array([256.0]), np.array([1.0]), np.array([1.0]), np.array([1.0])]
    assert O.accumulate_rounded(seq, "bf16")[0] == 256.0
    assert O.accumulate_rounded(seq, "kahan")[0] == 260.0       # 256 ->256 (comp -1) -> 258 (comp 0) -> 260 (tie 259, comp 1)
    # random terms: compensation beats plain rounding, both are exact to within the format
    rng = np.random.default_rng(32)
    terms = [rng.standard_normal(4000) for _ in range(64)]
    exact = O.accumulate_rounded(terms, "exact")
    e_b = np.linalg.norm(O.accumulate_rounded(terms, "bf16") - exact) / np.linalg.norm(exact)
    e_k = np.linalg.norm(O.accumulate_rounded(terms, "kahan") - exact) / np.linalg.norm(exact)
    e_1 = np.linalg.norm(O.round_to_bf16(exact) - exact) / np.linalg.norm(exact)
    assert e_1 < e_k < 2.0 * e_1 and e_b > 2.0 * e_k


def test_slab_accumulated_dE_reduces_to_the_plain_gradient():
    E, C, x, lam = rand_problem(33, N=10, D=6, V=50, ignore=(4,))
    for cap in (0.0, 2.5):
        _, lse = O.forward(E, C, x, cap, IGN)
        dE, _ = O.backward(E, C, x, lse, lam, cap, IGN)
        for slab in (7, 16, 50, 64):      # ragged last slab, exact division, one slab, more than |V|
            got = O.backward_dE_slab_accumulated(E, C, x, lse, lam, slab, "exact", cap, IGN)
            assert np.allclose(got, dE, rtol=0, atol=1e-13)
        one = O.backward_dE_slab_accumulated(E, C, x, lse, lam, 50, "bf16", cap, IGN)
        assert np.array_equal(one, O.round_to_bf16(dE)) or np.allclose(one, O.round_to_bf16(dE), rtol=2.0 ** -7, atol=0)
        many_b = O.backward_dE_slab_accumulated(E, C, x, lse, lam, 5, "bf16", cap, IGN)
        many_k = O.backward_dE_slab_accumulated(E, C, x, lse, lam, 5, "kahan", cap, IGN)
        n = np.linalg.norm(dE)
        assert np.linalg.norm(many_k - dE) / n <= 2.0 ** -8 and np.linalg.norm(many_b - dE) / n <= 10 * 2.0 ** -8
        assert np.all(many_b[4] == 0) and np.all(many_k[4] == 0)          # ignored token


# ------------------------------------------------------------------ paper values
def _paper_values():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, value = line.split()[:2]
        out[name] = float(value)
    return out


def test_memory_figures_the_paper_prints():
    pv = _paper_values()
    mib = 1 << 20
    assert round((8192 * 2304 + 256000 * 2304) * 2 / mib) == pv["grad_lower_bound_gemma2_2b"]
    assert round((8192 * 3072 + 32064 * 3072) * 2 / mib) == pv["grad_lower_bound_phi35"]
    assert round((8192 * 5120 + 131072 * 5120) * 2 / mib) == pv["grad_lower_bound_nemo"]
    assert 65536 * 256000 * 4 / mib == pv["logits_gemma2_65536"]
    assert 65536 * 128256 * 4 / mib == pv["logits_llama3_65536"]
    assert 1 / O.FILTER_EPS_BF16 == pv["max_significant_per_row"]


# ------------------------------------------------------------- workload generator
def test_generator_is_seeded_and_has_the_stated_structure():
    a = make("gemma2_2b", N=512, D=128, V=4096)
    b = make("gemma2_2b", N=512, D=128, V=4096)
    assert np.array_equal(a.E, b.E) and np.array_equal(a.C, b.C) and np.array_equal(a.targets, b.targets)
    assert a.E.dtype == np.uint16 and a.softcap == 30.0
    e = a.E64()
    assert np.allclose(np.sqrt((e ** 2).mean(1)), 1.0, atol=5e-3)          # RMS-normalised rows
    assert abs(a.C64().std() - 0.02) < 1e-3
    frac = np.mean(a.targets == IGN)
    assert 0.0 < frac < 0.06
    t = a.targets[a.targets != IGN]
    assert t.min() >= 0 and t.max() < 4096
    # Zipf: the most frequent class takes a large share
    assert np.bincount(t).max() > 0.05 * len(t)
    tiny = make("tiny")
    assert tiny.E.dtype == np.float32 and tiny.N == 256 and tiny.V == 1024 and tiny.softcap == 0.0
    pk = make("stress_peaked", N=64, D=64, V=2000)
    assert len(pk.boosted) == 20
    assert pk.C64()[pk.boosted].std() > 4 * pk.C64().std() * 0.5


def test_bf16_rounding_is_round_to_nearest_even():
    from workloads import f32_to_bf16_bits, bf16_bits_to_f64
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -2.5, 0.0], dtype=np.float32)
    got = bf16_bits_to_f64(f32_to_bf16_bits(x))
    assert list(got) == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0]
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    ref = torch.tensor(r).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(bf16_bits_to_f64(f32_to_bf16_bits(r)), ref)


# ---------------------------------------------------------------- planted mistakes
def test_planted_mistakes_are_caught(monkeypatch):
    """Mutate the oracle in plausible ways and check the pins above notice."""
    E, C, x, lam = rand_problem(20, N=8, D=5, V=9, ignore=(2,))
    cap = 1.5

    def pins_pass():
        try:
            loss, lse = O.forward(E, C, x, cap, IGN)
            Z = torch.tensor(E) @ torch.tensor(C).T
            A = cap * torch.tanh(Z / cap)
            ref = torch.nn.functional.cross_entropy(A, torch.tensor(x), reduction="none", ignore_index=IGN).numpy()
            if not np.allclose(loss, ref, atol=1e-12):
                return False
            dE, dC = O.backward(E, C, x, lse, lam, cap, IGN)
            Et = torch.tensor(E, requires_grad=True)
            Ct = torch.tensor(C, requires_grad=True)
            Zt = Et @ Ct.T
            At = cap * torch.tanh(Zt / cap)
            pt = torch.nn.functional.cross_entropy(At, torch.tensor(x), reduction="none", ignore_index=IGN)
            (pt * torch.tensor(np.where(x != IGN, lam, 0.0))).sum().backward()
            return bool(np.allclose(dE, Et.grad.numpy(), atol=1e-11) and np.allclose(dC, Ct.grad.numpy(), atol=1e-11))
        except Exception:
            return False

    assert pins_pass()
    orig_soh = O.softmax_minus_onehot
    orig_gp = O.grad_wrt_preactivation
    orig_lse = O.lse_of_logits

    monkeypatch.setattr(O, "softmax_minus_onehot", lambda A, l, t, ok: -orig_soh(A, l, t, ok))       # wrong sign
    assert not pins_pass()
    monkeypatch.setattr(O, "softmax_minus_onehot", orig_soh)
    monkeypatch.setattr(O, "grad_wrt_preactivation", lambda A, G, d, c: orig_gp(A, G, d, 0.0))        # dropped cap'
    assert not pins_pass()
    monkeypatch.setattr(O, "grad_wrt_preactivation", orig_gp)
    monkeypatch.setattr(O, "lse_of_logits", lambda A: np.log(np.sum(np.exp(A), axis=1)) + 1e-3)       # biased LSE
    assert not pins_pass()
    monkeypatch.setattr(O, "lse_of_logits", orig_lse)

    def onehot_off_by_one(A, l, t, ok):
        return orig_soh(A, l, np.where(ok, (t + 1) % A.shape[1], t), ok)
    monkeypatch.setattr(O, "softmax_minus_onehot", onehot_off_by_one)                                 # wrong index
    assert not pins_pass()
    monkeypatch.setattr(O, "softmax_minus_onehot", orig_soh)
    assert pins_pass()
