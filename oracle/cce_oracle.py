"""Plain fp64 CPU oracle for linear cross-entropy (test infrastructure only).

This module is the slow, obviously-correct definition that the HIP path is
checked against.  It materialises the logit matrix (in row chunks, purely to
bound host memory: every row is independent, so chunking changes nothing) and
applies the textbook formulas in float64.  It shares no code with the GPU
library and must never be imported by the product package; only tests, the
smoke check and the benchmark's CPU-baseline leg use it.

Definitions followed (paper section / equation):
  * Section 3 "Cut Cross-Entropy", Eq. 4: per-token log-likelihood
        l_i = C_{x_i}^T E_i - log sum_j exp(C_j^T E_i).
    The returned `loss` is the negative log-likelihood  -l_i  (so that C = 0
    gives log|V|), and is 0 for ignored tokens.
  * Section 4.2, Alg. 2: LSE_i = log sum_j exp(a_ij), evaluated with the row
    maximum subtracted so that no exponential overflows.
  * Section 4.3 (gradient of the LSE term) and Alg. 4 (merged backward):
        S = exp(A - LSE),  G = S - onehot(x)   (sign follows the NLL),
        dE = (G . dloss) C,   dC = (G . dloss)^T E.
  * Section 4.3 "Gradient filtering": entries (or whole blocks, Alg. 4's
    all(|G| < eps) test) below eps = 2^-12 are dropped before the two products.
  * Section 5 (ablations "CCE" vs "CCE-Kahan"): the paper's kernels keep their
    sums in global memory in the gradient's storage type (bf16), optionally
    with Kahan-compensated summation.  round_to_bf16, accumulate_rounded and
    backward_dE_slab_accumulated model exactly that for a sum over vocabulary
    slabs, so that the library's accumulation variants have something to be
    compared with beyond the exact gradient.
  * Table A2 names logit soft-capping; the paper gives no formula.  Reading
    used here: a = cap * tanh(z / cap), applied to every logit including the
    target's, with derivative 1 - (a/cap)^2 chained into the gradient.

Layout: E is [N, D], C is [V, D] (the paper's D x N and D x |V| matrices of
Appendix A, whose columns are the tokens / vocabulary entries, stored with that
index outermost), targets int64 [N].

Every function is pinned by tests/test_oracle_pins.py against closed forms,
finite differences, scipy/torch library routines and brute force; none is
"parity unpinned".  What is unpinned is the absolute loss/gradient value on the
paper's own workloads: the paper prints none.
"""
from __future__ import annotations

import numpy as np

FILTER_EPS_BF16 = 2.0 ** -12   # Section 4.3: smallest bf16 value not truncated


def _as64(x):
    return np.asarray(x, dtype=np.float64)


def valid_mask(targets, V, ignore_index):
    """Tokens that carry a loss: target != ignore_index and inside [0, V)."""
    t = np.asarray(targets, dtype=np.int64)
    return (t != ignore_index) & (t >= 0) & (t < V)


def logits(E, C, softcap=0.0):
    """A = softcap(E C^T), [n, V] float64.  softcap == 0 disables the cap."""
    Z = _as64(E) @ _as64(C).T
    if softcap and softcap > 0:
        return softcap * np.tanh(Z / softcap)
    return Z


def lse_of_logits(A):
    """Row-wise log-sum-exp with the row maximum subtracted (Alg. 2)."""
    m = np.max(A, axis=1)
    return m + np.log(np.sum(np.exp(A - m[:, None]), axis=1))


def forward(E, C, targets, softcap=0.0, ignore_index=-100, row_chunk=1024):
    """Per-token NLL and LSE (Eq. 4).  Returns (loss [N], lse [N]) float64.

    lse is defined for every row; loss is 0 where the token is ignored."""
    E = np.asarray(E)
    C64 = _as64(C)
    N, V = E.shape[0], C64.shape[0]
    t = np.asarray(targets, dtype=np.int64)
    ok = valid_mask(t, V, ignore_index)
    loss = np.zeros(N, dtype=np.float64)
    lse = np.empty(N, dtype=np.float64)
    for r0 in range(0, N, row_chunk):
        r1 = min(N, r0 + row_chunk)
        A = logits(E[r0:r1], C64, softcap)
        l = lse_of_logits(A)
        lse[r0:r1] = l
        rows = np.nonzero(ok[r0:r1])[0]
        loss[r0 + rows] = l[rows] - A[rows, t[r0 + rows]]
    return loss, lse


def softmax_minus_onehot(A, lse, targets, ok):
    """G = exp(A - lse) - onehot(target) for valid rows, identically 0 otherwise."""
    G = np.exp(A - lse[:, None])
    rows = np.nonzero(ok)[0]
    G[rows, targets[rows]] -= 1.0
    G[~ok] = 0.0
    return G


def apply_filter(G, eps, mode="element", block=(128, 128), row0=0):
    """Gradient filtering of Section 4.3 / Alg. 4.

    mode "element": zero every entry with |G| < eps (finest granularity).
    mode "block":   zero a (B_N x B_V) block only when all its entries are
                    < eps in magnitude (the algorithm's block-level skip).
                    row0 is the global index of G's first row so that blocks
                    line up when the caller passes row chunks."""
    if not eps or eps <= 0 or mode == "none":
        return G
    if mode == "element":
        return np.where(np.abs(G) < eps, 0.0, G)
    if mode != "block":
        raise ValueError(mode)
    bn, bv = block
    if row0 % bn:
        raise ValueError("row chunks must start on a block boundary")
    out = G.copy()
    n, V = G.shape
    small = np.abs(G) < eps
    for i0 in range(0, n, bn):
        for j0 in range(0, V, bv):
            if small[i0:i0 + bn, j0:j0 + bv].all():
                out[i0:i0 + bn, j0:j0 + bv] = 0.0
    return out


def grad_wrt_preactivation(A, G, dloss, softcap):
    """GZ_ij = dloss_i * G_ij * d a_ij / d z_ij, with a = cap*tanh(z/cap)."""
    GZ = G * _as64(dloss)[:, None]
    if softcap and softcap > 0:
        GZ = GZ * (1.0 - (A / softcap) ** 2)
    return GZ


def backward(E, C, targets, lse, dloss, softcap=0.0, ignore_index=-100,
             eps=0.0, filter_mode="element", block=(128, 128),
             filter_dE=True, filter_dC=True, row_chunk=1024):
    """dE [N, D], dC [V, D] in float64 (Section 4.3 gradient; Alg. 4).

    lse must be the forward's LSE; dloss is the upstream gradient of the
    per-token NLL (not read for ignored rows).  eps == 0: exact gradient."""
    E64, C64 = _as64(E), _as64(C)
    N, V = E64.shape[0], C64.shape[0]
    t = np.asarray(targets, dtype=np.int64)
    ok = valid_mask(t, V, ignore_index)
    lam = np.where(ok, _as64(dloss), 0.0)
    lse = _as64(lse)
    dE = np.zeros_like(E64)
    dC = np.zeros_like(C64)
    if filter_mode == "block" and row_chunk % block[0]:
        row_chunk = max(block[0], (row_chunk // block[0]) * block[0])
    for r0 in range(0, N, row_chunk):
        r1 = min(N, r0 + row_chunk)
        A = logits(E64[r0:r1], C64, softcap)
        G = softmax_minus_onehot(A, lse[r0:r1], t[r0:r1], ok[r0:r1])
        Gf = apply_filter(G, eps, filter_mode, block, r0)
        G_e = Gf if filter_dE else G
        G_c = Gf if filter_dC else G
        dE[r0:r1] = grad_wrt_preactivation(A, G_e, lam[r0:r1], softcap) @ C64
        dC += grad_wrt_preactivation(A, G_c, lam[r0:r1], softcap).T @ E64[r0:r1]
    return dE, dC


def backward_dE_rows(E, C, targets, lse, dloss, rows, softcap=0.0, ignore_index=-100,
                     eps=0.0):
    """dE restricted to the given token rows: each row of dE depends only on
    its own row of E, its target, its LSE and all of C."""
    rows = np.asarray(rows, dtype=np.int64)
    E64, C64 = _as64(np.asarray(E)[rows]), _as64(C)
    V = C64.shape[0]
    t = np.asarray(targets, dtype=np.int64)[rows]
    ok = valid_mask(t, V, ignore_index)
    lam = np.where(ok, _as64(dloss)[rows], 0.0)
    A = logits(E64, C64, softcap)
    G = softmax_minus_onehot(A, _as64(lse)[rows], t, ok)
    G = apply_filter(G, eps, "element")
    return grad_wrt_preactivation(A, G, lam, softcap) @ C64


def backward_dC_rows(E, C, targets, lse, dloss, vocab_rows, softcap=0.0, ignore_index=-100,
                     eps=0.0):
    """dC restricted to the given vocabulary rows J: dC_j = sum_i GZ_ij E_i only
    needs column j of the logits, given the full-vocabulary LSE of every token."""
    J = np.asarray(vocab_rows, dtype=np.int64)
    E64, CJ = _as64(E), _as64(np.asarray(C)[J])
    V = np.asarray(C).shape[0]
    t = np.asarray(targets, dtype=np.int64)
    ok = valid_mask(t, V, ignore_index)
    lam = np.where(ok, _as64(dloss), 0.0)
    Z = E64 @ CJ.T
    A = softcap * np.tanh(Z / softcap) if softcap and softcap > 0 else Z
    G = np.exp(A - _as64(lse)[:, None])
    G[~ok] = 0.0
    hit = ok[:, None] & (t[:, None] == J[None, :])
    G[hit] -= 1.0
    G = apply_filter(G, eps, "element")
    return grad_wrt_preactivation(A, G, lam, softcap).T @ E64


def significant_entries_per_row(E, C, lse, softcap=0.0, eps=FILTER_EPS_BF16, row_chunk=1024):
    """Number of softmax entries >= eps in each row (Section 4.3 bounds it by 1/eps)."""
    E = np.asarray(E)
    C64 = _as64(C)
    out = np.empty(E.shape[0], dtype=np.int64)
    for r0 in range(0, E.shape[0], row_chunk):
        r1 = min(E.shape[0], r0 + row_chunk)
        S = np.exp(logits(E[r0:r1], C64, softcap) - _as64(lse)[r0:r1, None])
        out[r0:r1] = np.count_nonzero(S >= eps, axis=1)
    return out


def round_to_bf16(x):
    """Nearest bfloat16 (8 significant bits, ties to even) of every float64 in x, returned as float64.

    Rounded directly from float64 (no intermediate float32).  The exponent range of bfloat16 is not
    modelled: it equals float32's and nothing on this path comes near its ends."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2**e with 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)   # rint: ties to even


def accumulate_rounded(terms, mode="bf16"):
    """Sum terms[0] + terms[1] + ... with the running sum kept in bf16 (Section 5).

    mode "exact": plain float64 sum.
    mode "bf16":  sum <- round_to_bf16(sum + term) after every term.
    mode "kahan": Kahan's compensated summation with both the running sum and the compensation
                  stored in bf16:  y = term - comp;  t = round(sum + y);  comp = round((t - sum) - y);  sum = t."""
    terms = [np.asarray(t, dtype=np.float64) for t in terms]
    total = np.zeros_like(terms[0])
    comp = np.zeros_like(terms[0])
    for term in terms:
        if mode == "exact":
            total = total + term
        elif mode == "bf16":
            total = round_to_bf16(total + term)
        elif mode == "kahan":
            y = term - comp
            t = round_to_bf16(total + y)
            comp = round_to_bf16((t - total) - y)
            total = t
        else:
            raise ValueError(mode)
    return total


def backward_dE_slab_accumulated(E, C, targets, lse, dloss, slab_cols, mode="bf16", softcap=0.0,
                                 ignore_index=-100):
    """dE as a sum over vocabulary slabs of slab_cols entries, accumulated as accumulate_rounded does.

    Slab s contributes sum_{j in slab} GZ_ij C_j (exact, float64); the contributions are then added in
    slab order with the running sum in the chosen precision."""
    E64, C64 = _as64(E), _as64(C)
    V = C64.shape[0]
    t = np.asarray(targets, dtype=np.int64)
    ok = valid_mask(t, V, ignore_index)
    lam = np.where(ok, _as64(dloss), 0.0)
    lse = _as64(lse)
    terms = []
    for v0 in range(0, V, int(slab_cols)):
        v1 = min(V, v0 + int(slab_cols))
        A = logits(E64, C64[v0:v1], softcap)
        G = np.exp(A - lse[:, None])
        G[~ok] = 0.0
        hit = np.nonzero(ok & (t >= v0) & (t < v1))[0]
        G[hit, t[hit] - v0] -= 1.0
        terms.append(grad_wrt_preactivation(A, G, lam, softcap) @ C64[v0:v1])
    return accumulate_rounded(terms, mode)
