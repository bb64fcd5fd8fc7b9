"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  Tolerances:
  loss, LSE : max relative error <= 1e-3   (relative to max(|ref|, 1))
  dE, dC    : relative Frobenius error <= 1e-2 for bf16 storage with fp32 accumulation
For fp32 storage the bounds used are 1e-5 / 1e-4 (fp32 FMA accumulation of D- and
V-long sums).
Sizes here are ones the oracle finishes in seconds; they span several 256-wide
tiles with ragged tails in N and V."""
import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from oracle import cce_oracle as O
from workloads import make

from gpu_util import dtype_code, f64, max_rel, max_row_err, rel_fro, run_backward, run_forward, to_device, workspace

pytestmark = pytest.mark.gpu

TOL_LOSS = 1e-3
TOL_GRAD = 1e-2
TOL_ROW = 1e-2      # every row of dE / dC on its own: ||delta row|| <= TOL_ROW * max(||row||, median row norm)


def oracle_all(w, eps=0.0, mode="element"):
    E, C = w.E64(), w.C64()
    loss, lse = O.forward(E, C, w.targets, w.softcap, w.ignore_index)
    lam = w.mean_dloss().astype(np.float64)
    dE, dC = O.backward(E, C, w.targets, lse, lam, w.softcap, w.ignore_index, eps=eps, filter_mode=mode)
    return loss, lse, dE, dC


MID = [
    # name, N, D, V, extra
    ("gemma2_2b", 600, 128, 1500, {}),            # 3 token tiles (ragged), 6 vocab tiles (ragged), softcap 30
    ("small_vocab", 512, 192, 1024, {}),          # exact tiles, no cap
    ("llama3_8b", 300, 64, 700, {}),              # D = one K stage
    ("stress_peaked", 520, 256, 2100, {}),        # sharp softmax, cap 30
    ("gemma2_2b", 257, 128, 257, {"softcap": 50.0}),   # cap > 40: running-max variant of the capped fold
]


@pytest.mark.parametrize("name,N,D,V,kw", MID)
def test_forward_matches_oracle_mid(cce, name, N, D, V, kw):
    w = make(name, N=N, D=D, V=V, **kw)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    ref_loss, ref_lse = O.forward(w.E64(), w.C64(), w.targets, w.softcap, w.ignore_index)
    e1, e2 = max_rel(f64(lse), ref_lse), max_rel(f64(loss), ref_loss)
    print("fwd %s N=%d D=%d V=%d: lse err %.2e loss err %.2e" % (name, N, D, V, e1, e2))
    assert e1 <= TOL_LOSS and e2 <= TOL_LOSS
    ign = w.targets == w.ignore_index
    assert np.all(f64(loss)[ign] == 0.0)


@pytest.mark.parametrize("name,N,D,V,kw", MID)
def test_backward_unfiltered_matches_oracle_mid(cce, name, N, D, V, kw):
    w = make(name, N=N, D=D, V=V, **kw)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    rng = np.random.default_rng(7)
    lam = (rng.standard_normal(w.N) * 0.01 + 1.0 / w.N).astype(np.float32)   # non-uniform upstream gradient
    lam[w.targets == w.ignore_index] = np.nan                                 # must not be read
    dloss = torch.from_numpy(lam).cuda()
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    ref_loss, ref_lse = O.forward(w.E64(), w.C64(), w.targets, w.softcap, w.ignore_index)
    rdE, rdC = O.backward(w.E64(), w.C64(), w.targets, ref_lse, lam.astype(np.float64), w.softcap, w.ignore_index)
    eE, eC = rel_fro(f64(dE), rdE), rel_fro(f64(dC), rdC)
    rE, rC = max_row_err(f64(dE), rdE), max_row_err(f64(dC), rdC)
    print("bwd %s N=%d D=%d V=%d: dE err %.2e (worst row %.2e) dC err %.2e (worst row %.2e)" % (name, N, D, V, eE, rE, eC, rC))
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    assert rE <= TOL_ROW and rC <= TOL_ROW
    assert np.all(f64(dE)[w.targets == w.ignore_index] == 0.0)


@pytest.mark.parametrize("name,N,D,V,kw", MID[:4])
def test_backward_filtered_is_within_tolerance_of_the_exact_gradient(cce, name, N, D, V, kw):
    w = make(name, N=N, D=D, V=V, **kw)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE, dC, stats = run_backward(w, E, C, t, lse, dloss)          # defaults: both filters, eps 2^-12
    dE0, dC0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    _, ref_lse, rdE, rdC = oracle_all(w)
    _, _, fdE, fdC = oracle_all(w, eps=O.FILTER_EPS_BF16, mode="element")
    eE, eC = rel_fro(f64(dE), rdE), rel_fro(f64(dC), rdC)
    bound_E = rel_fro(fdE, rdE) + rel_fro(f64(dE0), rdE) + 1e-3
    bound_C = rel_fro(fdC, rdC) + rel_fro(f64(dC0), rdC) + 1e-3
    print("filtered %s: dE err %.2e (element-filter oracle %.2e) dC err %.2e (%.2e) blocks kept %d / %d"
          % (name, eE, rel_fro(fdE, rdE), eC, rel_fro(fdC, rdC), stats[1], stats[0]))
    assert eE <= TOL_GRAD and eC <= TOL_GRAD
    # a block skip drops only entries an element-wise filter would drop too
    assert eE <= bound_E and eC <= bound_C
    assert 0 < stats[1] <= stats[0]


def test_full_c_and_full_e_variants(cce):
    """Filtering only dE leaves dC exact and vice versa (the paper's FullC / FullE choices)."""
    w = make("stress_peaked", N=520, D=256, V=2100)
    E, C, t = to_device(w)
    _, lse = run_forward(w, E, C, t)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE0, dC0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    dEf, dCf, _ = run_backward(w, E, C, t, lse, dloss)
    dE1, dC1, _ = run_backward(w, E, C, t, lse, dloss, flags=L.CCE_FILTER_DE)
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, flags=L.CCE_FILTER_DC)
    assert torch.equal(dC1, dC0) and torch.equal(dE1, dEf)
    assert torch.equal(dE2, dE0) and torch.equal(dC2, dCf)


@pytest.mark.parametrize("name,N,D,V,kw", [MID[0], MID[3], ("stress_peaked", 700, 128, 5000, {})])
def test_vocabulary_sorting_changes_the_order_not_the_result(cce, name, N, D, V, kw):
    """Section 4.3 vocabulary sorting: the backward pass walks the vocabulary in mean-logit order."""
    w = make(name, N=N, D=D, V=V, **kw)
    E, C, t = to_device(w)
    _, lse = run_forward(w, E, C, t)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    _, _, rdE, rdC = oracle_all(w)
    # unfiltered: same gradients; dC rows are bitwise the same (their token sums do not depend on
    # the vocabulary order), dE differs only by fp32 summation order
    dE0, dC0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    dE1, dC1, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, flags=both | L.CCE_VOCAB_SORT)
    assert torch.equal(dC0, dC1)
    assert rel_fro(f64(dE1), rdE) <= TOL_GRAD and rel_fro(f64(dE1), f64(dE0)) <= 2e-3
    # narrow slabs with sorting (many gathers, ragged last slab)
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, flags=both | L.CCE_VOCAB_SORT, op=L.CCE_OP_BACKWARD_MIN)
    assert torch.equal(dC0, dC2) and rel_fro(f64(dE2), rdE) <= TOL_GRAD
    # filtered: still within tolerance of the exact gradient and of the element-wise filter bound
    dEf, dCf, st_plain = run_backward(w, E, C, t, lse, dloss)
    dEs, dCs, st_sort = run_backward(w, E, C, t, lse, dloss, flags=both | L.CCE_VOCAB_SORT)
    _, _, fdE, fdC = oracle_all(w, eps=O.FILTER_EPS_BF16, mode="element")
    eE, eC = rel_fro(f64(dEs), rdE), rel_fro(f64(dCs), rdC)
    print("sorted filter %s: dE err %.2e dC err %.2e; blocks kept %d / %d sorted, %d / %d unsorted"
          % (name, eE, eC, st_sort[1], st_sort[0], st_plain[1], st_plain[0]))
    assert eE <= rel_fro(fdE, rdE) + rel_fro(f64(dE0), rdE) + 1e-3
    assert eC <= rel_fro(fdC, rdC) + rel_fro(f64(dC0), rdC) + 1e-3
    assert st_sort[0] == st_plain[0] and 0 < st_sort[1] <= st_sort[0]
    # the plain-FMA path has no sorted walk
    o = L.make_opts(L.CCE_BF16, flags=L.CCE_VOCAB_SORT | L.CCE_PLAIN_KERNELS, workspace=workspace(1 << 26))
    with pytest.raises(L.CceError) as ei:
        L.cce_backward_ex(E, C, t, lse, dloss, w.softcap, w.ignore_index, o)
    assert ei.value.status == -3


@pytest.mark.parametrize("name,N,D,V,kw", [MID[0], ("gemma2_2b", 1100, 128, 9000, {}), ("small_vocab", 520, 64, 4100, {}),
                                           ("stress_peaked", 700, 128, 5000, {})])
def test_skipping_tiles_the_filter_drops_changes_nothing(cce, name, N, D, V, kw):
    """CCE_SKIP_TILES: tiles whose recorded logit maxima rule out any entry >= eps are not recomputed."""
    w = make(name, N=N, D=D, V=V, **kw)
    E, C, t = to_device(w)
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    bm = torch.full((L.cce_block_max_bytes(w.N, w.V),), 0x7f, dtype=torch.uint8, device="cuda")   # poison: large positive
    loss0, lse0 = run_forward(w, E, C, t)
    loss1, lse1 = run_forward(w, E, C, t, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(loss0, loss1) and torch.equal(lse0, lse1)     # recording does not touch the result
    # the record is an upper bound, within bf16 rounding, of the oracle's block maxima
    A = O.logits(w.E64(), w.C64(), w.softcap)
    nb = (w.V + 127) // 128
    stride = (w.N + 255) // 256 * 256
    rec = bm.view(torch.int16).view(nb, stride)[:, :w.N].to(torch.int32).cpu().numpy().astype(np.uint32) << 16
    rec = rec.view(np.float32).astype(np.float64).T                   # [N, nb]
    ref = np.stack([A[:, b * 128:(b + 1) * 128].max(axis=1) for b in range(nb)], axis=1)
    assert np.all(rec >= ref - 1e-3) and np.all(rec <= ref + np.abs(ref) * 2.0 ** -7 + 2e-3)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE0, dC0, st0 = run_backward(w, E, C, t, lse0, dloss)
    dE1, dC1, st1 = run_backward(w, E, C, t, lse0, dloss, flags=both | L.CCE_SKIP_TILES, block_max=bm)
    print("skip tiles %s: blocks kept %d / %d" % (name, st1[1], st1[0]))
    assert torch.equal(dE0, dE1) and torch.equal(dC0, dC1) and st0 == st1
    # narrow slabs, and filter off for one product (the lists must then not be used)
    dE2, dC2, _ = run_backward(w, E, C, t, lse0, dloss, flags=both | L.CCE_SKIP_TILES, block_max=bm,
                               op=L.CCE_OP_BACKWARD_MIN)
    dE2r, dC2r, _ = run_backward(w, E, C, t, lse0, dloss, op=L.CCE_OP_BACKWARD_MIN)
    assert torch.equal(dE2r, dE2) and torch.equal(dC2r, dC2)
    dE3, dC3, _ = run_backward(w, E, C, t, lse0, dloss, flags=L.CCE_FILTER_DE)
    dE4, dC4, _ = run_backward(w, E, C, t, lse0, dloss, flags=L.CCE_FILTER_DE | L.CCE_SKIP_TILES, block_max=bm)
    assert torch.equal(dE3, dE4) and torch.equal(dC3, dC4)
    # an undersized record is refused
    o = L.make_opts(L.CCE_BF16, flags=both | L.CCE_SKIP_TILES, workspace=workspace(1 << 24), block_max=bm[:256])
    with pytest.raises(L.CceError) as ei:
        L.cce_forward_ex(E, C, t, w.softcap, w.ignore_index, o)
    assert ei.value.status == -2


@pytest.mark.parametrize("frac", [0.0, 0.02, 0.6, 1.0])
def test_removing_ignored_tokens_changes_nothing_but_the_cost(cce, frac):
    """CCE_COMPACT_IGNORED (Appendix B): the kernels run on the valid tokens only."""
    w = make("gemma2_2b", N=1100, D=128, V=3000, ignore_frac=frac)
    E, C, t = to_device(w)
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    cmp_ = L.CCE_COMPACT_IGNORED
    valid = torch.from_numpy(w.targets != w.ignore_index).cuda()
    loss0, lse0 = run_forward(w, E, C, t)
    loss1, lse1 = run_forward(w, E, C, t, flags=both | cmp_)
    assert torch.equal(loss0, loss1)                                  # a token's LSE does not depend on its neighbours
    assert torch.equal(lse0[valid], lse1[valid])
    ref_loss, ref_lse, rdE, rdC = oracle_all(w)
    assert max_rel(f64(loss1), ref_loss) <= TOL_LOSS
    rng = np.random.default_rng(3)
    lam = (rng.standard_normal(w.N) * 0.01 + 1.0 / w.N).astype(np.float32)
    rdE, rdC = O.backward(w.E64(), w.C64(), w.targets, ref_lse, lam.astype(np.float64), w.softcap, w.ignore_index)
    lam[w.targets == w.ignore_index] = np.nan                          # must not be read
    dloss = torch.from_numpy(lam).cuda()
    for eps in (0.0, None):
        dE0, dC0, st0 = run_backward(w, E, C, t, lse0, dloss, eps=eps)
        dE1, dC1, st1 = run_backward(w, E, C, t, lse1, dloss, eps=eps, flags=both | cmp_)
        # rows of dE are per token; the contraction over a slab is cut into parts planned for the tokens
        # present, so the fp32 sums may be taken in another order
        assert rel_fro(f64(dE1), f64(dE0)) <= 2e-3 and max_row_err(f64(dE1), f64(dE0)) <= 4e-3
        assert torch.all(dE1[~valid] == 0)
        if frac < 1.0:
            assert rel_fro(f64(dC1), f64(dC0)) <= 2e-3                # other token order in the sums over tokens
            if eps == 0.0:
                assert rel_fro(f64(dE1), rdE) <= TOL_GRAD and rel_fro(f64(dC1), rdC) <= TOL_GRAD
        else:
            assert torch.all(dC1 == 0) and torch.all(dE1 == 0)
    # together with tile skipping, vocabulary sorting and narrow slabs
    bm = torch.empty(L.cce_block_max_bytes(w.N, w.V), dtype=torch.uint8, device="cuda")
    fl = both | cmp_ | L.CCE_SKIP_TILES
    loss2, lse2 = run_forward(w, E, C, t, flags=fl, block_max=bm)
    assert torch.equal(loss2, loss1)
    dE2, dC2, _ = run_backward(w, E, C, t, lse2, dloss, flags=fl, block_max=bm)
    dE3, dC3, _ = run_backward(w, E, C, t, lse1, dloss, flags=both | cmp_)
    assert torch.equal(dE2, dE3) and torch.equal(dC2, dC3)
    dE4, dC4, _ = run_backward(w, E, C, t, lse1, dloss, eps=0.0, flags=both | cmp_ | L.CCE_VOCAB_SORT,
                               op=L.CCE_OP_BACKWARD_MIN)
    dE5, dC5, _ = run_backward(w, E, C, t, lse1, dloss, eps=0.0, flags=both | cmp_)
    assert torch.equal(dC4, dC5) and rel_fro(f64(dE4), f64(dE5)) <= 2e-3


@pytest.mark.parametrize("name,N,D,V", [("small_vocab", 5120, 2304, 4000), ("gemma2_2b", 300, 192, 5000)])
def test_accumulation_precision_variants(cce, name, N, D, V):
    """Section 5 ("CCE" vs "CCE-Kahan"): dE's running sum over vocabulary slabs kept in bf16, with and
    without Kahan compensation, against the exact gradient and against the oracle's model of that sum."""
    w = make(name, N=N, D=D, V=V)
    E, C, t = to_device(w)
    _, lse = run_forward(w, E, C, t)
    lam = w.mean_dloss()
    dloss = torch.from_numpy(lam).cuda()
    both = L.CCE_FILTER_DE | L.CCE_FILTER_DC
    mn = L.CCE_OP_BACKWARD_MIN                                   # 256-wide slabs: as many roundings as possible
    slabs = (V + 255) // 256
    E64, C64 = w.E64(), w.C64()
    _, ref_lse = O.forward(E64, C64, w.targets, w.softcap, w.ignore_index)
    rdE, rdC = O.backward(E64, C64, w.targets, ref_lse, lam.astype(np.float64), w.softcap, w.ignore_index)
    dE0, dC0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=mn)
    dE1, dC1, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=mn, flags=both | L.CCE_ACCUM_BF16)
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=mn, flags=both | L.CCE_ACCUM_KAHAN)
    assert torch.equal(dC0, dC1) and torch.equal(dC0, dC2)       # dC has no sum in device memory
    e0, e1, e2 = (rel_fro(f64(x), rdE) for x in (dE0, dE1, dE2))
    m1 = O.backward_dE_slab_accumulated(E64, C64, w.targets, ref_lse, lam, 256, "bf16", w.softcap, w.ignore_index)
    m2 = O.backward_dE_slab_accumulated(E64, C64, w.targets, ref_lse, lam, 256, "kahan", w.softcap, w.ignore_index)
    o1, o2 = rel_fro(m1, rdE), rel_fro(m2, rdE)
    print("accumulation %s, %d slabs: fp32 %.2e | bf16 %.2e (oracle model %.2e) | bf16 + Kahan %.2e (oracle model %.2e)"
          % (name, slabs, e0, e1, o1, e2, o2))
    # compensation brings the bf16 sum back to the fp32 accumulator's level; without it the error grows
    assert e2 <= TOL_GRAD and e2 <= 1.5 * e0 + 1e-3
    assert e1 > 1.5 * e2
    if N * D >= 171 * 65536:
        # Enough (token tile, D tile) pairs that every slab is one contraction (small batches cut it into parts
        # with a running sum each): the kernels then reproduce the modelled sums, up to the rounding decisions
        # that the bf16 rounding of GZ moves.
        assert 0.6 * o1 <= e1 <= 1.6 * o1 + 1e-3
        assert rel_fro(f64(dE1), m1) <= 2.0 * o1 + 3e-3 and rel_fro(f64(dE2), m2) <= TOL_GRAD
    # one slab: one rounding of every sum either way
    w1 = make(name, N=N, D=D, V=256)
    E1, C1, t1 = to_device(w1)
    _, lse1 = run_forward(w1, E1, C1, t1)
    a, _, _ = run_backward(w1, E1, C1, t1, lse1, dloss, eps=0.0)
    b, _, _ = run_backward(w1, E1, C1, t1, lse1, dloss, eps=0.0, flags=both | L.CCE_ACCUM_BF16)
    c, _, _ = run_backward(w1, E1, C1, t1, lse1, dloss, eps=0.0, flags=both | L.CCE_ACCUM_KAHAN)
    if N * D >= 171 * 65536:
        assert torch.equal(a, b) and torch.equal(a, c)
    else:
        assert rel_fro(f64(b), f64(a)) <= 5e-3 and rel_fro(f64(c), f64(a)) <= 5e-3
    # together with removing ignored tokens, filtering, and on the plain path (refused)
    d0, _, _ = run_backward(w, E, C, t, lse, dloss, op=mn, flags=both | L.CCE_ACCUM_KAHAN | L.CCE_COMPACT_IGNORED)
    d1, _, _ = run_backward(w, E, C, t, lse, dloss, op=mn, flags=both | L.CCE_ACCUM_KAHAN)
    assert rel_fro(f64(d0), f64(d1)) <= 4e-3
    o = L.make_opts(L.CCE_BF16, flags=L.CCE_ACCUM_BF16 | L.CCE_PLAIN_KERNELS, workspace=workspace(1 << 26))
    with pytest.raises(L.CceError) as ei:
        L.cce_backward_ex(E, C, t, lse, dloss, w.softcap, w.ignore_index, o)
    assert ei.value.status == -3


def test_tiny_config_fp32_full_parity(cce):
    """Config 1 (N=256, D=64, V=1024, fp32, 5% ignored): the oracle covers every output."""
    w = make("tiny")
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    ref_loss, ref_lse, rdE, rdC = oracle_all(w)
    assert max_rel(f64(lse), ref_lse) <= 1e-5 and max_rel(f64(loss), ref_loss) <= 1e-5
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss)
    eE, eC = rel_fro(f64(dE), rdE), rel_fro(f64(dC), rdC)
    print("tiny fp32: lse %.2e dE %.2e dC %.2e" % (max_rel(f64(lse), ref_lse), eE, eC))
    assert eE <= 1e-4 and eC <= 1e-4
    assert max_row_err(f64(dE), rdE) <= 1e-4 and max_row_err(f64(dC), rdC) <= 1e-4
    # narrowest slab (many slabs) gives the same answer
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, op=L.CCE_OP_BACKWARD_MIN)
    assert rel_fro(f64(dE2), rdE) <= 1e-4 and rel_fro(f64(dC2), rdC) <= 1e-4


@pytest.mark.parametrize("name,N,D,V", [("gemma2_2b", 300, 128, 700), ("small_vocab", 130, 72, 333)])
def test_plain_kernels_on_bf16_match_oracle(cce, name, N, D, V):
    """The plain-FMA path (also taken when D is not a multiple of 64) on bf16 storage."""
    w = make(name, N=N, D=D, V=V)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t, flags=L.CCE_PLAIN_KERNELS)
    ref_loss, ref_lse, rdE, rdC = oracle_all(w)
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss, flags=L.CCE_PLAIN_KERNELS, eps=0.0)
    assert rel_fro(f64(dE), rdE) <= TOL_GRAD and rel_fro(f64(dC), rdC) <= TOL_GRAD


def test_narrow_slabs_and_small_workspace(cce):
    """Many vocabulary slabs (minimum workspace) must give the same gradients as one wide slab."""
    w = make("small_vocab", N=300, D=128, V=1300)
    E, C, t = to_device(w)
    _, lse = run_forward(w, E, C, t)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=L.CCE_OP_BACKWARD_MIN)
    _, _, rdE, rdC = oracle_all(w)
    assert rel_fro(f64(dE2), rdE) <= TOL_GRAD and rel_fro(f64(dC2), rdC) <= TOL_GRAD
    assert torch.equal(dC, dC2)       # dC rows are final within their slab: identical whatever the slab width
    # the same kernels in plain sequence on the caller's stream give the same bits
    dE3, dC3, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0,
                               flags=L.CCE_FILTER_DE | L.CCE_FILTER_DC | L.CCE_SINGLE_STREAM)
    assert torch.equal(dE, dE3) and torch.equal(dC, dC3)
    o = L.make_opts(L.CCE_BF16, workspace=workspace(4096))
    with pytest.raises(L.CceError) as ei:
        L.cce_backward_ex(E, C, t, lse, dloss, 0.0, w.ignore_index, o)
    assert ei.value.status == -2


def test_wide_slabs_with_a_larger_workspace(cce):
    """A workspace of CCE_OP_BACKWARD_WIDE bytes gives fewer, wider slabs and the same gradients."""
    w = make("gemma2_2b", N=4400, D=64, V=30000)
    o = L.make_opts(L.CCE_BF16)
    rec = L.cce_workspace_bytes(L.CCE_OP_BACKWARD, w.N, w.D, w.V, o)
    wide = L.cce_workspace_bytes(L.CCE_OP_BACKWARD_WIDE, w.N, w.D, w.V, o)
    assert wide > 2 * rec
    E, C, t = to_device(w)
    _, lse = run_forward(w, E, C, t)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    _, _, rdE, rdC = oracle_all(w)
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    dE2, dC2, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, op=L.CCE_OP_BACKWARD_WIDE)
    assert rel_fro(f64(dE2), rdE) <= TOL_GRAD and rel_fro(f64(dC2), rdC) <= TOL_GRAD
    assert torch.equal(dC, dC2)
    # more than the widest slab needs is accepted and changes nothing further
    dE3, dC3, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0, ws_bytes=wide + (64 << 20))
    assert torch.equal(dE2, dE3) and torch.equal(dC2, dC3)
    # filtered: the same blocks are kept whatever the slab width
    dEf, dCf, st = run_backward(w, E, C, t, lse, dloss)
    dEf2, dCf2, st2 = run_backward(w, E, C, t, lse, dloss, op=L.CCE_OP_BACKWARD_WIDE)
    assert st == st2 and torch.equal(dCf, dCf2)
    assert rel_fro(f64(dEf2), f64(dEf)) <= 1e-2


def test_edge_cases(cce):
    # all tokens ignored: loss 0, gradients 0
    w = make("gemma2_2b", N=260, D=64, V=300, ignore_frac=1.0)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    assert torch.all(loss == 0) and torch.all(torch.isfinite(lse))
    dloss = torch.full((w.N,), float("nan"), device="cuda")
    dE, dC, _ = run_backward(w, E, C, t, lse, dloss)
    assert torch.all(dE == 0) and torch.all(dC == 0)
    # single token, single-tile vocabulary, out-of-range target treated as ignored
    w = make("small_vocab", N=3, D=64, V=5, ignore_frac=0.0)
    w.targets[1] = 99
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    ref_loss, ref_lse = O.forward(w.E64(), w.C64(), w.targets, 0.0, w.ignore_index)
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS
    assert float(loss[1]) == 0.0
    # V = 1: loss exactly 0 for valid tokens
    w = make("small_vocab", N=70, D=64, V=1, ignore_frac=0.0)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    assert float(loss.abs().max()) <= 1e-3
    # C = 0: LSE = loss = log V (closed form), on device
    w = make("small_vocab", N=300, D=128, V=1000, ignore_frac=0.0)
    E, C, t = to_device(w)
    C.zero_()
    loss, lse = run_forward(w, E, C, t)
    assert float((lse - np.log(1000)).abs().max()) <= 1e-4 and float((loss - np.log(1000)).abs().max()) <= 1e-4


def test_large_logits_without_cap_do_not_overflow(cce):
    w = make("small_vocab", N=300, D=128, V=900, ignore_frac=0.0)
    from workloads import f32_to_bf16_bits
    w.C[:] = f32_to_bf16_bits((w.C64() * 400).astype(np.float32))
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    ref_loss, ref_lse = O.forward(w.E64(), w.C64(), w.targets, 0.0, w.ignore_index)
    assert np.abs(ref_lse).max() > 100          # the test really has large logits
    assert torch.all(torch.isfinite(lse))
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS


def test_results_are_bitwise_reproducible(cce):
    w = make("gemma2_2b", N=700, D=128, V=3000)
    E, C, t = to_device(w)
    loss1, lse1 = run_forward(w, E, C, t)
    loss2, lse2 = run_forward(w, E, C, t)
    assert torch.equal(loss1, loss2) and torch.equal(lse1, lse2)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    a = run_backward(w, E, C, t, lse1, dloss)
    b = run_backward(w, E, C, t, lse1, dloss)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and a[2] == b[2]


def test_plain_entry_points_draw_on_the_lent_workspace(cce):
    """cce_forward / cce_backward (the plain signatures, without options) allocate nothing: their scratch is the
    buffer registered with cce_set_workspace, and without one they refuse."""
    w = make("gemma2_2b", N=300, D=128, V=1000)
    E, C, t = to_device(w)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    L.cce_set_workspace(None)
    with pytest.raises(L.CceError) as ei:
        L.cce_forward(E, C, t, w.softcap, w.ignore_index)
    assert ei.value.status == -2
    o = L.make_opts(L.CCE_BF16)
    small = workspace(L.cce_workspace_bytes(L.CCE_OP_FORWARD, w.N, w.D, w.V, o))
    L.cce_set_workspace(small)
    loss, lse = L.cce_forward(E, C, t, w.softcap, w.ignore_index)
    with pytest.raises(L.CceError) as ei:                    # enough for the forward, not for the backward
        L.cce_backward(E, C, t, lse, dloss, w.softcap, w.ignore_index)
    assert ei.value.status == -2
    lent = workspace(L.cce_workspace_bytes(L.CCE_OP_BACKWARD, w.N, w.D, w.V, o))
    L.cce_set_workspace(lent)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    dE, dC = torch.empty_like(E), torch.empty_like(C)
    L.cce_forward(E, C, t, w.softcap, w.ignore_index, out_loss=loss, out_lse=lse)
    L.cce_backward(E, C, t, lse, dloss, w.softcap, w.ignore_index, out_dE=dE, out_dC=dC)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0             # the library allocated nothing on the device
    ref_loss, ref_lse, rdE, rdC = oracle_all(w)
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS
    assert rel_fro(f64(dE), rdE) <= TOL_GRAD and rel_fro(f64(dC), rdC) <= TOL_GRAD
    total, kept = L.cce_backward_filter_stats()
    assert total > 0
    L.cce_set_workspace(None)


@pytest.mark.parametrize("flags", [None, "compact", "plain"])
def test_out_of_range_targets_are_ignored_and_counted(cce, flags):
    w = make("small_vocab", N=700, D=128, V=900, ignore_frac=0.1)
    bad = [3, 255, 256, 699]
    w.targets[bad] = [900, -1, 1 << 40, -101]                 # none equals ignore_index (-100)
    E, C, t = to_device(w)
    fl = {None: None, "compact": L.CCE_FILTER_DE | L.CCE_FILTER_DC | L.CCE_COMPACT_IGNORED,
          "plain": L.CCE_PLAIN_KERNELS}[flags]
    o = L.make_opts(L.CCE_BF16, flags=fl)
    ws = workspace(L.cce_workspace_bytes(L.CCE_OP_FORWARD, w.N, w.D, w.V, o))
    o = L.make_opts(L.CCE_BF16, flags=fl, workspace=ws)
    for expect in (4, 4, 0):                                  # the counter is per call, not cumulative
        if expect == 0:
            t[torch.tensor(bad).cuda()] = w.ignore_index
            w.targets[bad] = w.ignore_index
        loss, lse = L.cce_forward_ex(E, C, t, w.softcap, w.ignore_index, o)
        assert L.cce_forward_target_stats(ws) == expect
        ref_loss, _ = O.forward(w.E64(), w.C64(), w.targets, w.softcap, w.ignore_index)
        assert max_rel(f64(loss), ref_loss) <= TOL_LOSS and torch.all(loss[torch.tensor(bad).cuda()] == 0)


def test_calls_on_a_side_stream_and_under_graph_capture(cce):
    """The entry points take any stream and can be captured into a HIP graph: the helper streams of
    the backward pass fork from and join back into the capturing stream, nothing is allocated and
    no memset node is recorded.  Every replay is checked against the eager result."""
    w = make("gemma2_2b", N=600, D=128, V=7000)
    E, C, t = to_device(w)
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    o0 = L.make_opts(L.CCE_BF16)
    ws_f = workspace(L.cce_workspace_bytes(L.CCE_OP_FORWARD, w.N, w.D, w.V, o0))
    ws_b = workspace(L.cce_workspace_bytes(L.CCE_OP_BACKWARD, w.N, w.D, w.V, o0))
    loss, lse = torch.empty(w.N, device="cuda"), torch.empty(w.N, device="cuda")
    dE, dC = torch.empty_like(E), torch.empty_like(C)

    def step(stream):
        of = L.make_opts(L.CCE_BF16, workspace=ws_f, stream=stream.cuda_stream)
        ob = L.make_opts(L.CCE_BF16, workspace=ws_b, stream=stream.cuda_stream)
        L.cce_forward_ex(E, C, t, w.softcap, w.ignore_index, of, out_loss=loss, out_lse=lse)
        L.cce_backward_ex(E, C, t, lse, dloss, w.softcap, w.ignore_index, ob, out_dE=dE, out_dC=dC)

    def eager():
        step(torch.cuda.current_stream())
        torch.cuda.synchronize()
        return loss.clone(), dE.clone(), dC.clone()

    ref0 = eager()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    step(side)
    side.synchronize()
    assert torch.equal(loss, ref0[0]) and torch.equal(dE, ref0[1]) and torch.equal(dC, ref0[2])

    g = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=cap):
        step(cap)
    E_orig = E.clone()
    for k in range(3):
        E.copy_(E_orig.roll(k + 1, 0))             # new inputs for every replay
        ref = eager()
        loss.zero_(); dE.zero_(); dC.zero_()       # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss, ref[0]) and torch.equal(dE, ref[1]) and torch.equal(dC, ref[2]), "replay %d" % k


def test_more_tokens_than_a_filtered_dC_contraction_can_list(cce):
    """N > 131072: the dC product's contraction over tokens is longer than the list of kept steps it keeps in LDS,
    so it runs unfiltered whatever CCE_FILTER_DC says (documented); everything stays within the tolerances."""
    w = make("stress_peaked", N=131072 + 256 + 5, D=64, V=700)
    E, C, t = to_device(w)
    loss, lse = run_forward(w, E, C, t)
    ref_loss, ref_lse, rdE, rdC = oracle_all(w)
    assert max_rel(f64(lse), ref_lse) <= TOL_LOSS and max_rel(f64(loss), ref_loss) <= TOL_LOSS
    dloss = torch.from_numpy(w.mean_dloss()).cuda()
    dE0, dC0, _ = run_backward(w, E, C, t, lse, dloss, eps=0.0)
    assert rel_fro(f64(dE0), rdE) <= TOL_GRAD and rel_fro(f64(dC0), rdC) <= TOL_GRAD
    assert max_row_err(f64(dE0), rdE) <= TOL_ROW and max_row_err(f64(dC0), rdC) <= TOL_ROW
    dE1, dC1, st = run_backward(w, E, C, t, lse, dloss)                 # filters on: dC comes out as without
    assert torch.equal(dC1, dC0) and 0 < st[1] <= st[0]
    _, _, fdE, _ = oracle_all(w, eps=O.FILTER_EPS_BF16, mode="element")
    assert rel_fro(f64(dE1), rdE) <= rel_fro(fdE, rdE) + rel_fro(f64(dE0), rdE) + 1e-3


def test_largest_sizes_forward_works_and_backward_refuses_cleanly(cce):
    """E of 4 GiB and more: the forward addresses it with 64-bit offsets; the MFMA backward, whose gradient
    products use 32-bit byte offsets into E, refuses with CCE_EUNSUPPORTED before launching anything."""
    N, D, V = (1 << 25) + 300, 64, 300                                  # N * D * 2 bytes = 4 GiB + 38 KB
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    E = torch.randn(N, D, device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    C = (torch.randn(V, D, device="cuda", generator=g, dtype=torch.float32) * 0.3).to(torch.bfloat16)
    t = torch.randint(0, V, (N,), device="cuda", generator=g)
    o = L.make_opts(L.CCE_BF16)
    ws = workspace(L.cce_workspace_bytes(L.CCE_OP_FORWARD, N, D, V, o))
    o = L.make_opts(L.CCE_BF16, workspace=ws)
    loss, lse = L.cce_forward_ex(E, C, t, 0.0, -100, o)
    torch.cuda.synchronize()
    # the oracle on sampled tokens, among them the first and the last ones and both sides of the 4 GiB line
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(N - 300, N), np.arange((1 << 25) - 150, (1 << 25) + 150),
                                     np.random.default_rng(6).integers(0, N, 2000)]))
    idx = torch.from_numpy(rows).cuda()
    E_s = E[idx].float().cpu().numpy().astype(np.float64)
    r_loss, r_lse = O.forward(E_s, C.float().cpu().numpy().astype(np.float64), t[idx].cpu().numpy(), 0.0, -100)
    assert max_rel(f64(lse[idx]), r_lse) <= TOL_LOSS and max_rel(f64(loss[idx]), r_loss) <= TOL_LOSS
    assert bool(torch.isfinite(lse).all())
    wb = workspace(1 << 20)
    ob = L.make_opts(L.CCE_BF16, workspace=wb)
    dE = torch.full((4096,), 7.0, device="cuda")                        # stand-ins: nothing may be written
    import ctypes
    with pytest.raises(L.CceError) as ei:        # (straight through ctypes: the binding's wrapper would check the outputs' shapes)
        st = L.load().cce_backward_ex(E.data_ptr(), C.data_ptr(), t.data_ptr(), N, D, V, 0.0, -100, lse.data_ptr(),
                                      loss.data_ptr(), dE.data_ptr(), dE.data_ptr(), ctypes.byref(ob))
        if st != 0:
            raise L.CceError(st, L.cce_strerror(st))
    assert ei.value.status == -3
    torch.cuda.synchronize()
    assert bool((dE == 7.0).all())
