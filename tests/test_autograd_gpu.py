"""torch.autograd front end (linear_cross_entropy) against the fp64 oracle.

The wrapper adds nothing to the arithmetic: the loss comes from cce_forward_ex, the gradients
from cce_backward_ex with the upstream gradient autograd hands over.  Tolerances as in
test_parity_gpu.py.
"""
import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from oracle import cce_oracle as O
from workloads import make

from gpu_util import f64, max_rel, rel_fro, to_device

pytestmark = pytest.mark.gpu

TOL_LOSS = 1e-3
TOL_GRAD = 1e-2


def oracle(w, dloss):
    E, C = w.E64(), w.C64()
    loss, lse = O.forward(E, C, w.targets, w.softcap, w.ignore_index)
    dE, dC = O.backward(E, C, w.targets, lse, np.asarray(dloss, dtype=np.float64), w.softcap, w.ignore_index)
    return loss, lse, dE, dC


@pytest.mark.parametrize("kw", [{}, {"skip_tiles": True}, {"compact_ignored": True, "wide_workspace": True},
                                {"vocab_sort": True}])
def test_mean_reduction_matches_oracle(cce, kw):
    w = make("gemma2_2b", N=600, D=128, V=1500)
    E, C, t = to_device(w)
    e = E.clone().requires_grad_(True)
    c = C.clone().requires_grad_(True)
    loss = L.linear_cross_entropy(e, c, t, softcap=w.softcap, ignore_index=w.ignore_index, filter_eps=0.0, **kw)
    loss.backward()
    torch.cuda.synchronize()
    n_valid = int((w.targets != w.ignore_index).sum())
    r_loss, _, r_dE, r_dC = oracle(w, w.mean_dloss())
    assert abs(float(loss.detach()) - r_loss.sum() / n_valid) <= TOL_LOSS * max(1.0, abs(r_loss.sum() / n_valid))
    assert rel_fro(f64(e.grad), r_dE) <= TOL_GRAD and rel_fro(f64(c.grad), r_dC) <= TOL_GRAD
    assert e.grad.dtype == torch.bfloat16 and c.grad.shape == C.shape


def test_per_token_loss_with_arbitrary_upstream_gradient_and_batch_shape(cce):
    w = make("small_vocab", N=512, D=64, V=700)
    E, C, t = to_device(w)
    e = E.view(4, 128, 64).clone().requires_grad_(True)      # [batch, sequence, D]
    c = C.clone().requires_grad_(True)
    rng = np.random.default_rng(5)
    up = rng.standard_normal(w.N) / w.N
    loss, lse = L.linear_cross_entropy(e, c, t.view(4, 128), softcap=w.softcap, ignore_index=w.ignore_index,
                                       reduction="none", filter_eps=0.0, return_lse=True)
    assert loss.shape == (4, 128) and lse.shape == (4, 128) and not lse.requires_grad
    (loss * torch.from_numpy(up.astype(np.float32)).cuda().view(4, 128)).sum().backward()
    torch.cuda.synchronize()
    up32 = up.astype(np.float32).astype(np.float64)
    r_loss, r_lse, r_dE, r_dC = oracle(w, up32)
    assert max_rel(f64(loss).reshape(-1), r_loss) <= TOL_LOSS and max_rel(f64(lse).reshape(-1), r_lse) <= TOL_LOSS
    assert rel_fro(f64(e.grad).reshape(w.N, w.D), r_dE) <= TOL_GRAD and rel_fro(f64(c.grad), r_dC) <= TOL_GRAD


def test_float32_inputs_take_the_plain_kernels(cce):
    w = make("tiny")
    E, C, t = to_device(w)
    e = E.clone().requires_grad_(True)
    c = C.clone().requires_grad_(True)
    loss = L.linear_cross_entropy(e, c, t, ignore_index=w.ignore_index, reduction="sum")
    loss.backward()
    torch.cuda.synchronize()
    r_loss, _, r_dE, r_dC = oracle(w, np.ones(w.N))
    assert abs(float(loss.detach()) - r_loss.sum()) <= 1e-5 * abs(r_loss.sum())
    assert rel_fro(f64(e.grad), r_dE) <= 1e-4 and rel_fro(f64(c.grad), r_dC) <= 1e-4
