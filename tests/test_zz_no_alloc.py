"""cce_forward_noalloc: the forward on the library's static scratch array, for callers that
cannot allocate.  Called through the C ABI and compared with cce_forward_ex (same kernels:
bit-identical) and with the fp64 oracle (loss / LSE max relative error <= 1e-3), on two calls
in a row, the second with a smaller input, so that what the first call left in the array
would show if it were ever read."""
import numpy as np
import pytest
import torch

import paper_2411_09009_amd as L
from oracle import cce_oracle as O
from workloads import make

from gpu_util import f64, max_rel, run_forward, to_device

pytestmark = pytest.mark.gpu


def test_forward_on_static_scratch_matches_forward_ex_twice(cce):
    assert L.cce_noalloc_scratch_bytes() == 8 << 20
    for call, (name, N, D, V) in enumerate((("gemma2_2b", 1300, 128, 5000), ("small_vocab", 300, 64, 700))):
        w = make(name, N=N, D=D, V=V)
        E, C, t = to_device(w)
        ref_loss, ref_lse = run_forward(w, E, C, t)
        loss = torch.full((N,), float("nan"), device="cuda")
        lse = torch.full((N,), float("nan"), device="cuda")
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        o = L.make_opts(L.CCE_BF16)
        L.cce_forward_noalloc(E, C, t, w.softcap, w.ignore_index, o, loss, lse)
        torch.cuda.synchronize()
        if call > 0:     # (the first call on a device may make the runtime load the library's code object)
            assert torch.cuda.mem_get_info()[0] == free0        # nothing was allocated on the device
        assert torch.equal(loss, ref_loss) and torch.equal(lse, ref_lse)
        o_loss, o_lse = O.forward(w.E64(), w.C64(), w.targets, w.softcap, w.ignore_index)
        assert max_rel(f64(lse), o_lse) <= 1e-3 and max_rel(f64(loss), o_loss) <= 1e-3


def test_problem_beyond_the_static_scratch_is_refused(cce):
    w = make("small_vocab", N=300, D=64, V=700)
    E, C, t = to_device(w)
    loss, lse = torch.zeros(300, device="cuda"), torch.zeros(300, device="cuda")
    # a compacted copy of E of 9 MiB cannot live in the 8 MiB array; nothing may be launched or written
    wb = make("small_vocab", N=36864, D=128, V=300)
    Eb, Cb, tb = to_device(wb)
    lb, sb = torch.full((wb.N,), 7.0, device="cuda"), torch.full((wb.N,), 7.0, device="cuda")
    o = L.make_opts(L.CCE_BF16, flags=L.CCE_FILTER_DE | L.CCE_FILTER_DC | L.CCE_COMPACT_IGNORED)
    with pytest.raises(L.CceError) as ei:
        L.cce_forward_noalloc(Eb, Cb, tb, 0.0, wb.ignore_index, o, lb, sb)
    assert ei.value.status == -5 and "8388608" in str(ei.value)
    torch.cuda.synchronize()
    assert torch.all(lb == 7.0) and torch.all(sb == 7.0)
    # the array still serves the next call
    ref_loss, ref_lse = run_forward(w, E, C, t)
    L.cce_forward_noalloc(E, C, t, 0.0, w.ignore_index, L.make_opts(L.CCE_BF16), loss, lse)
    torch.cuda.synchronize()
    assert torch.equal(loss, ref_loss) and torch.equal(lse, ref_lse)


def test_forward_on_static_scratch_under_graph_capture(cce):
    """The call allocates nothing and records no memset, so it can be captured into a HIP graph; every replay
    (new inputs, eager work and a synchronisation in between) is checked against the eager result."""
    w = make("gemma2_2b", N=900, D=128, V=4000)
    E, C, t = to_device(w)
    loss = torch.empty(w.N, device="cuda")
    lse = torch.empty(w.N, device="cuda")
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        o = L.make_opts(L.CCE_BF16, stream=cap.cuda_stream)
        L.cce_forward_noalloc(E, C, t, w.softcap, w.ignore_index, o, loss, lse)
    E0 = E.clone()
    for k in range(3):
        E.copy_(E0.roll(k + 1, 0))
        ref_loss, ref_lse = run_forward(w, E, C, t)          # eager, through cce_forward_ex
        loss.zero_()
        lse.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss, ref_loss) and torch.equal(lse, ref_lse), "replay %d" % k
