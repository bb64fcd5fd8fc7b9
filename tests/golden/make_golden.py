"""Writes the stored oracle values for the full-size configurations.

Calls only oracle/ and the seeded input generator (never the HIP path):
    python tests/golden/make_golden.py [--reuse-forward] [config ...]
(--reuse-forward keeps lse / loss from an existing file of this script when the input
checksums still match, and only rewrites the sampled gradient rows.)
For each configuration it stores, in tests/golden/<config>.npz:
  lse, loss        float32 [N]   oracle forward on every token (computed in fp64; stored
                                 as float32, 6e-8 relative, far inside the 1e-3 tolerance)
  dE_rows, dE      int64 [r], float32 [r, D]   oracle dE for sampled tokens
  dC_rows, dC      int64 [r], float32 [r, D]   oracle dC for sampled vocabulary entries
  dE_f, dC_f       the same rows with the element-wise gradient filter at eps = 2^-12
                   (the finest granularity a block filter can be compared with)
  tok_rows, voc_rows, cols        the >= 1024 tokens / >= 1024 vocabulary entries / 16 columns of sampling.py
  dE_sub  float32 [tokens, 16]    oracle dE at (tok_rows, cols): sampled entries of >= 1024 rows, every token tile
  dC_sub  float32 [entries, 16]   oracle dC at (voc_rows, cols): every slab of every slab width holds several
  dE_norm, dC_norm  float64       Euclidean norm of each of those complete rows
                   (a complete row would be 9 - 20 KB; 2048 of them per configuration do not belong in a repository:
                   tests/test_full_size_gpu.py recomputes the complete rows with the oracle and checks them against
                   these entries and norms before it compares the kernels with them)
  (upstream gradient = 1 / N_valid for every valid token)
  e_sum, c_sum, t_sum            checksums of the generated inputs, so that a test can
                                 verify it regenerated bit-identical inputs.
The full forward costs 2*N*D*|V| fp64 flop (about 35 s / 60 s / 5 min for the Gemma-2-2B /
Llama-3-8B / stress shapes on 8 cores); the sampled rows of dE and dC are exact restrictions
of the full gradient (each dE row needs only its own token, each dC row only its own logit
column once the LSE of every token is known).
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import cce_oracle as O   # noqa: E402
from workloads import CONFIGS, make  # noqa: E402
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from sampling import sample_columns, sample_tokens, sample_vocab  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
FULL = ["small_vocab", "gemma2_2b", "llama3_8b", "stress", "stress_peaked", "gemma2_9b", "qwen25_7b", "gemma2_2b_n1024"]


def checksums(w):
    return (np.uint64(w.E.astype(np.uint64).sum()), np.uint64(w.C.astype(np.uint64).sum()),
            np.int64(w.targets.sum()))


def sample_rows(w):
    rng = np.random.default_rng(1000 + w.spec.seed)
    rows = {0, w.N - 1, w.N // 2 + 1}
    ign = np.nonzero(w.targets == w.ignore_index)[0]
    if len(ign):
        rows.add(int(ign[0]))
    while len(rows) < 16:
        rows.add(int(rng.integers(0, w.N)))
    valid_t = w.targets[w.targets != w.ignore_index]
    counts = np.bincount(valid_t, minlength=w.V)
    vrows = {0, w.V - 1, w.V - 257} | {int(v) for v in np.argsort(-counts)[:3]}
    if w.boosted is not None:
        vrows |= {int(w.boosted[0]), int(w.boosted[-1])}
    never = np.nonzero(counts == 0)[0]
    vrows.add(int(never[len(never) // 2]))
    while len(vrows) < 16:
        vrows.add(int(rng.integers(0, w.V)))
    return np.array(sorted(rows)), np.array(sorted(vrows))


def build(name, reuse_forward=False):
    t0 = time.time()
    w = make(name)
    print("%s: generated in %.1f s" % (name, time.time() - t0), flush=True)
    C64 = w.C64()
    t0 = time.time()
    path = os.path.join(HERE, name + ".npz")
    old = np.load(path) if reuse_forward and os.path.exists(path) else None
    if old is not None and (int(old["e_sum"]), int(old["c_sum"]), int(old["t_sum"])) == tuple(int(x) for x in checksums(w)):
        loss, lse = old["loss"].astype(np.float64), old["lse"].astype(np.float64)
        print("%s: forward reused from %s" % (name, path), flush=True)
    else:
        loss, lse = forward_chunked(w, C64)
        print("%s: forward oracle %.1f s" % (name, time.time() - t0), flush=True)
    rows, vrows = sample_rows(w)
    lam = w.mean_dloss().astype(np.float64)
    t0 = time.time()
    dE = O.backward_dE_rows(w.E64(rows), C64, w.targets[rows], lse[rows], lam[rows], np.arange(len(rows)),
                            w.softcap, w.ignore_index)
    E64 = w.E64()
    dC = O.backward_dC_rows(E64, C64, w.targets, lse, lam, vrows, w.softcap, w.ignore_index)
    eps = O.FILTER_EPS_BF16
    dE_f = O.backward_dE_rows(w.E64(rows), C64, w.targets[rows], lse[rows], lam[rows], np.arange(len(rows)),
                              w.softcap, w.ignore_index, eps=eps)
    dC_f = O.backward_dC_rows(E64, C64, w.targets, lse, lam, vrows, w.softcap, w.ignore_index, eps=eps)
    print("%s: sampled backward oracle %.1f s" % (name, time.time() - t0), flush=True)
    t0 = time.time()
    tok, voc, cols = sample_tokens(w), sample_vocab(w), sample_columns(w)
    wide_dE = O.backward_dE_rows(w.E64(tok), C64, w.targets[tok], lse[tok], lam[tok], np.arange(len(tok)),
                                 w.softcap, w.ignore_index)
    wide_dC = O.backward_dC_rows(E64, C64, w.targets, lse, lam, voc, w.softcap, w.ignore_index)
    print("%s: %d + %d sampled rows %.1f s" % (name, len(tok), len(voc), time.time() - t0), flush=True)
    es, cs, ts = checksums(w)
    np.savez_compressed(path, lse=lse.astype(np.float32), loss=loss.astype(np.float32),
                        dE_rows=rows, dE=dE.astype(np.float32), dC_rows=vrows, dC=dC.astype(np.float32),
                        dE_f=dE_f.astype(np.float32), dC_f=dC_f.astype(np.float32), e_sum=es, c_sum=cs, t_sum=ts, N=w.N, D=w.D, V=w.V,
                        tok_rows=tok, voc_rows=voc, cols=cols,
                        dE_sub=wide_dE[:, cols].astype(np.float32), dC_sub=wide_dC[:, cols].astype(np.float32),
                        dE_norm=np.linalg.norm(wide_dE, axis=1), dC_norm=np.linalg.norm(wide_dC, axis=1))


def forward_chunked(w, C64):
    """O.forward on row chunks of E widened on the fly (keeps the fp64 copy of E out of memory)."""
    loss = np.zeros(w.N)
    lse = np.zeros(w.N)
    step = 4096
    for r0 in range(0, w.N, step):
        r1 = min(w.N, r0 + step)
        l, s = O.forward(w.E64(np.arange(r0, r1)), C64, w.targets[r0:r1], w.softcap, w.ignore_index)
        loss[r0:r1], lse[r0:r1] = l, s
        print("   rows %d / %d" % (r1, w.N), flush=True)
    return loss, lse


if __name__ == "__main__":
    args = sys.argv[1:]
    reuse = "--reuse-forward" in args
    names = [a for a in args if not a.startswith("--")] or FULL
    for n in names:
        assert n in CONFIGS, n
        build(n, reuse)
