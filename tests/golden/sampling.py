"""Which rows and columns of the gradients the full-size checks look at.  Shared by the script that writes the
stored oracle values (make_golden.py) and by tests/test_full_size_gpu.py; no arithmetic of the method here.

Tokens (rows of dE): both sides of every 256-token tile edge, the first and last token, some ignored tokens,
random ones up to `count`.  Vocabulary entries (rows of dC): both sides of every multiple of 2048 (every slab
edge of every slab width the library uses: 6144 k, 16384 k, 24576 k, and their small-batch multiples), the edges
of the (possibly ragged) last 256-wide tile, the most frequent and some never-used targets, boosted rows of the
peaked variant, random ones up to `count`.  Columns (entries of a row): the first and last, both sides of the
256-wide tile edges of D, random ones up to `count`."""
import numpy as np

ROWS = 1024
COLS = 16


def sample_tokens(w, count=ROWS):
    rng = np.random.default_rng(2000 + w.spec.seed)
    rows = {0, w.N - 1}
    for e in range(256, w.N, 256):
        rows |= {e - 1, e}
    ign = np.nonzero(w.targets == w.ignore_index)[0]
    rows |= {int(i) for i in ign[:8]}
    rows = {r for r in rows if 0 <= r < w.N}
    while len(rows) < min(count, w.N):
        rows.add(int(rng.integers(0, w.N)))
    return np.array(sorted(rows))


def sample_vocab(w, count=ROWS):
    rng = np.random.default_rng(3000 + w.spec.seed)
    rows = {0, w.V - 1}
    for e in range(2048, w.V, 2048):
        rows |= {e - 1, e}
    last_tile = (w.V - 1) // 256 * 256
    rows |= {last_tile - 1, last_tile, w.V - 2}
    valid_t = w.targets[w.targets != w.ignore_index]
    counts = np.bincount(valid_t, minlength=w.V)
    rows |= {int(v) for v in np.argsort(-counts)[:8]}
    never = np.nonzero(counts == 0)[0]
    rows |= {int(v) for v in never[:: max(len(never) // 8, 1)][:8]}
    if w.boosted is not None:
        rows |= {int(v) for v in w.boosted[:: max(len(w.boosted) // 16, 1)]}
    rows = {r for r in rows if 0 <= r < w.V}
    while len(rows) < min(count, w.V):
        rows.add(int(rng.integers(0, w.V)))
    return np.array(sorted(rows))


def sample_columns(w, count=COLS):
    rng = np.random.default_rng(4000 + w.spec.seed)
    cols = {0, w.D - 1}
    for e in range(256, w.D, 256):
        if len(cols) + 2 <= count - 4:
            cols |= {e - 1, e}
    while len(cols) < min(count, w.D):
        cols.add(int(rng.integers(0, w.D)))
    return np.array(sorted(cols))
