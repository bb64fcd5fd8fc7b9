"""The five benchmark configurations, three more model shapes, and their seeded generator.

Shapes follow the models the paper measures (Table 1: Gemma-2-2B, N=8192,
D=2304, |V|=256000; Table A3: Phi-3.5-mini D=3072 |V|=32064, Mistral NeMo
D=5120 |V|=131072, Gemma-2 9B D=3584 |V|=256000, Qwen-2.5 7B D=3584 |V|=152064;
Table A4: Llama-3-8B |V|=128256; Fig. A1 / A2: smaller batches at the Gemma-2 2B
shape).  The paper's real weights and Alpaca token batches are replaced by
seeded distributions.

Recipe (fixed here, identical for every consumer):
  rng   = numpy.random.default_rng(seed)
  E     : rows of 4096 at a time, standard_normal float32, then either divided
          by sqrt(D) ("scaled") or by the row's RMS ("rms")
  C     : rows of 4096 at a time, standard_normal float32 times c_std
  perm  : rng.permutation(V)                       (only for Zipf targets)
  rank  : inverse-CDF sample of P(r) ~ r^-1.1, r = 1..V, from rng.random(N)
          target = perm[rank-1]; uniform targets use rng.integers(0, V, N)
  mask  : rng.random(N) < ignore_frac -> target = ignore_index
  boost : (peaked variant) rng.choice(V, V//100, replace=False) rows of C * 8
  Values are rounded to bf16 (round-to-nearest-even) once, on the host; every
  consumer sees exactly those bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

IGNORE_INDEX = -100
_CHUNK_ROWS = 4096


@dataclass(frozen=True)
class Spec:
    name: str
    N: int
    D: int
    V: int
    dtype: str            # "bf16" | "f32"
    e_norm: str           # "scaled" (N(0,1)/sqrt(D)) | "rms" (row / rms(row))
    c_std: float
    targets: str          # "uniform" | "zipf"
    ignore_frac: float
    softcap: float        # 0 = none
    seed: int
    peaked: bool = False  # 1% of C rows scaled x8


CONFIGS = {
    "tiny": Spec("tiny", 256, 64, 1024, "f32", "scaled", 1.0, "uniform", 0.05, 0.0, 0),
    "small_vocab": Spec("small_vocab", 8192, 3072, 32064, "bf16", "rms", 0.02, "zipf", 0.02, 0.0, 2),
    "gemma2_2b": Spec("gemma2_2b", 8192, 2304, 256000, "bf16", "rms", 0.02, "zipf", 0.02, 30.0, 3),
    "llama3_8b": Spec("llama3_8b", 16384, 4096, 128256, "bf16", "rms", 0.02, "zipf", 0.0, 0.0, 4),
    "stress": Spec("stress", 65536, 5120, 131072, "bf16", "rms", 0.02, "zipf", 0.0, 30.0, 5),
    "stress_peaked": Spec("stress_peaked", 65536, 5120, 131072, "bf16", "rms", 0.02, "zipf", 0.0, 30.0, 5,
                          peaked=True),
    # further shapes of Table A3 and a small batch (Fig. A1 / A2), same distributions
    "gemma2_9b": Spec("gemma2_9b", 8192, 3584, 256000, "bf16", "rms", 0.02, "zipf", 0.02, 30.0, 6),
    "qwen25_7b": Spec("qwen25_7b", 8192, 3584, 152064, "bf16", "rms", 0.02, "zipf", 0.02, 0.0, 7),
    "gemma2_2b_n1024": Spec("gemma2_2b_n1024", 1024, 2304, 256000, "bf16", "rms", 0.02, "zipf", 0.02, 30.0, 8),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 storage (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)


@dataclass
class Workload:
    spec: Spec
    N: int
    D: int
    V: int
    dtype: str
    softcap: float
    ignore_index: int
    E: np.ndarray            # uint16 bf16 bits [N,D] (dtype "bf16") or float32 [N,D]
    C: np.ndarray            # uint16 bf16 bits [V,D] or float32 [V,D]
    targets: np.ndarray      # int64 [N]
    boosted: Optional[np.ndarray] = field(default=None)

    def E64(self, rows=None) -> np.ndarray:
        e = self.E if rows is None else self.E[rows]
        return bf16_bits_to_f64(e) if self.dtype == "bf16" else e.astype(np.float64)

    def C64(self, rows=None) -> np.ndarray:
        c = self.C if rows is None else self.C[rows]
        return bf16_bits_to_f64(c) if self.dtype == "bf16" else c.astype(np.float64)

    @property
    def n_valid(self) -> int:
        return int(np.count_nonzero(self.targets != self.ignore_index))

    def mean_dloss(self) -> np.ndarray:
        """Upstream gradient of the mean loss over valid tokens, float32 [N]."""
        nv = max(self.n_valid, 1)
        return np.full(self.N, 1.0 / nv, dtype=np.float32)


def _draw_rows(rng, rows: int, D: int) -> np.ndarray:
    out = np.empty((rows, D), dtype=np.float32)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        out[r0:r1] = rng.standard_normal((r1 - r0, D), dtype=np.float32)
    return out


def make(name: str, N: Optional[int] = None, D: Optional[int] = None, V: Optional[int] = None,
         seed: Optional[int] = None, dtype: Optional[str] = None,
         softcap: Optional[float] = None, ignore_frac: Optional[float] = None) -> Workload:
    """Generate a workload.  Size / option overrides keep the config's distributions."""
    s = CONFIGS[name]
    N = s.N if N is None else int(N)
    D = s.D if D is None else int(D)
    V = s.V if V is None else int(V)
    seed = s.seed if seed is None else int(seed)
    dtype = s.dtype if dtype is None else dtype
    cap = s.softcap if softcap is None else float(softcap)
    ign = s.ignore_frac if ignore_frac is None else float(ignore_frac)
    rng = np.random.default_rng(seed)

    E = _draw_rows(rng, N, D)
    if s.e_norm == "scaled":
        E *= np.float32(1.0 / np.sqrt(D))
    else:
        rms = np.sqrt(np.mean(E.astype(np.float64) ** 2, axis=1))
        E /= rms.astype(np.float32)[:, None]
    C = _draw_rows(rng, V, D)
    C *= np.float32(s.c_std)

    if s.targets == "uniform":
        targets = rng.integers(0, V, size=N, dtype=np.int64)
    else:
        perm = rng.permutation(V)
        w = np.arange(1, V + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = rng.random(N)
        rank = np.minimum(np.searchsorted(cdf, u, side="left"), V - 1)
        targets = perm[rank].astype(np.int64)
    mask = rng.random(N) < ign
    targets = np.where(mask, np.int64(IGNORE_INDEX), targets)

    boosted = None
    if s.peaked:
        boosted = np.sort(rng.choice(V, size=max(V // 100, 1), replace=False))
        C[boosted] *= np.float32(8.0)

    if dtype == "bf16":
        E = f32_to_bf16_bits(E)
        C = f32_to_bf16_bits(C)
    return Workload(s, N, D, V, dtype, cap, IGNORE_INDEX, E, C, targets, boosted)
