"""Seeded synthetic inputs for the ASTRA classifier-layer hot path.

This module only *makes inputs*: classifier rows W, query embeddings Z, positive
label lists and the five workload descriptions.  It holds none of the method's
arithmetic (no scores, no sampling of negatives, no loss) and is the one piece
that tests of the CPU oracle and of the HIP library both use, so that both see
identical input bits.

The value recipe uses integer hashing only, followed by one float32 multiply,
so the same call gives the same bits on a CPU tensor and on a GPU tensor:
element e of a tensor with tag t is (u1+u2+u3+u4 - 2*65535) * c, with u1..u4 the
four 16-bit fields of a 64-bit hash of (seed, t, e) (an Irwin-Hall sum, close
to a normal law) and c chosen so the variance is 1/d.  The shapes stand in for
the datasets of the paper's dataset-statistics table (label counts 131K, 670K,
1.3M, 120M; a few positives per point; heavy-tailed label frequencies modelled
by a Zipf law over a permuted label order).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 20240930
TAG_W = 1
TAG_Z = 2

_GOLD = -7046029254386353131      # 0x9E3779B97F4A7C15 as signed 64-bit
_C1 = -4658895280553007687        # 0xBF58476D1CE4E5B9
_C2 = -7723592293110705685        # 0x94D049BB133111EB


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _hash64(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _C1
    x = x ^ _lsr(x, 27)
    x = x * _C2
    x = x ^ _lsr(x, 31)
    return x


def _tensor_seed(seed: int, tag: int) -> int:
    v = (seed * 0x9E3779B97F4A7C15 + tag * 0xD1B54A32D192ED03) & ((1 << 64) - 1)
    return v - (1 << 64) if v >= (1 << 63) else v


def gaussian_rows(seed: int, tag: int, row0: int, nrows: int, d: int,
                  dtype: torch.dtype, device="cpu") -> torch.Tensor:
    """Rows row0..row0+nrows-1 of the [*, d] tensor identified by (seed, tag),
    entries approximately N(0, 1/d), rounded to `dtype`.  A row is a pure
    function of (seed, tag, row index), so any slice can be made anywhere."""
    e = torch.arange(row0 * d, (row0 + nrows) * d, dtype=torch.int64, device=device)
    h = _hash64(e * _GOLD + _tensor_seed(seed, tag))
    s = (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    s = (s - 2 * 65535).to(torch.float32)
    var = 4.0 * (65536.0 ** 2 - 1.0) / 12.0
    c = torch.tensor(1.0 / math.sqrt(d * var), dtype=torch.float32, device=device)
    return (s * c).to(dtype).reshape(nrows, d)


def gaussian_rows_at(seed: int, tag: int, rows: torch.Tensor, d: int, dtype: torch.dtype) -> torch.Tensor:
    """The rows with the given indices (int64 tensor, any device) of the same tensor."""
    rows = rows.to(torch.int64)
    e = (rows[:, None] * d + torch.arange(d, dtype=torch.int64, device=rows.device)[None, :]).reshape(-1)
    h = _hash64(e * _GOLD + _tensor_seed(seed, tag))
    s = (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    s = (s - 2 * 65535).to(torch.float32)
    var = 4.0 * (65536.0 ** 2 - 1.0) / 12.0
    c = torch.tensor(1.0 / math.sqrt(d * var), dtype=torch.float32, device=rows.device)
    return (s * c).to(dtype).reshape(rows.numel(), d)


def make_matrix(seed: int, tag: int, nrows: int, d: int, dtype: torch.dtype,
                device="cpu", chunk_rows: int | None = None) -> torch.Tensor:
    """Whole [nrows, d] tensor, generated in chunks to bound temporaries."""
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 24) // d)
    out = torch.empty((nrows, d), dtype=dtype, device=device)
    for r0 in range(0, nrows, chunk_rows):
        n = min(chunk_rows, nrows - r0)
        out[r0:r0 + n] = gaussian_rows(seed, tag, r0, n, d, dtype, device)
    return out


# --------------------------------------------------------------------------
# positives
# --------------------------------------------------------------------------
def _affine_perm(L: int, seed: int):
    """Multiplier and offset of the bijection rank -> (a*rank + b) mod L that
    spreads the frequent labels over the id range."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    while True:
        a = int(rng.integers(L // 3 + 1, L)) | 1
        if math.gcd(a, L) == 1:
            break
    b = int(rng.integers(0, L))
    return a, b


def zipf_positives(seed: int, nq: int, L: int, zipf_s: float, count_law: str,
                   k_p: int) -> np.ndarray:
    """int32 [nq, k_p] positive label ids, -1 padded.  Label popularity follows
    Zipf(zipf_s) over ranks 1..L, ranks mapped to ids by an affine bijection.
    count_law: 'one', 'uniform:a:b', 'poisson:mean' (at least 1, at most k_p).
    Labels within a query are distinct."""
    rng = np.random.default_rng(seed)
    ranks = np.arange(1, L + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-zipf_s))
    cdf /= cdf[-1]
    a, b = _affine_perm(L, seed)
    if count_law == "one":
        counts = np.ones(nq, dtype=np.int64)
    elif count_law.startswith("uniform:"):
        _, lo, hi = count_law.split(":")
        counts = rng.integers(int(lo), int(hi) + 1, size=nq)
    elif count_law.startswith("poisson:"):
        counts = np.maximum(1, rng.poisson(float(count_law.split(":")[1]), size=nq))
    else:
        raise ValueError(count_law)
    counts = np.minimum(counts, min(k_p, L))
    pos = np.full((nq, k_p), -1, dtype=np.int32)
    for i in range(nq):
        chosen: list[int] = []
        while len(chosen) < counts[i]:
            r = int(np.searchsorted(cdf, rng.random(), side="right"))
            r = min(r, L - 1)
            lab = (a * r + b) % L
            if lab not in chosen:
                chosen.append(lab)
        pos[i, :len(chosen)] = chosen
    return pos


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    d: int
    dtype: str            # 'f32' or 'bf16' storage of W and Z
    B: int
    k_p: int              # padded width of the positive lists
    count_law: str
    zipf_s: float
    k_h: int
    k_r: int
    pool: int             # number of queries mined per refresh
    steps: int
    refresh: int          # steps between shortlist refreshes (0 = mine once)
    lr: float = 0.05
    config_id: int = 0

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS = {
    "tiny": Workload("tiny", 4096, 64, "f32", 32, 1, "one", 1.0, 8, 16,
                     pool=32, steps=1, refresh=0, config_id=1),
    "c2": Workload("c2", 131072, 768, "bf16", 512, 4, "uniform:1:4", 1.0, 64, 256,
                   pool=10240, steps=100, refresh=20, config_id=2),
    "c3": Workload("c3", 670000, 768, "bf16", 1024, 16, "poisson:5", 1.1, 100, 512,
                   pool=8192, steps=50, refresh=0, config_id=3),
    "c4": Workload("c4", 1300000, 768, "bf16", 2048, 8, "uniform:1:8", 1.0, 100, 1024,
                   pool=65536, steps=200, refresh=0, config_id=4),
    "c5": Workload("c5", 120000000, 256, "bf16", 4096, 3, "uniform:1:3", 1.2, 50, 2048,
                   pool=16384, steps=100, refresh=0, lr=0.01, config_id=5),
}


def step_seed(base: int, config_id: int, step: int) -> int:
    """Seed handed to the negative sampler for one step."""
    v = (base * 0x9E3779B97F4A7C15 + config_id * 0xD1B54A32D192ED03
         + step * 0x2545F4914F6CDD1D) & ((1 << 64) - 1)
    return v


def add_positive_signal(Z: torch.Tensor, W: torch.Tensor, pos: np.ndarray,
                        alpha: float = 0.5) -> torch.Tensor:
    """Structured variant: z_i <- z_i + alpha * w_{pos_i[0]}, so that positives
    score high and mined shortlists contain them (exercises masking)."""
    idx = torch.as_tensor(pos[:, 0].astype(np.int64), device=Z.device)
    out = Z.to(torch.float32) + alpha * W[idx].to(torch.float32)
    return out.to(Z.dtype)
