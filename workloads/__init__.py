"""Seeded synthetic inputs for the Ok-Topk one-GPU hot path.

This module only draws numbers.  It holds none of the method's arithmetic
(no accumulate, no threshold, no selection, no partition, no reduction) and
imports neither the CPU oracle nor the HIP binding, so both can be fed the
very same bytes.

The paper trains VGG-16 / LSTM / BERT on Cifar-10 / AN4 / Wikipedia
(Sec. 5, Table 2); none of that data is available here.  The generators
below stand in for it with flat fp32 gradients that keep what the paper says
about gradient values: zero-centred, sharply peaked, heavier than Gaussian
tails (Sec. 3.1.3, Fig. 4), differing scale per layer, top-k coordinates that
are consistent across workers at region level (Sec. 3.1.1).

Every array is a pure function of (workload, seed, iteration, chunk), drawn
with numpy's counter-based Philox generator in float64 and cast to float32,
in fixed chunks of 2**22 elements so that a large vector can be produced by
several threads and still be bit-identical to a single-threaded run.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 1 << 22


# --------------------------------------------------------------------------
# workload table (the five configurations this repository is measured on)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    n: int                 # flat gradient length
    density_num: int       # density = density_num / density_den
    density_den: int
    P: int                 # simulated workers contributing to one region
    dist: str              # "laplace" | "normal" | "student3"
    segments: int          # 0 = iid, else number of layer segments
    scale_lo: float        # per-segment scale range (log-uniform) or the iid scale
    scale_hi: float
    iterations: int
    refresh_period: int    # threshold re-evaluation period (tau'); 0 = only at iteration 0
    contrib: str           # "uniform" | "overlap30" | "zipf"
    contrib_dist: str
    contrib_scale: float
    lr: float = 1.0

    @property
    def k(self) -> int:
        # k = ceil(n * density), integer arithmetic
        return -(-self.n * self.density_num // self.density_den)

    @property
    def m(self) -> int:
        # entries each simulated worker contributes
        return self.k // self.P

    def refresh(self, it: int) -> bool:
        if self.refresh_period == 0:
            return it == 0
        return it % self.refresh_period == 0

    def scaled(self, n: int, iterations: int | None = None) -> "Workload":
        """Same recipe at another length (for element-by-element parity runs)."""
        return dataclasses.replace(
            self, name=f"{self.name}@n={n}", n=int(n),
            iterations=self.iterations if iterations is None else iterations)


WORKLOADS = {
    "cfg1": Workload("cfg1", 1001, 1_048_576, 1, 100, 4, "laplace", 0, 1e-3, 1e-3,
                     1, 0, "uniform", "laplace", 1e-3),
    "cfg2": Workload("cfg2", 2002, 25_557_032, 1, 100, 16, "normal", 161, 1e-5, 1e-2,
                     10, 0, "uniform", "normal", 1e-3),
    "cfg3": Workload("cfg3", 3003, 110_000_000, 1, 100, 32, "laplace", 199, 1e-6, 1e-2,
                     64, 32, "overlap30", "laplace", 1e-3),
    "cfg4": Workload("cfg4", 4004, 336_000_000, 1, 1000, 64, "student3", 0, 1e-4, 1e-4,
                     3, 1, "uniform", "student3", 1e-4),
    "cfg5": Workload("cfg5", 5005, 110_000_000, 1, 100, 256, "normal", 0, 1e-3, 1e-3,
                     0, 0, "zipf", "normal", 1e-3),
}


# --------------------------------------------------------------------------
# random streams
# --------------------------------------------------------------------------
def _rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    key = np.array([seed & 0xFFFFFFFFFFFFFFFF,
                    ((stream & 0xFFFFFFFF) << 32) | (chunk & 0xFFFFFFFF)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _draw(rng: np.random.Generator, dist: str, size: int) -> np.ndarray:
    if dist == "laplace":
        return rng.laplace(0.0, 1.0, size)
    if dist == "normal":
        return rng.standard_normal(size)
    if dist == "student3":
        return rng.standard_t(3.0, size)
    raise ValueError(dist)


def _threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


# --------------------------------------------------------------------------
# dense gradients
# --------------------------------------------------------------------------
def segment_table(w: Workload) -> tuple[np.ndarray, np.ndarray]:
    """(bounds[nseg+1] int64, scale[nseg] float64) of the layer segments.

    Segment lengths come from log-uniform weights (one decade each side of
    the mean) with a floor of 64 elements, rescaled so they sum to n; scales
    are log-uniform in [scale_lo, scale_hi].  With segments == 0 the vector is
    one segment of scale scale_lo.
    """
    if w.segments <= 0:
        return np.array([0, w.n], dtype=np.int64), np.array([w.scale_lo])
    nseg = min(w.segments, max(1, w.n // 64))
    rng = _rng(w.seed, 0xFFFF0001)
    weights = np.exp(rng.uniform(np.log(0.1), np.log(10.0), nseg))
    scale = np.exp(rng.uniform(np.log(w.scale_lo), np.log(w.scale_hi), nseg))
    spare = w.n - 64 * nseg
    extra = np.floor(weights / weights.sum() * spare).astype(np.int64)
    extra[-1] += spare - extra.sum()
    lengths = 64 + extra
    bounds = np.zeros(nseg + 1, dtype=np.int64)
    np.cumsum(lengths, out=bounds[1:])
    assert bounds[-1] == w.n
    return bounds, scale


def _scale_vector(bounds: np.ndarray, scale: np.ndarray, a: int, b: int) -> np.ndarray:
    """Per-element scale for elements [a, b)."""
    pos = np.arange(a, b, dtype=np.int64)
    seg = np.searchsorted(bounds, pos, side="right") - 1
    return scale[seg]


def gradient(w: Workload, it: int, out: np.ndarray | None = None) -> np.ndarray:
    """The stochastic gradient G of iteration `it` (0-based): fp32[n].

    Fresh noise every iteration, same segment table throughout (the value
    distribution changes slowly over time, Sec. 3.1.3).
    """
    bounds, scale = segment_table(w)
    g = np.empty(w.n, dtype=np.float32) if out is None else out
    assert g.shape == (w.n,) and g.dtype == np.float32
    nchunk = -(-w.n // CHUNK)

    def fill(c: int) -> None:
        a, b = c * CHUNK, min(w.n, (c + 1) * CHUNK)
        x = _draw(_rng(w.seed, it, c), w.dist, b - a)
        if len(scale) == 1:
            x *= scale[0]
        else:
            x *= _scale_vector(bounds, scale, a, b)
        g[a:b] = x.astype(np.float32)

    if nchunk <= 2:
        for c in range(nchunk):
            fill(c)
    else:
        with ThreadPoolExecutor(_threads()) as ex:
            list(ex.map(fill, range(nchunk)))
    return g


# --------------------------------------------------------------------------
# sparse contributions for the local reduction
# --------------------------------------------------------------------------
def _unique_uniform(rng: np.random.Generator, width: int, count: int) -> np.ndarray:
    count = min(count, width)
    if count == 0:
        return np.zeros(0, dtype=np.int64)
    return np.sort(rng.choice(width, size=count, replace=False, shuffle=False)).astype(np.int64)


def _zipf_unique(rng: np.random.Generator, cdf: np.ndarray, perm: np.ndarray,
                 count: int) -> np.ndarray:
    """`count` distinct offsets whose ranks follow the truncated Zipf law in `cdf`."""
    width = len(cdf)
    count = min(count, width)
    seen = np.zeros(width, dtype=bool)
    got = 0
    while got < count:
        r = np.searchsorted(cdf, rng.random(2 * (count - got) + 16), side="right")
        r = np.minimum(r, width - 1)
        u, first = np.unique(r, return_index=True)
        fresh = ~seen[u]
        u, first = u[fresh], first[fresh]
        u = u[np.argsort(first, kind="stable")][:count - got]   # first occurrences, draw order
        seen[u] = True
        got += len(u)
    return np.sort(perm[np.flatnonzero(seen)]).astype(np.int64)


def contributions(w: Workload, lo: int, hi: int, m: int | None = None,
                  P: int | None = None, stream: int = 0):
    """P sorted COO chunks, as one region's owner would receive them.

    Returns (idx_cat uint32[E], val_cat fp32[E], chunk_off uint64[P+1]); chunk p
    is the slice [chunk_off[p], chunk_off[p+1]).  Indices are global, strictly
    ascending inside a chunk, and all lie in [lo, hi).

    uniform   : each worker draws m distinct indices uniformly in the region.
    overlap30 : floor(0.3 m) indices are one pool shared by all workers; the
                rest are private uniform draws outside the pool.
    zipf      : ranks follow Zipf(s = 1.1) truncated to the region width and map
                to offsets through one permutation shared by all workers, so the
                same hot indices collide across workers.
    `stream` picks an independent replica of the same recipe (other regions of a
    batch).
    """
    P = w.P if P is None else P
    m = w.m if m is None else m
    width = hi - lo
    assert width > 0
    base = 0x1000 + (stream << 12)
    shared = _rng(w.seed, 0xFFFF0002 + stream)
    pool = np.zeros(0, dtype=np.int64)
    if w.contrib == "overlap30":
        pool = _unique_uniform(shared, width, int(0.3 * min(m, width)))
        outside = np.setdiff1d(np.arange(width, dtype=np.int64), pool, assume_unique=True) \
            if width <= (1 << 24) else None
    if w.contrib == "zipf":
        pmf = np.arange(1, width + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(pmf)
        cdf /= cdf[-1]
        perm = shared.permutation(width)
    idx_parts, val_parts = [], []
    off = np.zeros(P + 1, dtype=np.uint64)
    for p in range(P):
        rng = _rng(w.seed, base + p + 1)
        if w.contrib == "uniform":
            loc = _unique_uniform(rng, width, m)
        elif w.contrib == "overlap30":
            priv = min(m, width) - len(pool)
            if outside is not None:
                pick = _unique_uniform(rng, len(outside), priv)
                mine = outside[pick]
            else:
                cand = np.unique(rng.integers(0, width, size=2 * priv + 64))
                cand = np.setdiff1d(cand, pool, assume_unique=True)
                mine = rng.permutation(cand)[:priv]
            loc = np.sort(np.concatenate([pool, mine]))
        elif w.contrib == "zipf":
            loc = _zipf_unique(rng, cdf, perm, m)
        else:
            raise ValueError(w.contrib)
        v = (_draw(rng, w.contrib_dist, len(loc)) * w.contrib_scale).astype(np.float32)
        idx_parts.append((loc + lo).astype(np.uint32))
        val_parts.append(v)
        off[p + 1] = off[p] + np.uint64(len(loc))
    return (np.concatenate(idx_parts) if idx_parts else np.zeros(0, np.uint32),
            np.concatenate(val_parts) if val_parts else np.zeros(0, np.float32),
            off)


def whole_space_contributions(w: Workload):
    """cfg1-style chunks: each worker's m entries spread over the whole index
    space [0, n); the reduce then picks out one region of it."""
    return contributions(w, 0, w.n)
