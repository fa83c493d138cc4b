"""Seeded synthetic workloads shaped like the paper's datasets (Table 2 of the paper lists the
real ones; none of them is used or reconstructed here).

This module only draws random numbers.  It contains none of the search method's arithmetic and is
the single piece of code that the CPU oracle's tests and the HIP path's tests both call.

Each workload is a Gaussian mixture: a vector is
`transform(mean[c] + sigma * z + spread * z_r @ basis[c])`, i.e. every component has an isotropic
part and (except for the tiny workload) a low-rank part, so that neighbourhoods have a low
intrinsic dimension as real descriptor data does and components overlap.  Base
vectors and queries come from the same mixture through independent streams; queries are never
members of the base set.  Streams: seed*16 + 0 mixture parameters, + 1 base vectors, + 2 queries.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload plus the index/search parameters quoted with it."""

    name: str
    n: int                 # base vectors
    d: int                 # dimensions
    nq: int                # queries
    comps: int             # mixture components
    kind: str              # "gmm" | "sift" | "dense" | "sphere"
    raw_u8: bool           # keep base vectors as uint8 (SIFT1B-like storage)
    nlist: int
    M: int                 # PQ sub-quantizers (4 bits each), d / 2 in the paper's experiments
    k: int
    refine_k: int          # bigK = K * K_FACTOR of Alg. 2
    nprobes: tuple
    seed: int


WORKLOADS = {
    # small case used by the element-wise parity tests
    "tiny": Workload("tiny", 20_000, 32, 200, 100, "gmm", False, 64, 16, 10, 40,
                     (1, 4, 16, 64), 1),
    # SIFT1M-shaped: 1M x 128, integer valued in [0, 255]
    "sift1m": Workload("sift1m", 1_000_000, 128, 10_000, 1000, "sift", False, 1024, 64, 10, 100,
                       (1, 2, 4, 8, 16, 32, 64, 128), 2),
    # GIST-shaped: 1M x 960 dense non-negative
    "gist1m": Workload("gist1m", 1_000_000, 960, 1000, 1000, "dense", False, 1024, 240, 10, 100,
                       (1, 2, 4, 8, 16, 32, 64, 128), 3),
    # 10M x 96 unit-norm
    "sphere10m": Workload("sphere10m", 10_000_000, 96, 10_000, 4000, "sphere", False, 4096, 48,
                          10, 100, (4, 8, 16, 32, 64, 128, 256), 4),
    # SIFT1B-like slice: 100M x 128 kept as uint8
    "sift100m": Workload("sift100m", 100_000_000, 128, 10_000, 10_000, "sift", True, 16384, 64,
                         10, 200, (8, 16, 32, 64, 128, 256, 512), 5),
}


def scaled(w: Workload, n: int, nq: int | None = None, nlist: int | None = None) -> Workload:
    """Same generator and dimensions at a smaller base size (for tests that must finish quickly)."""
    return replace(w, name=f"{w.name}@{n}", n=n, nq=nq or w.nq, nlist=nlist or w.nlist)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed * 16 + stream))


class Mixture:
    """Mixture parameters of a workload, drawn once from stream 0."""

    def __init__(self, w: Workload):
        self.w = w
        g = _rng(w.seed, 0)
        c, d = w.comps, w.d
        self.rank, self.spread, self.basis = 0, 0.0, None
        if w.kind == "gmm":
            self.mean = g.uniform(-1.0, 1.0, size=(c, d)).astype(np.float32)
            self.sigma = 0.1
        elif w.kind == "sift":
            zero = g.random(size=(c, d)) < 0.35
            mag = np.minimum(50.0, g.exponential(10.0, size=(c, d)))
            self.mean = np.where(zero, 0.0, mag).astype(np.float32)
            self.sigma = 10.0
            self._low_rank(g, 16, 60.0)
        elif w.kind == "dense":
            self.scale = g.uniform(0.01, 0.2, size=(d,)).astype(np.float32)
            self.mean = (1.0 + 0.03 * g.uniform(-1.0, 1.0, size=(c, d))).astype(np.float32)
            self.sigma = 0.05
            self._low_rank(g, 24, 0.5)
        elif w.kind == "sphere":
            self.mean = (0.25 * g.standard_normal(size=(c, d))).astype(np.float32)
            self.sigma = 0.1
            self._low_rank(g, 24, 1.0)
        else:
            raise ValueError(w.kind)

    def _low_rank(self, g, rank, spread):
        b = g.standard_normal(size=(self.w.comps, rank, self.w.d)).astype(np.float32)
        b /= np.linalg.norm(b, axis=2, keepdims=True)
        self.rank, self.spread, self.basis = rank, spread, b

    def draw(self, g: np.random.Generator, n: int, as_u8: bool = False) -> np.ndarray:
        w = self.w
        out = np.empty((n, w.d), dtype=np.uint8 if as_u8 else np.float32)
        step = max(1, (1 << 25) // w.d)
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            comp = g.integers(0, w.comps, size=hi - lo)
            x = g.standard_normal(size=(hi - lo, w.d), dtype=np.float32)
            x *= np.float32(self.sigma)
            x += self.mean[comp]
            if self.rank:
                # low-rank part of each component's covariance: x += s * z_r @ B_c
                z = g.standard_normal(size=(hi - lo, self.rank), dtype=np.float32)
                order = np.argsort(comp, kind="stable")
                cnt = np.bincount(comp, minlength=w.comps)
                pos = 0
                for c in np.flatnonzero(cnt):
                    rows = order[pos:pos + cnt[c]]
                    x[rows] += np.float32(self.spread) * (z[rows] @ self.basis[c])
                    pos += cnt[c]
            if w.kind == "sift":
                np.rint(x, out=x)
                np.clip(x, 0.0, 255.0, out=x)
            elif w.kind == "dense":
                x *= self.scale
                np.maximum(x, 0.0, out=x)
            elif w.kind == "sphere":
                x /= np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-12).astype(np.float32)
            out[lo:hi] = x
        return out


def make_base(w: Workload) -> np.ndarray:
    """Base vectors [n][d]; uint8 when the workload keeps raw vectors as bytes, else float32."""
    return Mixture(w).draw(_rng(w.seed, 1), w.n, as_u8=w.raw_u8)


def make_queries(w: Workload, nq: int | None = None) -> np.ndarray:
    """Query vectors [nq][d], always float32."""
    return Mixture(w).draw(_rng(w.seed, 2), nq or w.nq, as_u8=False)


def random_vectors(seed: int, n: int, d: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """Unstructured uniform vectors for small unit tests."""
    return _rng(seed, 3).uniform(lo, hi, size=(n, d)).astype(np.float32)
