"""Seeded synthetic workloads shaped like the paper's experiments.

The paper benchmarks on random dense data (Experimental results, single-node
performance: 50x50 and 200x200 maps, 1,000 dimensions) and on a sparse
text-mining vector space (Visualization on real data).  None of those files
exist here, so every input is drawn from a seeded ``numpy`` generator with the
same shapes and structure.  The task's five configurations and two further sparse
shapes of the paper are defined; ``CONFIGS[c]``
describes configuration ``c`` (1-based) and ``make_workload(c)`` draws it.

Only random draws live here: no distance, neighbourhood or update arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Callable, Dict, Optional, Tuple

import numpy as np

DATA_SEED_BASE = 1305_1422_00
CODEBOOK_SEED_BASE = 1422_00


@dataclass(frozen=True)
class Workload:
    """One configuration: data recipe, map geometry and training schedule."""

    config: int
    name: str
    kind: str                 # "dense" or "csr"
    n: int                    # instances
    dim: int                  # features
    rows: int                 # map rows (y direction)
    cols: int                 # map columns (x direction)
    map_type: str             # "planar" or "toroid"
    grid_type: str            # "square" or "hexagonal"
    radius0: float
    radiusN: float
    scale0: float
    scaleN: float
    epochs: int
    recipe: str               # "uniform", "mixture" or "zipf"
    params: Dict[str, float] = field(default_factory=dict)

    @property
    def k(self) -> int:
        return self.rows * self.cols

    @property
    def data_seed(self) -> int:
        return DATA_SEED_BASE + self.config

    @property
    def codebook_seed(self) -> int:
        return CODEBOOK_SEED_BASE + self.config

    def data(self):
        """Dense: float32 [n, dim].  CSR: (indptr int64 [n+1], indices int32, values float32)."""
        if self.recipe == "uniform":
            return dense_uniform(self.n, self.dim, self.data_seed)
        if self.recipe == "mixture":
            return dense_mixture(self.n, self.dim, self.data_seed, **self.params)
        if self.recipe == "zipf":
            return sparse_zipf_csr(self.n, self.dim, self.data_seed, **self.params)
        if self.recipe == "sparse_uniform":
            return sparse_uniform_csr(self.n, self.dim, self.data_seed, **self.params)
        raise ValueError(self.recipe)

    def codebook(self) -> np.ndarray:
        return codebook_uniform(self.k, self.dim, self.codebook_seed)


def dense_uniform(n: int, dim: int, seed: int) -> np.ndarray:
    """i.i.d. uniform [0, 1) values, drawn in fp64 and cast to fp32."""
    rng = np.random.default_rng(seed)
    return rng.random((n, dim)).astype(np.float32)


def dense_mixture(n: int, dim: int, seed: int, components: int = 16, lo: float = 0.0,
                  hi: float = 1.0, sigma: float = 0.05) -> np.ndarray:
    """Equal-weight mixture of isotropic Gaussians.

    Means are drawn first (uniform [lo, hi) per coordinate), then one component
    per instance, then mean + sigma * N(0, I).  Drawn in row chunks so the fp64
    intermediate stays small.
    """
    rng = np.random.default_rng(seed)
    components = int(components)
    means = lo + (hi - lo) * rng.random((components, dim))
    which = rng.integers(components, size=n)
    out = np.empty((n, dim), dtype=np.float32)
    chunk = max(1, min(n, (1 << 24) // max(dim, 1)))
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = (means[which[s:e]] + sigma * rng.standard_normal((e - s, dim))).astype(np.float32)
    return out


def sparse_zipf_csr(n: int, dim: int, seed: int, mean_len: float = 100.0, max_len: int = 400,
                    zipf_s: float = 1.1, poisson_lam: float = 2.0
                    ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Text-mining-shaped CSR rows.

    Row length ~ Poisson(mean_len) clipped to [1, min(max_len, dim)].  Column
    indices are distinct draws from a Zipf(zipf_s) law over 0..dim-1 (column 0
    the most frequent), duplicates rejected, sorted ascending.  Values are
    log(2 + Poisson(poisson_lam)) (term-frequency style), then every row is
    scaled to unit Euclidean length.  Indices are zero-based, as in the paper's
    sparse file format example.
    """
    rng = np.random.default_rng(seed)
    max_len = int(min(max_len, dim))
    lens = np.clip(rng.poisson(mean_len, size=n), 1, max_len).astype(np.int64)
    pmf = 1.0 / np.arange(1, dim + 1, dtype=np.float64) ** zipf_s
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=indptr[1:])
    nnz = int(indptr[-1])
    indices = np.empty(nnz, dtype=np.int32)
    values = np.empty(nnz, dtype=np.float32)
    for j in range(n):
        need = int(lens[j])
        got = np.empty(0, dtype=np.int64)
        while got.size < need:
            draw = np.searchsorted(cdf, rng.random(2 * need + 8), side="right")
            draw = np.minimum(draw, dim - 1)
            merged = np.concatenate([got, draw])
            _, first = np.unique(merged, return_index=True)
            got = merged[np.sort(first)][:need]      # keep draw order, drop repeats
        cols = np.sort(got)
        v = np.log(2.0 + rng.poisson(poisson_lam, size=need))
        v /= np.sqrt(np.sum(v * v))
        indices[indptr[j]:indptr[j + 1]] = cols
        values[indptr[j]:indptr[j + 1]] = v
    return indptr, indices, values


def sparse_uniform_csr(n: int, dim: int, seed: int, density: float = 0.05
                       ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Random sparse rows as in the paper's sparse-versus-dense comparison: every row has
    round(density * dim) nonzeros at distinct uniformly drawn columns (sorted), values uniform [0, 1)."""
    rng = np.random.default_rng(seed)
    per = max(1, int(round(density * dim)))
    indptr = (np.arange(n + 1, dtype=np.int64) * per)
    indices = np.empty(n * per, dtype=np.int32)
    chunk = max(1, (1 << 22) // dim)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        keys = rng.random((e - s, dim))
        cols = np.sort(np.argpartition(keys, per - 1, axis=1)[:, :per], axis=1)
        indices[s * per:e * per] = cols.reshape(-1)
    values = rng.random(n * per).astype(np.float32)
    return indptr, indices, values


def codebook_uniform(k: int, dim: int, seed: int) -> np.ndarray:
    """Random initial code book: uniform [0, 1), fp32, node-major [k, dim]."""
    rng = np.random.default_rng(seed)
    out = np.empty((k, dim), dtype=np.float32)
    chunk = max(1, (1 << 24) // max(dim, 1))          # same stream as one big draw, small fp64 intermediate
    for s in range(0, k, chunk):
        e = min(k, s + chunk)
        out[s:e] = rng.random((e - s, dim)).astype(np.float32)
    return out


CONFIGS: Dict[int, Workload] = {
    1: Workload(1, "toy-20x20-planar-square", "dense", 1_000, 10, 20, 20, "planar", "square",
                10.0, 1.0, 0.1, 0.01, 10, "uniform"),
    2: Workload(2, "dense-50x50-toroid-square", "dense", 100_000, 1_000, 50, 50, "toroid", "square",
                25.0, 1.0, 1.0, 0.01, 10, "mixture",
                {"components": 16, "lo": 0.0, "hi": 1.0, "sigma": 0.05}),
    3: Workload(3, "emergent-200x200-toroid-hex", "dense", 50_000, 256, 200, 200, "toroid", "hexagonal",
                100.0, 1.0, 1.0, 0.01, 5, "mixture",
                {"components": 64, "lo": -1.0, "hi": 1.0, "sigma": 0.1}),
    4: Workload(4, "sparse-50x50-planar-square", "csr", 100_000, 50_000, 50, 50, "planar", "square",
                25.0, 1.0, 1.0, 0.01, 10, "zipf",
                {"mean_len": 100.0, "max_len": 400, "zipf_s": 1.1, "poisson_lam": 2.0}),
    5: Workload(5, "large-100x100-planar-hex", "dense", 1_000_000, 128, 100, 100, "planar", "hexagonal",
                50.0, 1.0, 1.0, 0.01, 5, "mixture",
                {"components": 256, "lo": 0.0, "hi": 1.0, "sigma": 0.03}),
    # Two more sparse shapes from the paper's own experiments (not among the task's five):
    # the sparse-versus-dense comparison (1,000 dimensions, five per cent nonzeros, 50 x 50 map) and
    # the Reuters text-mining map (12,347 index terms in a space of about twenty thousand
    # dimensions, toroid emergent map of 336 x 205 nodes, radius 100 -> 1 over ten epochs).
    6: Workload(6, "sparse-uniform-50x50-planar-square", "csr", 100_000, 1_000, 50, 50, "planar", "square",
                25.0, 1.0, 1.0, 0.01, 10, "sparse_uniform", {"density": 0.05}),
    7: Workload(7, "text-esom-336x205-toroid-square", "csr", 12_347, 20_000, 205, 336, "toroid", "square",
                100.0, 1.0, 1.0, 0.1, 10, "zipf",
                {"mean_len": 100.0, "max_len": 400, "zipf_s": 1.1, "poisson_lam": 2.0}),
}


def make_workload(config: int) -> Workload:
    return CONFIGS[config]


def scaled_workload(config: int, *, n: Optional[int] = None, dim: Optional[int] = None,
                    rows: Optional[int] = None, cols: Optional[int] = None,
                    epochs: Optional[int] = None) -> Workload:
    """The same recipe at reduced sizes (for parity cases the oracle finishes in seconds).

    The start radius follows the map: half the smaller side, as the paper's
    default, whenever the map is resized.
    """
    w = CONFIGS[config]
    changes = {}
    if n is not None:
        changes["n"] = int(n)
    if dim is not None:
        changes["dim"] = int(dim)
    if rows is not None or cols is not None:
        r = int(rows if rows is not None else w.rows)
        c = int(cols if cols is not None else w.cols)
        changes.update(rows=r, cols=c, radius0=max(1.0, min(r, c) / 2.0))
    if epochs is not None:
        changes["epochs"] = int(epochs)
    return replace(w, **changes)
