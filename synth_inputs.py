"""Seeded synthetic inputs for the IVFPQ search path (tests, smoke, bench).

This module only *generates inputs*: Gaussian-mixture vectors with the shapes
and value ranges of the paper's evaluation sets (Sec. III: a d=128 set of
non-negative small-integer descriptors and a d=96 set of unit-normalised
floats), queries from the same mixtures, and the row indices a k-means
initialisation draws.  It holds none of the method's arithmetic and is the one
module both the CPU oracle's tests and the HIP library's tests may import.

Every stream is `numpy.random.Generator(PCG64(SeedSequence([SEED, stream, chunk])))`.
Rows are produced in fixed chunks of CHUNK_ROWS with the chunk index in the
seed, so row i of a set is the same no matter how many rows are asked for or
how many chunks are held at once.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np

SEED = 230106672
CHUNK_ROWS = 1_000_000

STREAM_CENTRES = 0
STREAM_DATA = 1
STREAM_QUERIES = 2
STREAM_COARSE_INIT = 3
STREAM_PQ_INIT = 4


def _rng(stream: int, chunk: int = 0, salt: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED + salt, stream, chunk])))


@dataclass(frozen=True)
class Workload:
    """One benchmark/test configuration: data recipe + index + search parameters."""
    name: str
    kind: str            # "gauss" | "intgrid" | "unitnorm"
    n: int
    d: int
    n_queries: int
    n_components: int
    sigma: float
    n_lists: int
    pq_dim: int
    pq_bits: int
    n_probes: int
    k: int
    kmeans_iters: int = 10
    salt: int = 0        # distinguishes otherwise identical recipes in tests

    @property
    def code_bytes(self) -> int:
        return self.pq_dim * self.pq_bits // 8

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The named configurations.  "tiny" is the case the oracle finishes in
# seconds; "intgrid_1m" is the d=128 integer-valued set the headline metric is
# quoted on; the others widen it.
WORKLOADS = {
    "tiny": Workload("tiny", "gauss", 10_000, 32, 1_000, 64, 0.1, 64, 16, 8, 8, 10),
    "intgrid_1m": Workload("intgrid_1m", "intgrid", 1_000_000, 128, 10_000, 1_000, 20.0,
                           1_024, 64, 8, 20, 10),
    "unitnorm_1m": Workload("unitnorm_1m", "unitnorm", 1_000_000, 96, 10_000, 2_000, 0.05,
                            1_024, 48, 8, 20, 10),
    "unitnorm_10m": Workload("unitnorm_10m", "unitnorm", 10_000_000, 96, 10_000, 2_000, 0.05,
                             10_000, 48, 8, 20, 10),
    "intgrid_100m_p4": Workload("intgrid_100m_p4", "intgrid", 100_000_000, 128, 10_000, 1_000, 20.0,
                                50_000, 64, 4, 64, 100),
    "intgrid_100m_p8": Workload("intgrid_100m_p8", "intgrid", 100_000_000, 128, 10_000, 1_000, 20.0,
                                50_000, 32, 8, 64, 100),
}


def mixture_centres(w: Workload) -> np.ndarray:
    """[n_components][d] fp32 centres of the mixture."""
    rng = _rng(STREAM_CENTRES, 0, w.salt)
    if w.kind == "gauss":
        c = rng.uniform(-1.0, 1.0, size=(w.n_components, w.d))
    elif w.kind == "intgrid":
        c = rng.uniform(0.0, 128.0, size=(w.n_components, w.d))
    elif w.kind == "unitnorm":
        c = rng.standard_normal(size=(w.n_components, w.d))
        c /= np.linalg.norm(c, axis=1, keepdims=True)
    else:
        raise ValueError(f"unknown kind {w.kind!r}")
    return c.astype(np.float32)


def _chunk(w: Workload, centres: np.ndarray, stream: int, chunk: int, rows: int) -> np.ndarray:
    rng = _rng(stream, chunk, w.salt)
    comp = rng.integers(0, w.n_components, size=CHUNK_ROWS)[:rows]
    noise = rng.standard_normal(size=(rows, w.d), dtype=np.float32)
    x = centres[comp] + np.float32(w.sigma) * noise
    if w.kind == "intgrid":
        x = np.rint(np.clip(x, 0.0, 255.0))
    elif w.kind == "unitnorm":
        x /= np.linalg.norm(x, axis=1, keepdims=True)
    return np.ascontiguousarray(x, dtype=np.float32)


def sample_rows(w: Workload, stream: int, start: int, count: int) -> np.ndarray:
    """Rows [start, start+count) of the set drawn on `stream`, fp32 [count][d]."""
    centres = mixture_centres(w)
    out = np.empty((count, w.d), dtype=np.float32)
    at = 0
    while at < count:
        row = start + at
        chunk, first = divmod(row, CHUNK_ROWS)
        take = min(count - at, CHUNK_ROWS - first)
        block = _chunk(w, centres, stream, chunk, first + take)
        out[at:at + take] = block[first:first + take]
        at += take
    return out


def dataset(w: Workload) -> np.ndarray:
    return sample_rows(w, STREAM_DATA, 0, w.n)


def queries(w: Workload, count: int | None = None) -> np.ndarray:
    return sample_rows(w, STREAM_QUERIES, 0, w.n_queries if count is None else count)


def kmeans_init_rows(stream: int, sub: int, n_rows: int, n_centres: int, salt: int = 0) -> np.ndarray:
    """`n_centres` row indices in [0, n_rows) for a k-means start: distinct when
    there are enough rows, cycling through the rows otherwise."""
    rng = _rng(stream, sub, salt)
    if n_rows >= n_centres:
        return np.sort(rng.choice(n_rows, size=n_centres, replace=False)).astype(np.int64)
    return (np.arange(n_centres, dtype=np.int64) % max(n_rows, 1))


def stride_sample(n_rows: int, limit: int) -> np.ndarray:
    """Indices of at most `limit` rows taken at a fixed stride over [0, n_rows)."""
    if n_rows <= limit:
        return np.arange(n_rows, dtype=np.int64)
    return (np.arange(limit, dtype=np.int64) * n_rows) // limit


def random_index_arrays(n: int, d: int, n_lists: int, pq_dim: int, pq_bits: int, salt: int = 0,
                        scale: float = 1.0, empty_lists: Tuple[int, ...] = ()):
    """A random but valid saved index (centroids, codebooks, list offsets, codes,
    ids) that no training produced: for tests that feed the same arrays to both
    sides.  List lengths are uneven; `empty_lists` are forced empty."""
    rng = _rng(7, 0, salt)
    ksub = 1 << pq_bits
    m = d // pq_dim
    centroids = (scale * rng.standard_normal(size=(n_lists, d))).astype(np.float32)
    codebooks = (0.3 * scale * rng.standard_normal(size=(pq_dim, ksub, m))).astype(np.float32)
    weights = rng.uniform(0.2, 3.0, size=n_lists)
    for l in empty_lists:
        weights[l] = 0.0
    weights /= weights.sum()
    labels = np.sort(rng.choice(n_lists, size=n, p=weights))
    counts = np.bincount(labels, minlength=n_lists)
    list_offsets = np.zeros(n_lists + 1, dtype=np.int64)
    np.cumsum(counts, out=list_offsets[1:])
    code_bytes = pq_dim * pq_bits // 8
    codes = rng.integers(0, 256, size=(n, code_bytes), dtype=np.uint8)
    ids = rng.permutation(n).astype(np.int64)
    return centroids, codebooks, list_offsets, codes, ids
