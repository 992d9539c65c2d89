"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws random fp32 vectors and picks the scale parameter; it holds
none of the method's arithmetic (no quantizer, no scoring, no selection) and is the
one module that both the HIP path's callers and the CPU oracle's callers use.

Every workload is generated in fixed blocks of ``BLOCK`` rows, block ``i`` of stream
``s`` from ``numpy.random.default_rng([seed, s, i])``, so any row range can be
produced without generating what comes before it.  Stream 0 is the database,
stream 1 the queries, stream 2 the mixture centres / cluster weights.  Rows are
L2-normalised in fp32 after generation.

The public datasets the paper measured on (word embeddings of dimension 200, CNN
descriptors of dimension 96, SIFT descriptors) are not available here; C4 and C5
stand in for the first two with Gaussian-mixture data of the same shape, C1/C2
for the paper's "128-d random data", C3 for high-dimensional non-negative
descriptors.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BLOCK = 65536


@dataclass(frozen=True)
class Workload:
    name: str
    n: int            # database rows
    d: int            # dimension
    m: int            # queries
    bits: tuple       # code widths to run
    ks: tuple         # K values to run
    kind: str         # "gauss" | "absgauss" | "mixture"
    seed: int = 0
    clusters: int = 0
    std: float = 0.0
    zipf: float | None = None
    note: str = field(default="", compare=False)


WORKLOADS = {
    "C1": Workload("C1", 10_000, 128, 100, (4,), (10,), "gauss",
                   note="i.i.d. N(0,1), small case the oracle finishes in seconds"),
    "C2": Workload("C2", 1_000_000, 128, 10_000, (4,), (100,), "gauss",
                   note="headline: 1M x 128, 4-bit, K=100"),
    "C3": Workload("C3", 1_000_000, 960, 1_000, (3, 4), (10,), "absgauss",
                   note="|N(0,1)| coordinates: constant sign plane, heavy score ties"),
    "C4": Workload("C4", 2_000_000, 200, 10_000, (3,), (10, 100), "mixture",
                   clusters=1000, std=0.3, zipf=1.1,
                   note="stand-in for 200-d word embeddings"),
    "C5": Workload("C5", 10_000_000, 96, 10_000, (4,), (100,), "mixture",
                   clusters=4096, std=0.25, zipf=None,
                   note="stand-in for 96-d CNN descriptors; HBM-streaming scale"),
}


def scaled_down(w: Workload, n: int | None = None, m: int | None = None) -> Workload:
    """Same recipe with fewer rows / queries (for tests that need a small instance)."""
    return Workload(w.name, n or w.n, w.d, m or w.m, w.bits, w.ks, w.kind, w.seed,
                    w.clusters, w.std, w.zipf, w.note)


def _centres(w: Workload):
    rng = np.random.default_rng([w.seed, 2, 0])
    centres = rng.standard_normal((w.clusters, w.d), dtype=np.float32)
    if w.zipf is None:
        p = np.full(w.clusters, 1.0 / w.clusters)
    else:
        p = np.arange(1, w.clusters + 1, dtype=np.float64) ** (-w.zipf)
        p /= p.sum()
    return centres, np.cumsum(p)


def _block(w: Workload, stream: int, i: int, rows: int, mix) -> np.ndarray:
    rng = np.random.default_rng([w.seed, stream, i])
    if w.kind == "gauss":
        x = rng.standard_normal((rows, w.d), dtype=np.float32)
    elif w.kind == "absgauss":
        x = np.abs(rng.standard_normal((rows, w.d), dtype=np.float32))
    elif w.kind == "mixture":
        centres, cdf = mix
        which = np.minimum(np.searchsorted(cdf, rng.random(rows)), w.clusters - 1)
        x = centres[which] + np.float32(w.std) * rng.standard_normal((rows, w.d), dtype=np.float32)
    else:
        raise ValueError(w.kind)
    norm = np.sqrt((x * x).sum(axis=1, dtype=np.float32), dtype=np.float32)
    x /= np.maximum(norm, np.float32(1e-30))[:, None]
    return x


def rows(w: Workload, stream: int, start: int, stop: int) -> np.ndarray:
    """Rows [start, stop) of stream 0 (database) or 1 (queries), fp32 [stop-start, d]."""
    total = w.n if stream == 0 else w.m
    if not 0 <= start <= stop <= total:
        raise ValueError("row range outside the workload")
    mix = _centres(w) if w.kind == "mixture" else None
    out = np.empty((stop - start, w.d), dtype=np.float32)

    def fill(i):
        lo, hi = i * BLOCK, min((i + 1) * BLOCK, total)
        blk = _block(w, stream, i, hi - lo, mix)
        a, b = max(lo, start), min(hi, stop)
        if a < b:
            out[a - start:b - start] = blk[a - lo:b - lo]

    blocks = range(start // BLOCK, (max(stop, 1) - 1) // BLOCK + 1)
    if len(blocks) > 1:          # blocks are independent: generate them on a few threads
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            list(pool.map(fill, blocks))
    else:
        for i in blocks:
            fill(i)
    return out


def database(w: Workload, start: int = 0, stop: int | None = None) -> np.ndarray:
    return rows(w, 0, start, w.n if stop is None else stop)


def queries(w: Workload, start: int = 0, stop: int | None = None) -> np.ndarray:
    return rows(w, 1, start, w.m if stop is None else stop)


def choose_scale(db_head: np.ndarray, quantile: float = 0.98) -> float:
    """Scale parameter handed to both encoders: fp32(1 / q) with q the given quantile
    of |x| over the rows passed in (callers pass the first min(n, 100000) database
    rows).  quantile=1.0 is the conservative choice (largest component)."""
    a = np.abs(np.asarray(db_head, dtype=np.float64)).ravel()
    q = float(np.quantile(a, quantile)) if quantile < 1.0 else float(a.max())
    return float(np.float32(1.0 / q))


def workload_scale(w: Workload, quantile: float = 0.98) -> float:
    return choose_scale(database(w, 0, min(w.n, 100_000)), quantile)


def clustered_rows(n: int, d: int, m: int, clusters: int, spread: float, seed: int, ordered: bool):
    """Rows and queries of a Gaussian mixture whose rows lie cluster by cluster (ordered) or
    shuffled: real collections are often stored in an order that correlates with their content,
    the workloads above are not.  Returns (rows [n, d], queries [m, d]), L2-normalised fp32."""
    rng = np.random.default_rng([seed, 7])
    centres = rng.standard_normal((clusters, d)).astype(np.float32)
    label = rng.integers(clusters, size=n)
    if ordered:
        label = np.sort(label)
    X = centres[label] + np.float32(spread) * rng.standard_normal((n, d), dtype=np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    Q = centres[rng.integers(clusters, size=m)] + np.float32(spread) * rng.standard_normal((m, d), dtype=np.float32)
    Q /= np.linalg.norm(Q, axis=1, keepdims=True)
    return X.astype(np.float32), Q.astype(np.float32)
