"""Seeded synthetic workloads shaped like the paper's evaluation data (Section 5.1).

This module only *draws inputs*: clustered vectors, Zipf-distributed label sets
and labelled queries.  It holds none of the search method's arithmetic and is
the one module that both the HIP path's tests and the CPU oracle's tests feed
from.  The public datasets of Section 5.1 (SIFT-1M with Zipf labels, YFCC-10M,
WIKI-ANN, DEEP-50M) are not available offline; the presets below stand in for
them with the same dimensionality, label-vocabulary size, labels-per-point and
long-tailed label-frequency structure (Figure "specificity").

Everything is a pure function of (spec, seed): numpy ``Generator(PCG64)`` with
``SeedSequence(seed).spawn(5)`` used in the fixed order
(centres, cluster assignment, noise, labels, queries).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

__all__ = ["WorkloadSpec", "Workload", "PRESETS", "make_workload", "make_and_pairs_by_selectivity"]


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    n: int                      # number of data vectors
    dim: int
    dtype: str                  # "uint8" | "float32"
    n_clusters: int
    centre: tuple               # ("uniform", lo, hi) | ("normal", mean, std)
    noise_std: float
    n_labels: int               # label vocabulary size
    label_count: tuple          # ("uniform", lo, hi) | ("geometric", mean)
    zipf_alpha: float
    T: int                      # specificity threshold (posting-list size)
    graph_degree: int
    nq: int
    query_mode: str             # "single" | "mixed" (70% single / 30% 2-label AND) | "and2"
    k: int = 10
    itopk: int = 32
    width: int = 1
    iters: int = 20
    seed: int = 0


PRESETS = {
    # parity configuration: small enough for the oracle to build every graph
    "tiny": WorkloadSpec("tiny", 10_000, 128, "uint8", 32, ("uniform", 0.0, 255.0), 20.0,
                         100, ("uniform", 1, 3), 1.0, 500, 16, 1_000, "single",
                         k=10, itopk=32, width=1, iters=20),
    # SIFT-1M-like: the configuration the throughput metric is quoted on
    "c2": WorkloadSpec("c2", 1_000_000, 128, "float32", 1024, ("normal", 0.0, 2.0), 1.0,
                       1_000, ("uniform", 1, 5), 1.1, 10_000, 32, 10_000, "single",
                       k=10, itopk=64, width=1, iters=32),
    # YFCC-10M-like (CLIP-embedding-like uint8, 200k labels, long tail)
    "c3": WorkloadSpec("c3", 10_000_000, 192, "uint8", 4096, ("normal", 128.0, 30.0), 30.0,
                       200_000, ("geometric", 10.0), 1.3, 2_000, 32, 100_000, "mixed",
                       k=10, itopk=64, width=1, iters=32),
    # DEEP-like multi-label stress, all queries 2-label AND
    "c5": WorkloadSpec("c5", 5_000_000, 96, "float32", 2048, ("normal", 0.0, 1.0), 1.0,
                       10_000, ("uniform", 1, 8), 1.0, 5_000, 32, 100_000, "and2",
                       k=10, itopk=64, width=1, iters=32),
}


@dataclass
class Workload:
    spec: WorkloadSpec
    vectors: np.ndarray         # [n, dim], spec.dtype, C-contiguous
    label_offsets: np.ndarray   # int64 [n+1]  CSR over label_ids (raw draws: duplicates possible)
    label_ids: np.ndarray       # int32
    queries: np.ndarray         # [nq, dim], spec.dtype
    qlabel_offsets: np.ndarray  # int64 [nq+1]
    qlabel_ids: np.ndarray      # int32

    def point_labels(self, i: int) -> np.ndarray:
        return np.unique(self.label_ids[self.label_offsets[i]:self.label_offsets[i + 1]])

    def query_labels(self, j: int) -> np.ndarray:
        return np.unique(self.qlabel_ids[self.qlabel_offsets[j]:self.qlabel_offsets[j + 1]])


def _zipf_cdf(n_labels: int, alpha: float) -> np.ndarray:
    w = np.arange(1, n_labels + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    cdf[-1] = 1.0
    return cdf


def _draw_zipf(rng: np.random.Generator, cdf: np.ndarray, count: int) -> np.ndarray:
    out = np.empty(count, dtype=np.int32)
    step = 1 << 24
    for s in range(0, count, step):
        u = rng.random(min(step, count - s))
        out[s:s + len(u)] = np.searchsorted(cdf, u, side="right").astype(np.int32)
    np.minimum(out, len(cdf) - 1, out=out)
    return out


def _centres(rng: np.random.Generator, spec: WorkloadSpec) -> np.ndarray:
    kind = spec.centre[0]
    if kind == "uniform":
        return rng.uniform(spec.centre[1], spec.centre[2], size=(spec.n_clusters, spec.dim)).astype(np.float32)
    if kind == "normal":
        c = rng.standard_normal((spec.n_clusters, spec.dim), dtype=np.float32)
        return (c * np.float32(spec.centre[2]) + np.float32(spec.centre[1])).astype(np.float32)
    raise ValueError(kind)


def _sample_points(rng_assign, rng_noise, centres, count, spec) -> np.ndarray:
    out = np.empty((count, spec.dim), dtype=np.uint8 if spec.dtype == "uint8" else np.float32)
    assign = rng_assign.integers(0, spec.n_clusters, size=count)
    step = max(1, (1 << 26) // spec.dim)
    for s in range(0, count, step):
        e = min(count, s + step)
        x = rng_noise.standard_normal((e - s, spec.dim), dtype=np.float32)
        x *= np.float32(spec.noise_std)
        x += centres[assign[s:e]]
        if spec.dtype == "uint8":
            np.rint(x, out=x)
            np.clip(x, 0.0, 255.0, out=x)
            out[s:e] = x.astype(np.uint8)
        else:
            out[s:e] = x
    return out


def _label_counts(rng, spec: WorkloadSpec) -> np.ndarray:
    kind = spec.label_count[0]
    if kind == "uniform":
        return rng.integers(spec.label_count[1], spec.label_count[2] + 1, size=spec.n).astype(np.int64)
    if kind == "geometric":
        return rng.geometric(1.0 / spec.label_count[1], size=spec.n).astype(np.int64)
    raise ValueError(kind)


def _dedupe_csr(offsets: np.ndarray, ids: np.ndarray):
    """Sorted, duplicate-free copy of a CSR label table (used only to sample AND pairs)."""
    n = len(offsets) - 1
    owner = np.repeat(np.arange(n, dtype=np.int64), np.diff(offsets))
    key = owner * (int(ids.max()) + 1 if len(ids) else 1) + ids
    key = np.unique(key)
    vmax = int(ids.max()) + 1 if len(ids) else 1
    o = key // vmax
    l = (key % vmax).astype(np.int32)
    off = np.zeros(n + 1, dtype=np.int64)
    np.add.at(off, o + 1, 1)
    return np.cumsum(off), l


def _pairs_from_points(rng, off_u, ids_u, count):
    """2-label AND pairs taken from random data points carrying >= 2 labels, so
    that every pair has a non-empty intersection."""
    sizes = np.diff(off_u)
    cand = np.flatnonzero(sizes >= 2)
    if len(cand) == 0:
        raise ValueError("no data point has two labels")
    pts = cand[rng.integers(0, len(cand), size=count)]
    a = np.empty(count, dtype=np.int32)
    b = np.empty(count, dtype=np.int32)
    r1 = rng.random(count)
    r2 = rng.random(count)
    s = sizes[pts]
    i1 = np.minimum((r1 * s).astype(np.int64), s - 1)
    i2 = np.minimum((r2 * (s - 1)).astype(np.int64), s - 2)
    i2 = i2 + (i2 >= i1)
    a[:] = ids_u[off_u[pts] + i1]
    b[:] = ids_u[off_u[pts] + i2]
    return a, b


def make_and_pairs_by_selectivity(rng, off_u, ids_u, n, count, lo=1e-5, hi=1e-1, pool=20_000):
    """2-label pairs whose intersection selectivity |C_a ∩ C_b| / n is spread
    log-uniformly over [lo, hi]: candidate pairs are bucketed by decade of the
    measured intersection size and decades are sampled uniformly."""
    a, b = _pairs_from_points(rng, off_u, ids_u, pool)
    pair = np.unique(np.stack([np.minimum(a, b), np.maximum(a, b)], axis=1), axis=0)
    owner = np.repeat(np.arange(len(off_u) - 1, dtype=np.int64), np.diff(off_u))
    order = np.argsort(ids_u, kind="stable")
    lab_sorted = ids_u[order]
    own_sorted = owner[order]
    starts = np.searchsorted(lab_sorted, np.arange(int(ids_u.max()) + 2))
    sel = np.empty(len(pair))
    for i, (x, y) in enumerate(pair):
        cx = own_sorted[starts[x]:starts[x + 1]]
        cy = own_sorted[starts[y]:starts[y + 1]]
        sel[i] = len(np.intersect1d(cx, cy, assume_unique=True)) / n
    dec = np.floor(np.log10(np.maximum(sel, 1e-300))).astype(int)
    lo_d, hi_d = int(np.floor(np.log10(lo))), int(np.ceil(np.log10(hi))) - 1
    buckets = [np.flatnonzero(dec == d) for d in range(lo_d, hi_d + 1)]
    buckets = [bk for bk in buckets if len(bk)]
    if not buckets:
        buckets = [np.arange(len(pair))]
    which = rng.integers(0, len(buckets), size=count)
    pick = np.empty(count, dtype=np.int64)
    for bi, bk in enumerate(buckets):
        m = which == bi
        pick[m] = bk[rng.integers(0, len(bk), size=int(m.sum()))]
    return pair[pick, 0].astype(np.int32), pair[pick, 1].astype(np.int32)


def make_workload(spec_or_name, *, n: Optional[int] = None, nq: Optional[int] = None,
                  T: Optional[int] = None, seed: Optional[int] = None, **overrides) -> Workload:
    """Draw a workload.  ``n``/``nq``/``T``/``seed`` and any other spec field can be
    overridden to obtain reduced-size versions of a preset with the same structure."""
    spec = PRESETS[spec_or_name] if isinstance(spec_or_name, str) else spec_or_name
    changes = {k: v for k, v in dict(n=n, nq=nq, T=T, seed=seed).items() if v is not None}
    changes.update(overrides)
    if changes:
        spec = replace(spec, **changes)
    ss = np.random.SeedSequence(spec.seed).spawn(5)
    rng_c, rng_a, rng_n, rng_l, rng_q = (np.random.Generator(np.random.PCG64(s)) for s in ss)

    centres = _centres(rng_c, spec)
    vectors = _sample_points(rng_a, rng_n, centres, spec.n, spec)

    counts = _label_counts(rng_l, spec)
    label_offsets = np.zeros(spec.n + 1, dtype=np.int64)
    np.cumsum(counts, out=label_offsets[1:])
    cdf = _zipf_cdf(spec.n_labels, spec.zipf_alpha)
    label_ids = _draw_zipf(rng_l, cdf, int(label_offsets[-1]))

    # queries: fresh samples of the same mixture (not data points)
    q_assign = np.random.Generator(np.random.PCG64(ss[4].spawn(1)[0]))
    queries = _sample_points(q_assign, rng_q, centres, spec.nq, spec)
    if spec.query_mode == "single":
        qlabel_ids = _draw_zipf(rng_q, cdf, spec.nq)
        qlabel_offsets = np.arange(spec.nq + 1, dtype=np.int64)
    else:
        off_u, ids_u = _dedupe_csr(label_offsets, label_ids)
        if spec.query_mode == "mixed":
            two = rng_q.random(spec.nq) < 0.30
            single = _draw_zipf(rng_q, cdf, spec.nq)
            a, b = _pairs_from_points(rng_q, off_u, ids_u, spec.nq)
        elif spec.query_mode == "and2":
            two = np.ones(spec.nq, dtype=bool)
            single = np.zeros(spec.nq, dtype=np.int32)
            a, b = make_and_pairs_by_selectivity(rng_q, off_u, ids_u, spec.n, spec.nq)
        else:
            raise ValueError(spec.query_mode)
        cnt = np.where(two, 2, 1).astype(np.int64)
        qlabel_offsets = np.zeros(spec.nq + 1, dtype=np.int64)
        np.cumsum(cnt, out=qlabel_offsets[1:])
        qlabel_ids = np.empty(int(qlabel_offsets[-1]), dtype=np.int32)
        first = qlabel_offsets[:-1]
        qlabel_ids[first] = np.where(two, a, single)
        qlabel_ids[first[two] + 1] = b[two]
    return Workload(spec, np.ascontiguousarray(vectors), label_offsets, label_ids,
                    np.ascontiguousarray(queries), qlabel_offsets, qlabel_ids)
