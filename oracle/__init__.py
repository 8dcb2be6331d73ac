"""ctypes wrapper around the CPU oracle (``vf_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the HIP package, and the HIP
package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vf_oracle.c")
_LIB = os.path.join(_HERE, "libvf_oracle.so")

_DT = {"uint8": 0, "float32": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE fp32: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def default_threads() -> int:
    """Threads the oracle runs its query loop on: the machine's own limit (OMP_NUM_THREADS) when it sets one,
    else every core the interpreter sees."""
    seen = os.cpu_count() or 1
    try:
        limit = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    except ValueError:
        limit = 0
    return min(seen, limit) if limit > 0 else seen


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.vfo_build.restype = p
        L.vfo_build.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, C.c_int, C.c_int]
        L.vfo_free.argtypes = [p]
        L.vfo_search.restype = C.c_int
        L.vfo_search.argtypes = [p, p, i64, p, p, i32, i32, i32, i32, i32, i64, C.c_int, p, p, p, p, p, C.c_int]
        L.vfo_search_routed.restype = C.c_int
        L.vfo_search_routed.argtypes = [p, p, i64, p, p, i32, i32, i32, i32, i32, i64, C.c_int, i64, p, p, p, p, p, C.c_int]
        L.vfo_search_multi.argtypes = [p, p, i64, p, p, C.c_int, i32, i32, i32, i32, i32, C.c_int, p, p, p, C.c_int]
        L.vfo_search_multi.restype = C.c_int
        for name in ("vfo_n_HS", "vfo_n_LS"):
            getattr(L, name).restype = i64
            getattr(L, name).argtypes = [p]
        for name in ("vfo_S", "vfo_O_HS", "vfo_O_LS", "vfo_M_HS", "vfo_M_LS", "vfo_G_HS"):
            getattr(L, name).restype = p
            getattr(L, name).argtypes = [p]
        L.vfo_graph_row.restype = C.c_int
        L.vfo_graph_row.argtypes = [p, i32, i64, p]
        L.vfo_build_pruned.restype = p
        L.vfo_build_pruned.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, i32, C.c_int]
        L.vfo_pruned_row.restype = C.c_int
        L.vfo_pruned_row.argtypes = [p, i32, i64, i32, p]
        L.vfo_dist_f32_ordered.restype = C.c_float
        L.vfo_dist_f32_ordered.argtypes = [p, p, i32]
        L.vfo_dist_u8.restype = i32
        L.vfo_dist_u8.argtypes = [p, p, i32]
        L.vfo_dist_f64.restype = C.c_double
        L.vfo_dist_f64.argtypes = [p, p, i32]
        L.vfo_predicate.restype = C.c_int
        L.vfo_predicate.argtypes = [p, i64, p, i32, p]
        L.vfo_store_interleaved.argtypes = [p, i64, i32, i32, p]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _view(addr, n, dtype):
    if n == 0:
        return np.empty(0, dtype=dtype)
    buf = (C.c_char * (n * np.dtype(dtype).itemsize)).from_address(addr)
    return np.frombuffer(buf, dtype=dtype).copy()


class OracleIndex:
    """Dual-structured label-centric index (Alg. 1) built on the CPU."""

    def __init__(self, vectors, label_offsets, label_ids, n_labels, T, graph_degree, lazy_graph=False, n_threads=0,
                 knn_degree=0):
        """knn_degree = D > 0: the graphs are built with degree D and reduced to graph_degree by rank-based
        pruning and reverse edges (vfo_build_pruned); 0: the exact graph_degree-nearest-neighbour graphs."""
        self.vectors = np.ascontiguousarray(vectors)
        self.dtype = str(self.vectors.dtype)
        self.n, self.dim = self.vectors.shape
        self.label_offsets = np.ascontiguousarray(label_offsets, dtype=np.int64)
        self.label_ids = np.ascontiguousarray(label_ids, dtype=np.int32)
        self.n_labels, self.T, self.R = int(n_labels), int(T), int(graph_degree)
        self.n_threads = n_threads or default_threads()
        self.knn_degree = int(knn_degree)
        if self.knn_degree > 0:
            if lazy_graph:
                raise ValueError("a pruned graph cannot be built row by row (reverse edges need every row)")
            self._h = lib().vfo_build_pruned(_ptr(self.vectors), _DT[self.dtype], self.n, self.dim,
                                             _ptr(self.label_offsets), _ptr(self.label_ids), self.n_labels, self.T,
                                             self.R, self.knn_degree, self.n_threads)
        else:
            self._h = lib().vfo_build(_ptr(self.vectors), _DT[self.dtype], self.n, self.dim, _ptr(self.label_offsets),
                                      _ptr(self.label_ids), self.n_labels, self.T, self.R, int(lazy_graph),
                                      self.n_threads)
        if not self._h:
            raise ValueError("vfo_build rejected its arguments")
        self.lazy = bool(lazy_graph)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().vfo_free(self._h)
            self._h = None

    # exported arrays (names follow Alg. 1)
    @property
    def n_HS(self):
        return lib().vfo_n_HS(self._h)

    @property
    def n_LS(self):
        return lib().vfo_n_LS(self._h)

    @property
    def S(self):
        return _view(lib().vfo_S(self._h), self.n_labels, np.int64)

    @property
    def O_HS(self):
        return _view(lib().vfo_O_HS(self._h), self.n_labels, np.int64)

    @property
    def O_LS(self):
        return _view(lib().vfo_O_LS(self._h), self.n_labels, np.int64)

    @property
    def M_HS(self):
        return _view(lib().vfo_M_HS(self._h), self.n_HS, np.int32)

    @property
    def M_LS(self):
        return _view(lib().vfo_M_LS(self._h), self.n_LS, np.int32)

    @property
    def G_HS(self):
        if self.lazy:
            raise RuntimeError("lazy index: use graph_row()")
        return _view(lib().vfo_G_HS(self._h), self.n_HS * self.R, np.int32).reshape(-1, self.R)

    def pruned_row(self, label, j, knn_degree):
        """Forward row (pruning step only) of one vertex, from brute-force degree-D rows of it and its neighbours."""
        row = np.empty(self.R, dtype=np.int32)
        if lib().vfo_pruned_row(self._h, int(label), int(j), int(knn_degree), _ptr(row)) != 0:
            raise IndexError((label, j))
        return row

    def graph_row(self, label, j):
        row = np.empty(self.R, dtype=np.int32)
        if lib().vfo_graph_row(self._h, int(label), int(j), _ptr(row)) != 0:
            raise IndexError((label, j))
        return row

    def search(self, queries, qlabel_offsets, qlabel_ids, k, itopk=32, width=1, iters=20, n_seeds=0,
               visited_cap=0, force_scan=False, n_threads=None, with_info=False, and_scan_limit=0):
        queries = np.ascontiguousarray(queries)
        assert str(queries.dtype) == self.dtype and queries.shape[1] == self.dim
        nq = queries.shape[0]
        qoff = np.ascontiguousarray(qlabel_offsets, dtype=np.int64)
        qids = np.ascontiguousarray(qlabel_ids, dtype=np.int32)
        ids = np.empty((nq, k), dtype=np.int64)
        dists = np.empty((nq, k), dtype=np.float32)
        method = np.empty(nq, dtype=np.int32)
        route = np.empty(nq, dtype=np.int32)
        counters = np.zeros((nq, 3), dtype=np.int64)
        rc = lib().vfo_search_routed(self._h, _ptr(queries), nq, _ptr(qoff), _ptr(qids), k, itopk, width, iters, n_seeds,
                                     visited_cap, int(force_scan), int(and_scan_limit), _ptr(ids), _ptr(dists),
                                     _ptr(method), _ptr(route), _ptr(counters),
                                     self.n_threads if n_threads is None else n_threads)
        if rc != 0:
            raise ValueError("vfo_search rejected its arguments")
        if with_info:
            return ids, dists, dict(method=method, route_label=route, counters=counters)
        return ids, dists


AND_PARALLEL, OR = 1, 2


def _search_multi(self, queries, qlabel_offsets, qlabel_ids, mode, k, itopk=32, width=1, iters=20, n_seeds=0,
                  force_scan=False, n_threads=None, with_info=False):
    """Multi-label queries through several single-list searches and a merge: OR (Section 4.3.1)
    and the parallel AND policy (Section 4.3.2)."""
    queries = np.ascontiguousarray(queries)
    assert str(queries.dtype) == self.dtype and queries.shape[1] == self.dim
    nq = queries.shape[0]
    qoff = np.ascontiguousarray(qlabel_offsets, dtype=np.int64)
    qids = np.ascontiguousarray(qlabel_ids, dtype=np.int32)
    ids = np.empty((nq, k), dtype=np.int64)
    dists = np.empty((nq, k), dtype=np.float32)
    ns = np.zeros(nq, dtype=np.int32)
    rc = lib().vfo_search_multi(self._h, _ptr(queries), nq, _ptr(qoff), _ptr(qids), int(mode), k, itopk, width, iters,
                                n_seeds, int(force_scan), _ptr(ids), _ptr(dists), _ptr(ns),
                                self.n_threads if n_threads is None else n_threads)
    if rc != 0:
        raise ValueError("vfo_search_multi rejected its arguments")
    if with_info:
        return ids, dists, dict(n_searches=ns)
    return ids, dists


OracleIndex.search_multi = _search_multi


def dist_f32_ordered(q, x):
    q = np.ascontiguousarray(q, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    return float(lib().vfo_dist_f32_ordered(_ptr(q), _ptr(x), q.shape[0]))


def dist_u8(q, x):
    q = np.ascontiguousarray(q, dtype=np.uint8)
    x = np.ascontiguousarray(x, dtype=np.uint8)
    return int(lib().vfo_dist_u8(_ptr(q), _ptr(x), q.shape[0]))


def predicate(point_labels, query_labels):
    """Section 4.3.2 predicate on sorted arrays; returns (found_all, positions)."""
    pl = np.ascontiguousarray(point_labels, dtype=np.int32)
    ql = np.ascontiguousarray(query_labels, dtype=np.int32)
    pos = np.full(len(ql), -1, dtype=np.int64)
    ok = lib().vfo_predicate(_ptr(pl), len(pl), _ptr(ql), len(ql), _ptr(pos))
    return bool(ok), pos


def store_interleaved(vectors):
    """Section 4.2.2 layout: groups of 32 vectors, 16-byte chunks interleaved."""
    v = np.ascontiguousarray(vectors)
    n, dim = v.shape
    es = v.dtype.itemsize
    veclen = 16 // es
    n_chunks = -(-dim // veclen)
    out = np.empty(-(-n // 32) * 32 * n_chunks * veclen, dtype=v.dtype)
    lib().vfo_store_interleaved(_ptr(v), n, dim, es, _ptr(out))
    return out
