"""Thin Python binding of the C ABI in ``include/vecflow.h``.

Argument marshalling only: every step of the search path runs in the HIP
library.  PyTorch supplies device memory (tensors) and the current HIP stream.
There is no CPU fallback: if ``libvecflow.so`` is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvecflow.so")

VF_U8, VF_F32 = 0, 1
ARR = dict(S=0, O_HS=1, O_LS=2, M_HS=3, M_LS=4, G_HS=5, GO_LS=6, X_LS=7, BITSET=8)
_ARR_DTYPE = dict(S=np.int64, O_HS=np.int64, O_LS=np.int64, M_HS=np.int32, M_LS=np.int32, G_HS=np.int32,
                  GO_LS=np.int64, X_LS=np.uint8, BITSET=np.uint32)

EXPORTED_SYMBOLS = ("vf_build_index", "vf_search", "vf_search_exact", "vf_index_export", "vf_index_stats",
                    "vf_index_free", "vf_last_error", "vf_profile_enable", "vf_profile_read", "vf_search_multi",
                    "vf_build_index_opt")


class VfStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n", "n_HS", "n_LS", "n_groups_LS")] + \
               [(n, C.c_int32) for n in ("dim", "dtype", "n_labels", "T", "graph_degree", "n_graph_labels",
                                         "n_scan_labels", "chunks_per_vector")] + \
               [(n, C.c_int64) for n in ("bytes_graph", "bytes_maps", "bytes_x_ls", "bytes_bitsets", "bytes_meta",
                                         "bytes_total")]


class VfProfile(C.Structure):
    _fields_ = [("scan_ms", C.c_float), ("seed_ms", C.c_float), ("beam_ms", C.c_float), ("scan_ms_sum", C.c_double),
                ("seed_ms_sum", C.c_double), ("beam_ms_sum", C.c_double), ("calls", C.c_int64)] + \
               [(n, C.c_int64) for n in ("nq", "n_scan_queries", "n_graph_queries", "n_scan_items",
                                         "scan_list_entries", "scan_pairs", "beam_scored", "beam_expanded",
                                         "beam_tested", "n_seed_tiles", "seed_pairs", "seed_tile_seeds",
                                         "seeds_on_matrix_cores", "seed_rescored", "seed_fallbacks", "beam_gathered",
                                         "scan_kernel")]


class VecflowError(RuntimeError):
    pass


_lib = None


def load_library():
    """dlopen the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise VecflowError(f"{LIB_PATH} is missing: run `python -m paper_2506_00812_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.vf_build_index.restype = C.c_int
        L.vf_build_index.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, p, C.POINTER(p)]
        L.vf_build_index_opt.restype = C.c_int
        L.vf_build_index_opt.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, i32, i32, p, C.POINTER(p)]
        L.vf_search.restype = C.c_int
        L.vf_search.argtypes = [p, p, i64, p, p, i32, i32, i32, i32, i32, p, p, p]
        L.vf_search_exact.restype = C.c_int
        L.vf_search_exact.argtypes = [p, p, i64, p, p, i32, p, p, p]
        L.vf_index_export.restype = C.c_int
        L.vf_index_export.argtypes = [p, C.c_int, p, C.POINTER(C.c_size_t)]
        L.vf_index_stats.restype = C.c_int
        L.vf_index_stats.argtypes = [p, C.POINTER(VfStats)]
        L.vf_search_multi.restype = C.c_int
        L.vf_search_multi.argtypes = [p, p, C.c_int64, p, p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, p, p, p]
        L.vf_profile_enable.restype = C.c_int
        L.vf_profile_enable.argtypes = [p, C.c_int]
        L.vf_profile_read.restype = C.c_int
        L.vf_profile_read.argtypes = [p, C.POINTER(VfProfile), p]
        L.vf_index_free.restype = None
        L.vf_index_free.argtypes = [p]
        L.vf_last_error.restype = C.c_char_p
        L.vf_last_error.argtypes = []
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise VecflowError(f"vecflow error {rc}: {load_library().vf_last_error().decode()}")


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _stream_handle(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.uint8:
        return VF_U8
    if t.dtype == torch.float32:
        return VF_F32
    raise VecflowError(f"unsupported dtype {t.dtype}")


class Index:
    """Handle of a built index.  Keeps the vector tensor alive (the library references it)."""

    def __init__(self, handle, vectors):
        self._h = handle
        self.vectors = vectors
        self._free = load_library().vf_index_free  # bound here: module globals may be gone at interpreter exit

    def __del__(self):
        self.free()

    def free(self):
        if getattr(self, "_h", None):
            self._free(self._h)
            self._h = None

    def stats(self) -> dict:
        st = VfStats()
        _check(load_library().vf_index_stats(self._h, C.byref(st)))
        return {n: getattr(st, n) for n, _ in VfStats._fields_}

    def profile_enable(self, on=True, serial: bool = False):
        """serial=True also runs the IVF-BFS and IVF-Graph launches one after the other."""
        _check(load_library().vf_profile_enable(self._h, 2 if (on and serial) else int(bool(on))))

    def profile_read(self, per_query: bool = False):
        """Durations and work counters of the last profiled search; waits for it."""
        pf = VfProfile()
        L = load_library()
        if per_query:
            # nq is only known after a first read
            _check(L.vf_profile_read(self._h, C.byref(pf), None))
            cn = np.zeros((pf.nq, 4), dtype=np.int32)
            _check(L.vf_profile_read(self._h, C.byref(pf), _np_ptr(cn)))
        else:
            cn = None
            _check(L.vf_profile_read(self._h, C.byref(pf), None))
        out = {n: getattr(pf, n) for n, _ in VfProfile._fields_}
        return (out, cn) if per_query else out

    def export(self, name: str) -> np.ndarray:
        L = load_library()
        nbytes = C.c_size_t(0)
        _check(L.vf_index_export(self._h, ARR[name], None, C.byref(nbytes)))
        dt = np.dtype(_ARR_DTYPE[name])
        out = np.empty(nbytes.value // dt.itemsize, dtype=dt)
        if nbytes.value:
            _check(L.vf_index_export(self._h, ARR[name], _np_ptr(out), C.byref(nbytes)))
        return out


GRAPH_KNN, GRAPH_PRUNED = 0, 1


def build_index(vectors, label_offsets, label_ids, n_labels, T, graph_degree, stream=None, graph_kind=GRAPH_KNN,
                knn_degree=0) -> Index:
    """vectors: CUDA tensor [n, dim] uint8/float32 (contiguous); labels: host CSR arrays.
    graph_kind=GRAPH_PRUNED: graphs of degree knn_degree (0 = the default) reduced to graph_degree by
    rank-based pruning and reverse edges (vf_build_index_opt)."""
    L = load_library()
    if not vectors.is_cuda or not vectors.is_contiguous() or vectors.dim() != 2:
        raise VecflowError("vectors must be a contiguous 2-D CUDA tensor")
    off = np.ascontiguousarray(label_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(label_ids, dtype=np.int32)
    if off.shape[0] != vectors.shape[0] + 1:
        raise VecflowError("label_offsets must have n + 1 entries")
    h = C.c_void_p()
    if graph_kind == GRAPH_KNN and knn_degree == 0:
        _check(L.vf_build_index(C.c_void_p(vectors.data_ptr()), _dtype_code(vectors), vectors.shape[0],
                                vectors.shape[1], _np_ptr(off), _np_ptr(ids), int(n_labels), int(T), int(graph_degree),
                                _stream_handle(stream), C.byref(h)))
    else:
        _check(L.vf_build_index_opt(C.c_void_p(vectors.data_ptr()), _dtype_code(vectors), vectors.shape[0],
                                    vectors.shape[1], _np_ptr(off), _np_ptr(ids), int(n_labels), int(T),
                                    int(graph_degree), int(graph_kind), int(knn_degree), _stream_handle(stream),
                                    C.byref(h)))
    return Index(h, vectors)


def _prep_queries(index, queries, qlabel_offsets, qlabel_ids):
    if not queries.is_cuda or not queries.is_contiguous() or queries.dim() != 2:
        raise VecflowError("queries must be a contiguous 2-D CUDA tensor")
    if queries.dtype != index.vectors.dtype or queries.shape[1] != index.vectors.shape[1]:
        raise VecflowError("queries must match the index dtype and dim")
    off = np.ascontiguousarray(qlabel_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(qlabel_ids, dtype=np.int32)
    if off.shape[0] != queries.shape[0] + 1:
        raise VecflowError("qlabel_offsets must have nq + 1 entries")
    return off, ids


def search(index: Index, queries, qlabel_offsets, qlabel_ids, k, itopk=64, width=1, iters=32, n_seeds=0,
           out_ids=None, out_dists=None, stream=None):
    """Asynchronous on the (current) stream; returns (ids int64 [nq,k], dists float32 [nq,k]) CUDA tensors."""
    import torch
    off, ids = _prep_queries(index, queries, qlabel_offsets, qlabel_ids)
    nq = queries.shape[0]
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
    if out_dists is None:
        out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    _check(load_library().vf_search(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids), int(k),
                                    int(itopk), int(width), int(iters), int(n_seeds),
                                    C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                    _stream_handle(stream)))
    return out_ids, out_dists


AND_GREEDY, AND_PARALLEL, OR = 0, 1, 2
MULTI_EXACT = 0x100


def search_multi(index: Index, queries, qlabel_offsets, qlabel_ids, mode, k, itopk=64, width=1, iters=32, n_seeds=0,
                 out_ids=None, out_dists=None, stream=None):
    """OR queries and the parallel AND policy: one search per query label, merged.  Asynchronous."""
    import torch
    off, ids = _prep_queries(index, queries, qlabel_offsets, qlabel_ids)
    nq = queries.shape[0]
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
    if out_dists is None:
        out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    _check(load_library().vf_search_multi(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids),
                                          int(mode), int(k), int(itopk), int(width), int(iters), int(n_seeds),
                                          C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                          _stream_handle(stream)))
    return out_ids, out_dists


def search_exact(index: Index, queries, qlabel_offsets, qlabel_ids, k, stream=None):
    """Exact filtered top-k (ground truth).  Synchronises the stream."""
    import torch
    off, ids = _prep_queries(index, queries, qlabel_offsets, qlabel_ids)
    nq = queries.shape[0]
    out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
    out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    _check(load_library().vf_search_exact(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids),
                                          int(k), C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                          _stream_handle(stream)))
    return out_ids, out_dists
