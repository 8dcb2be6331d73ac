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
                    "vf_build_index_opt", "vf_tune", "vf_debug_route", "vf_search_noalloc", "vf_serve_begin", "vf_serve_submit",
                    "vf_serve_poll", "vf_serve_end", "vf_serve_run", "vf_search_ex")

ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class VfAllocator(C.Structure):
    _fields_ = [("alloc", ALLOC_FN), ("free", FREE_FN), ("ctx", C.c_void_p)]


class VfStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n", "n_HS", "n_LS", "n_groups_LS")] + \
               [(n, C.c_int32) for n in ("dim", "dtype", "n_labels", "T", "graph_degree", "n_graph_labels",
                                         "n_scan_labels", "chunks_per_vector")] + \
               [(n, C.c_int64) for n in ("bytes_graph", "bytes_maps", "bytes_x_ls", "bytes_bitsets", "bytes_meta",
                                         "bytes_total", "bytes_x_ls_bf16")]


class VfProfile(C.Structure):
    _fields_ = [("scan_ms", C.c_float), ("seed_ms", C.c_float), ("beam_ms", C.c_float), ("scan_ms_sum", C.c_double),
                ("seed_ms_sum", C.c_double), ("beam_ms_sum", C.c_double), ("calls", C.c_int64)] + \
               [(n, C.c_int64) for n in ("nq", "n_scan_queries", "n_graph_queries", "n_scan_items",
                                         "scan_list_entries", "scan_pairs", "beam_scored", "beam_expanded",
                                         "beam_tested", "n_seed_tiles", "seed_pairs", "seed_tile_seeds",
                                         "seeds_on_matrix_cores", "seed_rescored", "seed_fallbacks", "beam_gathered",
                                         "scan_kernel", "seed_selected", "seed_run_keys", "scan_fallbacks")] + \
               [(n, C.c_double) for n in ("host_plan_ms_sum", "host_blob_ms_sum", "host_launch_ms_sum", "host_wait_ms_sum")]


class VfSearchParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k", "itopk", "width", "iters", "n_seeds", "and_scan_limit")] + \
               [("reserved", C.c_int32 * 2)]


class VfServeParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k", "itopk", "width", "iters", "n_seeds", "n_workers", "ring_slots", "waves_per_worker")] + \
               [(n, C.c_int64) for n in ("max_jobs", "idle_polls")]


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
        L.vf_build_index.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, C.POINTER(VfAllocator), p, C.POINTER(p)]
        L.vf_build_index_opt.restype = C.c_int
        L.vf_build_index_opt.argtypes = [p, C.c_int, i64, i32, p, p, i32, i32, i32, i32, i32, C.POINTER(VfAllocator), p,
                                         C.POINTER(p)]
        L.vf_tune.restype = C.c_int
        L.vf_tune.argtypes = [p, C.c_char_p, C.c_double]
        L.vf_debug_route.restype = C.c_int
        L.vf_debug_route.argtypes = [p, i32, i32, i64, p, p, i32, i32, p, p, p, p, i64, p, i64, p, p]
        L.vf_search.restype = C.c_int
        L.vf_search.argtypes = [p, p, i64, p, p, i32, i32, i32, i32, i32, p, p, p]
        L.vf_search_noalloc.restype = C.c_int
        L.vf_search_noalloc.argtypes = [p, p, i64, p, p, i32, i32, i32, i32, i32, p, p, p]
        L.vf_serve_begin.restype = C.c_int
        L.vf_serve_begin.argtypes = [p, C.POINTER(VfServeParams), C.POINTER(p)]
        L.vf_serve_submit.restype = C.c_int
        L.vf_serve_submit.argtypes = [p, p, p, i32, C.POINTER(i64)]
        L.vf_serve_poll.restype = C.c_int
        L.vf_serve_poll.argtypes = [p, i64, p, p, C.POINTER(i32)]
        L.vf_serve_end.restype = C.c_int
        L.vf_serve_end.argtypes = [p, C.POINTER(i64), C.POINTER(i32)]
        L.vf_serve_run.restype = C.c_int
        L.vf_serve_run.argtypes = [p, p, i64, p, p, i32, p, p, p]
        L.vf_search_ex.restype = C.c_int
        L.vf_search_ex.argtypes = [p, p, i64, p, p, C.POINTER(VfSearchParams), p, p, p]
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


class TorchAllocator:
    """vf_allocator backed by PyTorch's caching allocator: the index and its workspaces then live in memory that
    torch accounts for and reuses.  Blocks are requested on the stream of the call in progress (the binding sets
    it before every library call); the library frees a block only after the work that used it has completed."""

    def __init__(self, device):
        import torch
        self._torch = torch
        self.device = device
        self.stream = 0
        self.live = {}            # address -> bytes
        self.n_alloc = self.n_free = 0

        def _alloc(nbytes, _ctx):
            try:
                ptr = torch.cuda.caching_allocator_alloc(int(nbytes), device=self.device, stream=self.stream)
            except Exception:      # out of memory: the library reports VF_ENOMEM
                return None
            self.live[ptr] = int(nbytes)
            self.n_alloc += 1
            return ptr

        def _free(ptr, _ctx):
            try:
                if self.live.pop(ptr, None) is not None:
                    self.n_free += 1
                    torch.cuda.caching_allocator_delete(ptr)
            except Exception:      # interpreter shutdown: torch may be gone, the process is ending anyway
                pass

        self._alloc_cb, self._free_cb = ALLOC_FN(_alloc), FREE_FN(_free)   # kept alive with this object
        self.struct = VfAllocator(self._alloc_cb, self._free_cb, None)

    def live_bytes(self):
        return sum(self.live.values())


class Index:
    """Handle of a built index.  Keeps the vector tensor alive (the library references it)."""

    def __init__(self, handle, vectors, allocator=None):
        self._h = handle
        self.vectors = vectors
        self.allocator = allocator   # keeps the callbacks alive as long as the library may call them
        self._free = load_library().vf_index_free  # bound here: module globals may be gone at interpreter exit

    def _enter(self, stream=None):
        """Before a library call that may allocate: blocks come from the pool of the call's stream."""
        if self.allocator is not None:
            import torch
            s = stream if stream is not None else torch.cuda.current_stream()
            self.allocator.stream = s.cuda_stream

    def tune(self, name: str, value):
        """Experiment / test switch of this index (vf_tune)."""
        self._enter()
        _check(load_library().vf_tune(self._h, name.encode(), float(value)))

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

    def profile_enable(self, on=True, serial: bool = False, exact_counts: bool = False):
        """serial=True also runs the IVF-BFS and IVF-Graph launches one after the other; exact_counts=True has a
        small kernel count, before every call with AND queries, the seeds that pass each query's predicate."""
        mode = (2 if serial else 1) if on else 0
        _check(load_library().vf_profile_enable(self._h, mode | (4 if (on and exact_counts) else 0)))

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


def debug_route(S, T, qlabel_offsets, qlabel_ids, tile_rows=16, seg_groups=16):
    """Host-only routing and scan work list for posting-list sizes S (vf_debug_route); no device is touched."""
    L = load_library()
    S = np.ascontiguousarray(S, dtype=np.int32)
    off = np.ascontiguousarray(qlabel_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(qlabel_ids, dtype=np.int32)
    nq = len(off) - 1
    searched, method, n_others = (np.empty(nq, dtype=np.int32) for _ in range(3))
    counts = np.zeros(6, dtype=np.int64)
    args = [_np_ptr(S), len(S), int(T), nq, _np_ptr(off), _np_ptr(ids), int(tile_rows), int(seg_groups),
            _np_ptr(searched), _np_ptr(method), _np_ptr(n_others)]
    _check(L.vf_debug_route(*args, None, 0, None, 0, None, _np_ptr(counts)))      # sizes only
    items = np.zeros((max(int(counts[2]), 1), 8), dtype=np.int64)
    merges = np.zeros((max(int(counts[3]), 1), 5), dtype=np.int64)
    qrow = np.zeros(max(nq, 1), dtype=np.int32)
    _check(L.vf_debug_route(*args, _np_ptr(items), len(items), _np_ptr(merges), len(merges), _np_ptr(qrow),
                            _np_ptr(counts)))
    n_g, n_s, n_items, n_merges, part_rows, max_nseg = (int(c) for c in counts)
    return dict(searched=searched, method=method, n_others=n_others, items=items[:n_items], merges=merges[:n_merges],
                scan_rows=qrow[:n_s], graph_queries=qrow[n_s:n_s + n_g], part_rows=part_rows, max_nseg=max_nseg)


GRAPH_KNN, GRAPH_PRUNED = 0, 1


def tune_defaults(name: str, value):
    """Process-wide default of an experiment / test switch: indexes built afterwards start from it."""
    _check(load_library().vf_tune(None, name.encode(), float(value)))


def build_index(vectors, label_offsets, label_ids, n_labels, T, graph_degree, stream=None, graph_kind=GRAPH_KNN,
                knn_degree=0, torch_allocator=True) -> Index:
    """vectors: CUDA tensor [n, dim] uint8/float32 (contiguous); labels: host CSR arrays.
    graph_kind=GRAPH_PRUNED: graphs of degree knn_degree (0 = the default) reduced to graph_degree by
    rank-based pruning and reverse edges (vf_build_index_opt).
    torch_allocator: the index takes its device memory from PyTorch's caching allocator (False: hipMalloc)."""
    L = load_library()
    if not vectors.is_cuda or not vectors.is_contiguous() or vectors.dim() != 2:
        raise VecflowError("vectors must be a contiguous 2-D CUDA tensor")
    off = np.ascontiguousarray(label_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(label_ids, dtype=np.int32)
    if off.shape[0] != vectors.shape[0] + 1:
        raise VecflowError("label_offsets must have n + 1 entries")
    h = C.c_void_p()
    al = None
    if torch_allocator:
        import torch
        al = TorchAllocator(vectors.device)
        al.stream = (stream if stream is not None else torch.cuda.current_stream()).cuda_stream
    al_ref = C.byref(al.struct) if al is not None else None
    if graph_kind == GRAPH_KNN and knn_degree == 0:
        _check(L.vf_build_index(C.c_void_p(vectors.data_ptr()), _dtype_code(vectors), vectors.shape[0],
                                vectors.shape[1], _np_ptr(off), _np_ptr(ids), int(n_labels), int(T), int(graph_degree),
                                al_ref, _stream_handle(stream), C.byref(h)))
    else:
        _check(L.vf_build_index_opt(C.c_void_p(vectors.data_ptr()), _dtype_code(vectors), vectors.shape[0],
                                    vectors.shape[1], _np_ptr(off), _np_ptr(ids), int(n_labels), int(T),
                                    int(graph_degree), int(graph_kind), int(knn_degree), al_ref, _stream_handle(stream),
                                    C.byref(h)))
    return Index(h, vectors, al)


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
           out_ids=None, out_dists=None, stream=None, and_scan_limit=0):
    """Asynchronous on the (current) stream; returns (ids int64 [nq,k], dists float32 [nq,k]) CUDA tensors.
    and_scan_limit > 0: vf_search_ex with selectivity-aware routing of AND queries."""
    import torch
    off, ids = _prep_queries(index, queries, qlabel_offsets, qlabel_ids)
    nq = queries.shape[0]
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
    if out_dists is None:
        out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    index._enter(stream)
    if and_scan_limit:
        prm = VfSearchParams(int(k), int(itopk), int(width), int(iters), int(n_seeds), int(and_scan_limit))
        _check(load_library().vf_search_ex(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids),
                                           C.byref(prm), C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                           _stream_handle(stream)))
        return out_ids, out_dists
    _check(load_library().vf_search(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids), int(k),
                                    int(itopk), int(width), int(iters), int(n_seeds),
                                    C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                    _stream_handle(stream)))
    return out_ids, out_dists


def search_noalloc(index: Index, queries, qlabel_offsets, qlabel_ids, k, out_ids, out_dists, itopk=64, width=1,
                   iters=32, n_seeds=0, stream=None):
    """vf_search_noalloc: the same search with every temporary in the library's fixed scratch array; the caller
    passes the output tensors, nothing is allocated on the way.  Asynchronous on the (current) stream."""
    off, ids = _prep_queries(index, queries, qlabel_offsets, qlabel_ids)
    nq = queries.shape[0]
    if tuple(out_ids.shape) != (nq, k) or tuple(out_dists.shape) != (nq, k):
        raise VecflowError("out_ids / out_dists must be [nq, k]")
    _check(load_library().vf_search_noalloc(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids),
                                            int(k), int(itopk), int(width), int(iters), int(n_seeds),
                                            C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                            _stream_handle(stream)))
    return out_ids, out_dists


EBUSY = -5


class Server:
    """A serving session (vf_serve_*): a resident kernel that answers single queries from a job ring."""

    def __init__(self, index: Index, k, itopk=32, width=1, iters=8, n_seeds=0, n_workers=0, ring_slots=0, max_jobs=0,
                 idle_polls=0, waves_per_worker=0):
        self.index, self.k = index, int(k)
        prm = VfServeParams(int(k), int(itopk), int(width), int(iters), int(n_seeds), int(n_workers), int(ring_slots),
                            int(waves_per_worker), int(max_jobs), int(idle_polls))
        h = C.c_void_p()
        index._enter()
        _check(load_library().vf_serve_begin(index._h, C.byref(prm), C.byref(h)))
        self._h = h
        self._np_dtype = np.uint8 if _dtype_code(index.vectors) == VF_U8 else np.float32
        self.dim = index.vectors.shape[1]

    def submit(self, query, labels):
        """query: host array [dim]; labels: 1..8 ids.  Returns the job id, or None when the ring is full."""
        q = np.ascontiguousarray(query, dtype=self._np_dtype)
        if q.shape != (self.dim,):
            raise VecflowError("query must have dim elements")
        lab = np.ascontiguousarray(labels, dtype=np.int32).reshape(-1)
        job = C.c_int64(-1)
        rc = load_library().vf_serve_submit(self._h, _np_ptr(q), _np_ptr(lab), len(lab), C.byref(job))
        if rc == EBUSY:
            return None
        _check(rc)
        return job.value

    def poll(self, job):
        """(ids, dists) of a completed job, else None."""
        ids = np.empty(self.k, dtype=np.int64)
        d = np.empty(self.k, dtype=np.float32)
        done = C.c_int32(0)
        _check(load_library().vf_serve_poll(self._h, int(job), _np_ptr(ids), _np_ptr(d), C.byref(done)))
        return (ids, d) if done.value else None

    def run(self, queries, qlabel_offsets, qlabel_ids, in_flight=64):
        """A host batch through the session, one job per query (vf_serve_run): (ids, dists, latency_us)."""
        q = np.ascontiguousarray(queries, dtype=self._np_dtype)
        off = np.ascontiguousarray(qlabel_offsets, dtype=np.int64)
        lab = np.ascontiguousarray(qlabel_ids, dtype=np.int32)
        nq = q.shape[0]
        ids = np.empty((nq, self.k), dtype=np.int64)
        d = np.empty((nq, self.k), dtype=np.float32)
        lat = np.empty(nq, dtype=np.float32)
        _check(load_library().vf_serve_run(self._h, _np_ptr(q), nq, _np_ptr(off), _np_ptr(lab), int(in_flight),
                                           _np_ptr(ids), _np_ptr(d), _np_ptr(lat)))
        return ids, d, lat

    def end(self):
        """Stops the kernel and releases the session; returns (jobs completed, exit reason)."""
        if self._h is None:
            return None
        n, why = C.c_int64(0), C.c_int32(0)
        h, self._h = self._h, None
        _check(load_library().vf_serve_end(h, C.byref(n), C.byref(why)))
        return n.value, why.value

    def __del__(self):
        try:
            self.end()
        except Exception:
            pass


NOALLOC_SCRATCH_BYTES, NOALLOC_MAX_QUERIES = 8 << 20, 1024
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
    index._enter(stream)
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
    index._enter(stream)
    _check(load_library().vf_search_exact(index._h, C.c_void_p(queries.data_ptr()), nq, _np_ptr(off), _np_ptr(ids),
                                          int(k), C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_dists.data_ptr()),
                                          _stream_handle(stream)))
    return out_ids, out_dists
