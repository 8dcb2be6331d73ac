"""GPU tests of the boundary itself: the caller-supplied device allocator, the index sizes vf_index_stats reports
against the memory model of Section 4.2.4, and calls that overlap on several streams with different seed counts."""
import numpy as np
import pytest

from paper_2506_00812_amd.workloads import make_workload
from tests.gpu_util import to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vf():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2506_00812_amd import binding
    binding.load_library()
    return binding


def test_index_sizes_follow_the_memory_model(vf, tiny, tiny_oracle):
    """Section 4.2.4: N F_HS R b for the neighbour lists, N D F_LS b for the scan partition's vectors, N F b for
    the index mappings, evaluated on the realised F's of the tiny workload (from the oracle's posting lists), plus
    the extras this library documents: the graph rows a second time as global ids, padding of the interleaved
    lists to whole groups and an even chunk count, a norm per slot, bitsets of the graph labels.  The same sizes
    must be what the exported arrays hold and what the allocator was asked for."""
    import torch
    s = tiny.spec
    X = torch.from_numpy(tiny.vectors).cuda()
    ix = vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree)
    st = ix.stats()
    S = tiny_oracle.S
    N, D, R, b = s.n, s.dim, s.graph_degree, 1
    hs, ls = S[S >= s.T], S[(S > 0) & (S < s.T)]
    F_HS, F_LS = hs.sum() / N, ls.sum() / N
    F = F_HS + F_LS
    assert st["n_HS"] == round(N * F_HS) and st["n_LS"] == round(N * F_LS)
    # the model's three terms (ids and map entries are 4-byte integers whatever the data type)
    assert st["bytes_graph"] == 2 * round(N * F_HS * R * 4)
    assert st["bytes_maps"] == round(N * F * 4)
    groups = int(((ls + 31) // 32).sum())
    chunks = 2 * ((D * b // 16 + 1) // 2)
    assert st["n_groups_LS"] == groups and st["chunks_per_vector"] == chunks
    model_x_ls = round(N * D * F_LS * b)
    padding = (groups * 32 - int(ls.sum())) * D * b + groups * 32 * (chunks * 16 - D * b)
    assert st["bytes_x_ls"] == model_x_ls + padding + groups * 32 * 4
    assert st["bytes_bitsets"] == len(hs) * ((N + 31) // 32) * 4
    assert st["bytes_meta"] == s.n_labels * 24
    assert st["bytes_total"] == sum(st[k] for k in ("bytes_graph", "bytes_maps", "bytes_x_ls", "bytes_bitsets", "bytes_meta", "bytes_x_ls_bf16"))
    assert st["bytes_x_ls_bf16"] == 0   # uint8 data have no bfloat16 copy
    # what the index really holds
    assert 2 * ix.export("G_HS").nbytes == st["bytes_graph"]
    assert ix.export("M_HS").nbytes + ix.export("M_LS").nbytes == st["bytes_maps"]
    assert ix.export("X_LS").nbytes + groups * 32 * 4 == st["bytes_x_ls"]
    assert ix.export("BITSET").nbytes == st["bytes_bitsets"]
    # and what it asked the allocator for: the arrays above, the per-row norms of X (4 N) for seed scoring, and
    # rounding of every block to 256 bytes
    live = ix.allocator.live_bytes()
    assert st["bytes_total"] <= live <= st["bytes_total"] + 4 * N + 256 * len(ix.allocator.live) + 4096, (live, st)


def test_device_memory_comes_from_the_callers_allocator(vf, tiny):
    """Every device allocation of an index -- arrays, workspaces, seed copies -- goes through the vf_allocator the
    binding passes (PyTorch's caching allocator), and all of it is handed back by vf_index_free."""
    import torch
    s = tiny.spec
    X = torch.from_numpy(tiny.vectors).cuda()
    Q = torch.from_numpy(tiny.queries).cuda()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ix = vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree)
    al = ix.allocator
    built = al.live_bytes()
    assert al.n_alloc > 8 and built > 0
    assert torch.cuda.memory_allocated() - before >= built           # torch accounts for it
    ids, d = vf.search(ix, Q, tiny.qlabel_offsets, tiny.qlabel_ids, 10, itopk=32, width=1, iters=8, n_seeds=256)
    torch.cuda.synchronize()
    assert al.live_bytes() > built                                    # workspace and seed copy
    ref = (to_np(ids), to_np(d))
    del ids, d
    ix.free()
    assert not al.live and al.n_free == al.n_alloc
    assert torch.cuda.memory_allocated() == before
    # the same index on hipMalloc gives the same answers
    ix2 = vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree, torch_allocator=False)
    assert ix2.allocator is None
    ids, d = vf.search(ix2, Q, tiny.qlabel_offsets, tiny.qlabel_ids, 10, itopk=32, width=1, iters=8, n_seeds=256)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(ids), ref[0]) and np.array_equal(to_np(d), ref[1])


def test_allocator_failure_is_reported_not_thrown(vf, tiny):
    """An allocator that runs dry makes the call fail with VF_ENOMEM and a message; nothing leaks."""
    import ctypes as C
    import torch
    s = tiny.spec
    X = torch.from_numpy(tiny.vectors).cuda()
    al = vf.TorchAllocator(X.device)
    budget = {"left": 6}
    inner = al._alloc_cb

    def stingy(nbytes, ctx):
        if budget["left"] == 0:
            return None
        budget["left"] -= 1
        return inner(nbytes, ctx)
    cb = vf.ALLOC_FN(stingy)
    al.struct = vf.VfAllocator(cb, al._free_cb, None)
    L = vf.load_library()
    h = C.c_void_p()
    off = np.ascontiguousarray(tiny.label_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(tiny.label_ids, dtype=np.int32)
    rc = L.vf_build_index(C.c_void_p(X.data_ptr()), 0, s.n, s.dim, off.ctypes.data_as(C.c_void_p),
                          ids.ctypes.data_as(C.c_void_p), s.n_labels, s.T, s.graph_degree, C.byref(al.struct),
                          C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(h))
    assert rc == -2 and not h.value
    assert b"allocator returned NULL" in L.vf_last_error()
    assert not al.live and al.n_alloc == al.n_free == 6


def test_streams_with_different_seed_counts_overlap_safely(vf):
    """Calls on different streams may use different n_seeds at the same time: each seed count has its own
    interleaved copy of the seeds, so a call never overwrites what another stream's seed kernel is reading.
    Interleaved calls with five seed counts (one more than the index keeps copies of) on four streams, float32
    and uint8, every result equal to the same call made alone."""
    import torch
    for w in (make_workload("c2", n=30_000, nq=1500, n_labels=60, n_clusters=64, T=800, graph_degree=32),
              make_workload("tiny")):
        s = w.spec
        X = torch.from_numpy(w.vectors).cuda()
        Q = torch.from_numpy(w.queries).cuda()
        ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree)
        seeds = (700, 300, 1100, 96, 520)
        calls = []
        for i in range(20):
            lo = (i * 61) % (s.nq - 600)
            hi = lo + (600 if i % 2 == 0 else 40)            # large calls take the bfloat16 copy, small ones float32
            qo = (w.qlabel_offsets[lo:hi + 1] - w.qlabel_offsets[lo]).astype(np.int64)
            qi = np.ascontiguousarray(w.qlabel_ids[w.qlabel_offsets[lo]:w.qlabel_offsets[hi]])
            calls.append((lo, hi, qo, qi, dict(itopk=32, width=1, iters=6, n_seeds=seeds[i % len(seeds)])))
        alone = []
        for lo, hi, qo, qi, prm in calls:
            ids, d = vf.search(ix, Q[lo:hi], qo, qi, 10, **prm)
            torch.cuda.synchronize()
            alone.append((to_np(ids), to_np(d)))
        streams = [torch.cuda.Stream() for _ in range(4)]
        for rnd in range(3):
            outs = []
            for i, (lo, hi, qo, qi, prm) in enumerate(calls):
                with torch.cuda.stream(streams[(i + rnd) % len(streams)]):
                    outs.append(vf.search(ix, Q[lo:hi], qo, qi, 10, **prm))
            torch.cuda.synchronize()
            for i, (ids, d) in enumerate(outs):
                assert np.array_equal(to_np(ids), alone[i][0]), (s.name, rnd, i)
                assert np.array_equal(to_np(d).view(np.uint32), alone[i][1].view(np.uint32)), (s.name, rnd, i)
