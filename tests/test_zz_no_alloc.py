"""The entry point that allocates nothing (vf_search_noalloc) against vf_search on the same inputs: same bits,
on two calls in a row, the second with a smaller input, with and without a resident seed copy; sizes beyond the
fixed scratch array are rejected before anything is launched."""
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


def _and_mix(w, rng):
    """The workload's queries, every third one with a second label (an AND query)."""
    s = w.spec
    first = w.qlabel_ids[w.qlabel_offsets[:-1]]
    cnt = np.where(np.arange(s.nq) % 3 == 0, 2, 1)
    off = np.zeros(s.nq + 1, dtype=np.int64)
    np.cumsum(cnt, out=off[1:])
    ids = np.empty(off[-1], dtype=np.int32)
    ids[off[:-1]] = first
    two = np.flatnonzero(cnt == 2)
    ids[off[two] + 1] = rng.integers(0, min(8, s.n_labels), size=len(two))
    return off, ids


@pytest.mark.parametrize("name", ["uint8", "float32"])
def test_noalloc_equals_search_two_calls_in_a_row(vf, name):
    import torch
    if name == "uint8":
        w = make_workload("tiny", nq=900)
    else:
        w = make_workload("c2", n=30_000, nq=900, n_labels=60, n_clusters=64, T=800, graph_degree=32)
    s = w.spec
    X = torch.from_numpy(w.vectors).cuda()
    Q = torch.from_numpy(w.queries).cuda()
    ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree)
    rng = np.random.default_rng(17)
    off, ids = _and_mix(w, rng)
    params = dict(itopk=32, width=2, iters=8, n_seeds=400)
    k = 10

    def both(lo, hi, tag):
        qo = (off[lo:hi + 1] - off[lo]).astype(np.int64)
        qi = np.ascontiguousarray(ids[off[lo]:off[hi]])
        oi = torch.full((hi - lo, k), -7, dtype=torch.int64, device="cuda")
        od = torch.full((hi - lo, k), -7.0, dtype=torch.float32, device="cuda")
        vf.search_noalloc(ix, Q[lo:hi], qo, qi, k, oi, od, **params)
        torch.cuda.synchronize()
        return to_np(oi), to_np(od), qo, qi

    # 1) no seed copy is resident yet: the seed kernel gathers rows.  Two calls in a row, the second smaller.
    a_i, a_d, qo_a, qi_a = both(0, 900, "first")
    b_i, b_d, qo_b, qi_b = both(300, 420, "second, smaller")
    # reference: the allocating entry point (which also leaves a seed copy behind)
    r_i, r_d = vf.search(ix, Q[0:900], qo_a, qi_a, k, **params)
    s_i, s_d = vf.search(ix, Q[300:420], qo_b, qi_b, k, **params)
    torch.cuda.synchronize()
    for got_i, got_d, ref_i, ref_d, what in ((a_i, a_d, r_i, r_d, "900 queries"), (b_i, b_d, s_i, s_d, "120 queries")):
        assert np.array_equal(got_i, to_np(ref_i)), what
        assert np.array_equal(got_d.view(np.uint32), to_np(ref_d).view(np.uint32)), what
    assert (a_i >= 0).sum() > 5000 and (a_i[:, 0] == -1).sum() < 450
    # 2) with the seed copy resident (interleaved operand), again two calls in a row, the second smaller
    c_i, c_d, _, _ = both(0, 900, "third")
    d_i, d_d, _, _ = both(300, 420, "fourth, smaller")
    assert np.array_equal(c_i, a_i) and np.array_equal(c_d.view(np.uint32), a_d.view(np.uint32))
    assert np.array_equal(d_i, b_i) and np.array_equal(d_d.view(np.uint32), b_d.view(np.uint32))
    # 3) a single query, and the empty batch
    e_i, e_d, qo_e, qi_e = both(5, 6, "one query")
    t_i, t_d = vf.search(ix, Q[5:6], qo_e, qi_e, k, **params)
    torch.cuda.synchronize()
    assert np.array_equal(e_i, to_np(t_i)) and np.array_equal(e_d.view(np.uint32), to_np(t_d).view(np.uint32))


def test_noalloc_allocates_nothing_and_rejects_what_does_not_fit(vf, tiny):
    import torch
    s = tiny.spec
    X = torch.from_numpy(tiny.vectors).cuda()
    Q = torch.from_numpy(tiny.queries).cuda()
    T = 2000                                                          # lists of up to 1,999 vectors are scanned
    ix = vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, T, s.graph_degree)
    k = 10
    oi = torch.empty((s.nq, k), dtype=torch.int64, device="cuda")
    od = torch.empty((s.nq, k), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    live, n_alloc = ix.allocator.live_bytes(), ix.allocator.n_alloc
    free_before = torch.cuda.mem_get_info()[0]
    for _ in range(3):
        vf.search_noalloc(ix, Q, tiny.qlabel_offsets, tiny.qlabel_ids, k, oi, od, itopk=32, width=1, iters=8, n_seeds=256)
    torch.cuda.synchronize()
    assert ix.allocator.n_alloc == n_alloc and ix.allocator.live_bytes() == live     # nothing through the allocator
    assert torch.cuda.mem_get_info()[0] == free_before                                # and nothing beside it
    # more queries than the entry point takes
    nq_big = vf.NOALLOC_MAX_QUERIES + 1
    Qb = Q[:1].repeat(nq_big, 1).contiguous()
    with pytest.raises(vf.VecflowError, match="VF_NOALLOC_MAX_QUERIES"):
        vf.search_noalloc(ix, Qb, np.arange(nq_big + 1), np.zeros(nq_big, dtype=np.int32), k,
                          torch.empty((nq_big, k), dtype=torch.int64, device="cuda"),
                          torch.empty((nq_big, k), dtype=torch.float32, device="cuda"), itopk=32, width=1, iters=8, n_seeds=256)
    # a seed distance matrix larger than the scratch array is no error: the beam kernel gathers the seeds itself
    lab0 = np.zeros(s.nq, dtype=np.int32)                             # the largest list, a graph list
    vf.search_noalloc(ix, Q, np.arange(s.nq + 1), lab0, k, oi, od, itopk=32, width=1, iters=8, n_seeds=3000)
    ri, rd = vf.search(ix, Q, np.arange(s.nq + 1), lab0, k, itopk=32, width=1, iters=8, n_seeds=3000)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(oi), to_np(ri)) and np.array_equal(to_np(od).view(np.uint32), to_np(rd).view(np.uint32))
    # partial rows that do not fit are: one-group segments, 64 results per query, 1,000 queries on a 57-group list
    S = ix.export("S")
    scan_lab = int(np.argmax(np.where(S < T, S, -1)))
    assert S[scan_lab] > 1800
    ix.tune("seg_groups", 1)
    ix.tune("seg_groups_heavy", 1)
    labs = np.full(s.nq, scan_lab, dtype=np.int32)
    o64 = torch.empty((s.nq, 64), dtype=torch.int64, device="cuda")
    d64 = torch.empty((s.nq, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(vf.VecflowError, match="bytes of scratch"):
        vf.search_noalloc(ix, Q, np.arange(s.nq + 1), labs, 64, o64, d64, itopk=64, width=1, iters=8, n_seeds=256)
    # the same call with fewer queries fits, and equals vf_search
    vf.search_noalloc(ix, Q[:200], np.arange(201), labs[:200], 64, o64[:200], d64[:200], itopk=64, width=1, iters=8, n_seeds=256)
    ri, rd = vf.search(ix, Q[:200], np.arange(201), labs[:200], 64, itopk=64, width=1, iters=8, n_seeds=256)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(o64[:200]), to_np(ri)) and np.array_equal(to_np(d64[:200]).view(np.uint32), to_np(rd).view(np.uint32))
