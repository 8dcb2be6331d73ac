"""Pins for the CPU oracle: each test checks the oracle against something other
than itself -- the definitions in the paper, its worked examples, exact filtered
brute force written separately in numpy, special cases and invariants."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import OracleIndex
from paper_2506_00812_amd.workloads import make_workload
from tests.bruteforce import filtered_knn, membership, recall_at_k

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


# ------------------------------------------------------------------ index (Alg. 1, Section 4.1.2 / 4.2.1)

def test_posting_lists_match_definition(tiny, tiny_oracle):
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    S = tiny_oracle.S
    assert np.array_equal(S, mem.sum(axis=0))
    O_HS, O_LS, M_HS, M_LS = tiny_oracle.O_HS, tiny_oracle.O_LS, tiny_oracle.M_HS, tiny_oracle.M_LS
    run_hs = run_ls = 0
    for l in range(s.n_labels):
        C_l = np.flatnonzero(mem[:, l])          # C_l = { i : l in L_{X_i} }, ascending
        if S[l] >= s.T:                          # |C_l| == T is a graph list
            assert O_HS[l] == run_hs and O_LS[l] == -1
            assert np.array_equal(M_HS[run_hs:run_hs + S[l]], C_l)
            run_hs += S[l]
        elif S[l] > 0:
            assert O_LS[l] == run_ls and O_HS[l] == -1
            assert np.array_equal(M_LS[run_ls:run_ls + S[l]], C_l)
            run_ls += S[l]
        else:
            assert O_HS[l] == -1 and O_LS[l] == -1
    assert run_hs == tiny_oracle.n_HS and run_ls == tiny_oracle.n_LS
    # the tiny workload happens to hold a list of exactly T ids: the boundary case is live
    assert (S == s.T).any()


def test_graph_rows_are_exact_knn_uint8(tiny, tiny_oracle):
    s = tiny.spec
    S, O, M, G = tiny_oracle.S, tiny_oracle.O_HS, tiny_oracle.M_HS, tiny_oracle.G_HS
    rng = np.random.default_rng(1)
    X = tiny.vectors.astype(np.int64)
    for l in np.flatnonzero(S >= s.T):
        loc = M[O[l]:O[l] + S[l]]
        for j in rng.integers(0, S[l], size=12):
            d = ((X[loc] - X[loc[j]][None, :]) ** 2).sum(axis=1)
            d[j] = np.iinfo(np.int64).max          # no self edge
            want = np.lexsort((np.arange(S[l]), d))[:s.graph_degree]
            assert np.array_equal(G[O[l] + j], want), (l, j)
    assert G.min() >= 0
    # every entry is a local id of its own list
    for l in np.flatnonzero(S >= s.T):
        assert G[O[l]:O[l] + S[l]].max() < S[l]


def test_lazy_graph_rows_equal_eager(tiny, tiny_oracle):
    s = tiny.spec
    lazy = OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree,
                       lazy_graph=True)
    S, O, G = tiny_oracle.S, tiny_oracle.O_HS, tiny_oracle.G_HS
    for l in np.flatnonzero(S >= s.T)[:3]:
        for j in (0, 7, int(S[l]) - 1):
            assert np.array_equal(lazy.graph_row(l, j), G[O[l] + j])
    a = lazy.search(tiny.queries[:200], tiny.qlabel_offsets[:201], tiny.qlabel_ids[:200], 10, 32, 1, 20)
    b = tiny_oracle.search(tiny.queries[:200], tiny.qlabel_offsets[:201], tiny.qlabel_ids[:200], 10, 32, 1, 20)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_build_rejects_bad_arguments(tiny):
    s = tiny.spec
    with pytest.raises(ValueError):   # T must leave room for R neighbours besides the vertex itself
        OracleIndex(tiny.vectors[:100], tiny.label_offsets[:101], tiny.label_ids[:tiny.label_offsets[100]],
                    s.n_labels, 16, 16)
    with pytest.raises(ValueError):   # label id outside the vocabulary
        OracleIndex(tiny.vectors[:100], tiny.label_offsets[:101], tiny.label_ids[:tiny.label_offsets[100]],
                    3, 500, 16)


# ------------------------------------------------------------------ routing (Section 4.1.2 eq., Section 4.3.2)

def test_routing_threshold_and_boundary(tiny, tiny_oracle):
    s = tiny.spec
    S = tiny_oracle.S
    _, _, info = tiny_oracle.search(tiny.queries, tiny.qlabel_offsets, tiny.qlabel_ids, s.k, s.itopk, s.width,
                                    s.iters, with_info=True)
    ql = tiny.qlabel_ids
    want = np.where(S[ql] == 0, 0, np.where(S[ql] < s.T, 1, 2))
    assert np.array_equal(info["method"], want)
    assert np.array_equal(info["route_label"], np.where(S[ql] == 0, -1, ql))
    lab_T = int(np.flatnonzero(S == s.T)[0])
    _, _, info = tiny_oracle.search(tiny.queries[:1], np.array([0, 1]), np.array([lab_T]), s.k, s.itopk, 1, 5,
                                    with_info=True)
    assert info["method"][0] == 2


def test_and_searches_smallest_list_paper_example():
    g = _gold("paper_examples.json")["and_list_choice"]
    nA, nB, nC = g["label_sizes"]["A"], g["label_sizes"]["B"], g["label_sizes"]["C"]
    n = nA
    X = (np.arange(n) % 251).astype(np.uint8).reshape(n, 1)
    # label ids: A=0, B=1, C=2; B is carried by the first nB points, C by the first nC
    cnt = 1 + (np.arange(n) < nB) + (np.arange(n) < nC)
    off = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(cnt, out=off[1:])
    ids = np.empty(off[-1], dtype=np.int32)
    for i in range(n):
        labs = [0] + ([1] if i < nB else []) + ([2] if i < nC else [])
        ids[off[i]:off[i + 1]] = labs
    ix = OracleIndex(X, off, ids, 3, 100_000, 2, lazy_graph=True)   # T above every list: scan path
    assert list(ix.S) == [nA, nB, nC]
    _, _, info = ix.search(X[:1], np.array([0, 3]), np.array([0, 1, 2]), 5, with_info=True)
    assert info["route_label"][0] == {"A": 0, "B": 1, "C": 2}[g["searched"]]
    assert info["counters"][0, 2] == nB          # exactly the smallest list was predicate-tested
    # ties in list size go to the lower label id
    ix2 = OracleIndex(X[:10], np.arange(0, 21, 2), np.tile(np.array([1, 0], dtype=np.int32), 10), 2, 1000, 2,
                      lazy_graph=True)
    _, _, info = ix2.search(X[:1], np.array([0, 2]), np.array([1, 0]), 5, with_info=True)
    assert info["route_label"][0] == 0


# ------------------------------------------------------------------ predicate (Section 4.3.2)

def test_predicate_paper_example():
    g = _gold("paper_examples.json")["predicate"]
    ok, pos = oracle.predicate(g["point_labels"], g["query_labels"])
    assert ok == g["found"]
    assert pos[0] == g["position_of_smallest"] and pos[2] == g["position_of_largest"]
    lo, hi = g["middle_search_range"]
    assert lo <= pos[1] <= hi and pos[1] == g["position_of_middle"]
    assert lo == pos[0] + 1 and hi == pos[2] - 1


def test_predicate_equals_subset_test():
    rng = np.random.default_rng(3)
    for _ in range(3000):
        pl = np.unique(rng.integers(0, 24, size=rng.integers(0, 12)))
        ql = np.unique(rng.integers(0, 24, size=rng.integers(1, 5)))
        ok, pos = oracle.predicate(pl, ql)
        assert ok == set(ql.tolist()).issubset(set(pl.tolist()))
        if ok:
            assert np.array_equal(pl[pos], ql)


# ------------------------------------------------------------------ interleaved layout (Section 4.2.2)

def test_interleaved_layout_paper_example():
    n, dim = 70, 12
    v = (np.arange(n)[:, None] * 100 + np.arange(dim)[None, :]).astype(np.float32)
    out = oracle.store_interleaved(v)
    veclen = 4                                    # 16 / sizeof(float32)
    g = _gold("paper_examples.json")["interleaved_float32"]["order_prefix"]
    # (v0[0:3], v1[0:3], ..., v31[0:3], v0[4:7], v1[4:7], ...)
    where = {"v0": 0, "v1": 1, "v31": 31}
    for name, lo, hi in g:
        vec, chunk = where[name], lo // veclen
        pos = (chunk * 32 + vec) * veclen
        assert np.array_equal(out[pos:pos + veclen], v[vec, lo:hi + 1])
    # round trip of the whole table, ragged last group zero-filled
    n_chunks = dim // veclen
    blk = out.reshape(-1, n_chunks, 32, veclen)   # [group][chunk][vector][element]
    back = blk.transpose(0, 2, 1, 3).reshape(-1, dim)
    assert np.array_equal(back[:n], v)
    assert not back[n:].any()
    u = np.arange(40 * 32, dtype=np.uint8).reshape(40, 32)
    bu = oracle.store_interleaved(u).reshape(-1, 2, 32, 16).transpose(0, 2, 1, 3).reshape(-1, 32)
    assert np.array_equal(bu[:40], u)


# ------------------------------------------------------------------ distances

def test_distance_closed_forms():
    rng = np.random.default_rng(5)
    for dim in (1, 4, 31, 32, 96, 128, 200):
        q = rng.integers(-8, 9, size=dim).astype(np.float32)
        x = rng.integers(-8, 9, size=dim).astype(np.float32)
        # small integers: every partial sum is exact, so any summation order gives the integer result
        assert oracle.dist_f32_ordered(q, x) == float(((q.astype(np.int64) - x.astype(np.int64)) ** 2).sum())
        qu = rng.integers(0, 256, size=dim).astype(np.uint8)
        xu = rng.integers(0, 256, size=dim).astype(np.uint8)
        assert oracle.dist_u8(qu, xu) == int(((qu.astype(np.int64) - xu.astype(np.int64)) ** 2).sum())
        qf = rng.standard_normal(dim).astype(np.float32)
        xf = rng.standard_normal(dim).astype(np.float32)
        exact = ((qf.astype(np.float64) - xf.astype(np.float64)) ** 2).sum()
        # fp32 accumulation over <= dim terms: relative error well inside (dim+2) * 2^-24
        assert abs(oracle.dist_f32_ordered(qf, xf) - exact) <= (dim + 2) * 2.0 ** -24 * exact
    assert oracle.dist_f32_ordered(np.ones(7), np.ones(7)) == 0.0
    # swapping the operands cannot change a squared difference
    assert oracle.dist_f32_ordered(qf, xf) == oracle.dist_f32_ordered(xf, qf)


# ------------------------------------------------------------------ scan path = exact filtered kNN (Def. 1)

def test_scan_equals_brute_force_uint8(tiny, tiny_oracle):
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    ids, dists, info = tiny_oracle.search(tiny.queries, tiny.qlabel_offsets, tiny.qlabel_ids, s.k, s.itopk,
                                          s.width, s.iters, with_info=True)
    scan_q = np.flatnonzero(info["method"] == 1)
    assert len(scan_q) > 100
    for j in scan_q[:300]:
        wi, wd = filtered_knn(tiny.vectors, mem, tiny.queries[j], [tiny.qlabel_ids[j]], s.k)
        assert np.array_equal(ids[j], wi)
        assert np.array_equal(dists[j].astype(np.float64), wd)    # integer distances: exact


def test_force_scan_is_exact_filtered_knn_with_and(tiny, tiny_oracle):
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    rng = np.random.default_rng(7)
    nq = 150
    # AND pairs, some with empty intersections, some repeated labels
    a = rng.integers(0, 12, size=nq).astype(np.int32)
    b = rng.integers(0, 40, size=nq).astype(np.int32)
    qoff = np.arange(0, 2 * nq + 1, 2)
    qids = np.stack([a, b], axis=1).reshape(-1)
    ids, dists = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, force_scan=True)
    n_short = 0
    for j in range(nq):
        wi, wd = filtered_knn(tiny.vectors, mem, tiny.queries[j], [a[j], b[j]], s.k)
        assert np.array_equal(ids[j], wi)
        assert np.array_equal(dists[j].astype(np.float64), wd)
        n_short += int((wi < 0).any())
    assert n_short > 0           # padding with (-1, +inf) was exercised


def test_scan_float_matches_brute_force():
    w = make_workload("c2", n=6000, nq=120, n_labels=60, n_clusters=16, T=400)
    s = w.spec
    ix = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, 8, lazy_graph=True)
    mem = membership(w.label_offsets, w.label_ids, s.n_labels)
    ids, dists = ix.search(w.queries, w.qlabel_offsets, w.qlabel_ids, 10, force_scan=True)
    for j in range(s.nq):
        wi, wd = filtered_knn(w.vectors, mem, w.queries[j], [w.qlabel_ids[j]], 10)
        assert np.array_equal(ids[j], wi)
        ok = wi >= 0
        assert np.allclose(dists[j][ok], wd[ok], rtol=1e-6)


# ------------------------------------------------------------------ beam search (Alg. 2 loop) -- pins of this repo's reading

def _hand_index():
    g = _gold("beam_hand_worked.json")
    X = np.array(g["values"], dtype=np.uint8).reshape(-1, 1)
    n = len(X)
    ix = OracleIndex(X, np.arange(n + 1), np.zeros(n, dtype=np.int32), 1, g["T"], g["R"])
    return g, X, ix


def test_beam_hand_worked_example():
    g, X, ix = _hand_index()
    assert np.array_equal(ix.G_HS, np.array(g["graph_rows"]))
    for c in g["cases"]:
        q = np.array([[c["query"]]], dtype=np.uint8)
        ids, dists, info = ix.search(q, np.array([0, 1]), np.array([0]), c["k"], c["itopk"], c["width"], c["iters"],
                                     c["n_seeds"], with_info=True)
        assert ids[0].tolist() == c["ids"], c["why"]
        assert dists[0].tolist() == c["dists"]
        assert info["counters"][0, 0] == c["n_scored"] and info["counters"][0, 1] == c["n_expanded"]


def _small_graph_workload(dtype):
    base = "tiny" if dtype == "uint8" else "c2"
    return make_workload(base, n=1500, nq=80, n_labels=12, n_clusters=6, T=17, graph_degree=16)


@pytest.mark.parametrize("dtype", ["uint8", "float32"])
def test_beam_with_every_vertex_seeded_is_exact(dtype):
    """itopk >= n and n_seeds >= n: every list member is scored, so the result
    must be the exact filtered top-k, single label and AND alike."""
    w = _small_graph_workload(dtype)
    s = w.spec
    ix = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree)
    mem = membership(w.label_offsets, w.label_ids, s.n_labels)
    big = int(ix.S.max())
    rng = np.random.default_rng(11)
    other = rng.integers(0, s.n_labels, size=s.nq).astype(np.int32)
    for qoff, qids in ((w.qlabel_offsets, w.qlabel_ids),
                       (np.arange(0, 2 * s.nq + 1, 2), np.stack([w.qlabel_ids, other], 1).reshape(-1))):
        ids, dists, info = ix.search(w.queries, qoff, qids, 10, itopk=big, width=1, iters=0, n_seeds=big,
                                     with_info=True)
        assert (info["method"][ix.S[info["route_label"]] >= s.T] == 2).all()
        for j in range(s.nq):
            labs = qids[qoff[j]:qoff[j + 1]]
            wi, wd = filtered_knn(w.vectors, mem, w.queries[j], labs, 10)
            assert np.array_equal(ids[j], wi), j
            ok = wi >= 0
            assert np.allclose(dists[j][ok], wd[ok], rtol=1e-5)


def test_beam_iters_zero_returns_best_seeds(tiny, tiny_oracle):
    s = tiny.spec
    S, O, M = tiny_oracle.S, tiny_oracle.O_HS, tiny_oracle.M_HS
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    ids, dists, info = tiny_oracle.search(tiny.queries[:200], tiny.qlabel_offsets[:201], tiny.qlabel_ids[:200],
                                          s.k, itopk=32, width=1, iters=0, n_seeds=48, with_info=True)
    for j in np.flatnonzero(info["method"] == 2):
        l = tiny.qlabel_ids[j]
        n = int(S[l])
        seeds_local = (np.arange(48) * n) // 48
        seeds_global = M[O[l] + seeds_local]
        wi, wd = filtered_knn(tiny.vectors, mem, tiny.queries[j], [l], s.k, restrict=seeds_global)
        assert np.array_equal(ids[j], wi)
        assert np.array_equal(dists[j].astype(np.float64), wd)
        assert info["counters"][j, 0] == 48 and info["counters"][j, 1] == 0


def test_beam_invariants_and_recall(tiny, tiny_oracle):
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    rng = np.random.default_rng(13)
    nq = 400
    # half single-label, half 2-label AND between frequent labels so the graph path is used
    a = tiny.qlabel_ids[:nq].copy()
    b = rng.integers(0, 8, size=nq).astype(np.int32)
    two = rng.random(nq) < 0.5
    cnt = np.where(two, 2, 1)
    qoff = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(cnt, out=qoff[1:])
    qids = np.empty(qoff[-1], dtype=np.int32)
    qids[qoff[:-1]] = a
    qids[qoff[:-1][two] + 1] = b[two]
    ids, dists, info = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, itopk=64, width=2, iters=40,
                                          n_seeds=256, with_info=True)
    gt = np.empty_like(ids)
    X = tiny.vectors.astype(np.int64)
    for j in range(nq):
        labs = np.unique(qids[qoff[j]:qoff[j + 1]])
        got = ids[j][ids[j] >= 0]
        assert len(np.unique(got)) == len(got)                       # no duplicates
        assert mem[got][:, labs].all()                               # every id carries all query labels
        assert (np.diff(dists[j][:len(got)]) >= 0).all()             # non-decreasing
        assert np.isinf(dists[j][len(got):]).all() and (ids[j][len(got):] == -1).all()
        d = ((X[got] - tiny.queries[j].astype(np.int64)[None, :]) ** 2).sum(axis=1)
        assert np.array_equal(d.astype(np.float64), dists[j][:len(got)].astype(np.float64))
        for i in range(1, len(got)):                                 # ties in ascending id
            if dists[j][i] == dists[j][i - 1]:
                assert got[i] > got[i - 1]
        gt[j], _ = filtered_knn(tiny.vectors, mem, tiny.queries[j], labs, s.k)
    graph_q = info["method"] == 2
    assert graph_q.sum() > 100
    single = graph_q & ~two
    # with 256 seeds over 32 clusters the graph lists are navigable: recall must be high
    assert recall_at_k(ids[single], gt[single]) > 0.9
    assert recall_at_k(ids[info["method"] == 1], gt[info["method"] == 1]) == 1.0


def test_beam_result_independent_of_visited_capacity(tiny, tiny_oracle):
    s = tiny.spec
    nq = 300
    args = (tiny.queries[:nq], tiny.qlabel_offsets[:nq + 1], tiny.qlabel_ids[:nq], s.k)
    ref = tiny_oracle.search(*args, itopk=32, width=2, iters=30, n_seeds=64, with_info=True)
    for cap in (1, 7, 64, 1021):
        got = tiny_oracle.search(*args, itopk=32, width=2, iters=30, n_seeds=64, visited_cap=cap, with_info=True)
        assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])
    # forgetting costs extra distance evaluations, never fewer
    tiny_cap = tiny_oracle.search(*args, itopk=32, width=2, iters=30, n_seeds=64, visited_cap=1, with_info=True)
    assert (tiny_cap[2]["counters"][:, 0] >= ref[2]["counters"][:, 0]).all()


def test_search_rejects_bad_arguments(tiny, tiny_oracle):
    q = tiny.queries[:2]
    with pytest.raises(ValueError):    # k > itopk
        tiny_oracle.search(q, np.array([0, 1, 2]), np.array([0, 1]), 40, itopk=32)
    with pytest.raises(ValueError):    # a query with no label
        tiny_oracle.search(q, np.array([0, 0, 1]), np.array([0]), 10)
    with pytest.raises(ValueError):    # label outside the vocabulary
        tiny_oracle.search(q, np.array([0, 1, 2]), np.array([0, 100]), 10)


def test_unknown_or_empty_label_gives_empty_rows():
    w = make_workload("tiny", n=300, nq=4, n_labels=50, T=40, graph_degree=8)
    ix = OracleIndex(w.vectors, w.label_offsets, w.label_ids, 60, 40, 8)     # labels 50..59 never occur
    ids, dists = ix.search(w.queries, np.array([0, 1, 2, 4, 6]), np.array([55, 0, 0, 55, 55, 0]), 5, 32, 1, 5)
    assert (ids[0] == -1).all() and np.isinf(dists[0]).all()
    assert (ids[1] >= 0).any()
    assert (ids[2] == -1).all() and (ids[3] == -1).all()


# ------------------------------------------------------------------ recall (Eq. 1) and memory model (Section 4.2.4)

def test_recall_formula():
    a = np.array([[1, 2, 3, 4], [5, 6, 7, 8]])
    gt = np.array([[1, 2, 9, 10], [5, 6, 7, 8]])
    assert recall_at_k(a, gt) == (2 + 4) / 8


def test_memory_model_worked_numbers():
    g = _gold("paper_examples.json")["memory_model"]
    N, D, R, Rp, b = g["N"], g["D"], g["R"], g["R_prime"], g["b"]
    GiB = 2.0 ** 30
    hs = N * (D + g["F_HS"] * Rp) * b / GiB
    ls = N * D * g["F_LS"] * b / GiB
    assert round(hs, 2) == g["hs_GiB"] and round(ls, 2) == g["ls_GiB"]
    assert abs(hs + ls - g["total_GiB"]) < 0.011
    assert round(N * (D + R) * b / GiB, 2) == g["single_index_GiB"]
    assert round(N * g["F"] * b / GiB, 2) == g["mapping_GiB"]


# ------------------------------------------------------------------ OR and the parallel AND policy (Section 4.3.1, 4.3.2)

def _multi_label_queries(nq, n_labels, seed, lo=1, hi=4):
    rng = np.random.default_rng(seed)
    counts = rng.integers(lo, hi + 1, size=nq)
    qoff = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(counts, out=qoff[1:])
    # a mix of popular labels (graph lists) and rare ones (scan lists), duplicates allowed
    qids = np.where(rng.random(qoff[-1]) < 0.6, rng.integers(0, 8, size=qoff[-1]), rng.integers(0, n_labels, size=qoff[-1]))
    return qoff, qids.astype(np.int32)


def test_or_with_exact_searches_is_brute_force_over_the_union(tiny, tiny_oracle):
    """OR = nearest neighbours carrying ANY query label (Section 4.3.1).  With every
    per-label search exact, the merge must give exact kNN over the union of the lists,
    written here from the definition in numpy."""
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    nq = 150
    qoff, qids = _multi_label_queries(nq, s.n_labels, 5)
    ids, dists = tiny_oracle.search_multi(tiny.queries[:nq], qoff, qids, oracle.OR, s.k, force_scan=True)
    for j in range(nq):
        ls = np.unique(qids[qoff[j]:qoff[j + 1]])
        cand = np.flatnonzero(mem[:, ls].any(axis=1))
        d = ((tiny.vectors[cand].astype(np.float64) - tiny.queries[j].astype(np.float64)) ** 2).sum(axis=1)
        order = np.lexsort((cand, d))[:s.k]
        want = np.full(s.k, -1, dtype=np.int64)
        want[:len(order)] = cand[order]
        assert np.array_equal(ids[j], want), j
        assert np.array_equal(dists[j][:len(order)], d[order].astype(np.float32))
        assert len(np.unique(ids[j][ids[j] >= 0])) == (ids[j] >= 0).sum()       # an id shared by two lists appears once


def test_parallel_and_with_exact_searches_is_brute_force_over_the_intersection(tiny, tiny_oracle):
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    nq = 150
    qoff, qids = _multi_label_queries(nq, s.n_labels, 6, lo=2, hi=3)
    ids, dists = tiny_oracle.search_multi(tiny.queries[:nq], qoff, qids, oracle.AND_PARALLEL, s.k, force_scan=True)
    n_nonempty = 0
    for j in range(nq):
        want, wd = filtered_knn(tiny.vectors, mem, tiny.queries[j], np.unique(qids[qoff[j]:qoff[j + 1]]), s.k)
        assert np.array_equal(ids[j], want), j
        n_nonempty += int(want[0] >= 0)
    assert n_nonempty > 20


def test_multi_search_with_one_label_is_the_single_label_search(tiny, tiny_oracle):
    s = tiny.spec
    params = dict(itopk=32, width=1, iters=12, n_seeds=96)
    i0, d0 = tiny_oracle.search(tiny.queries, tiny.qlabel_offsets, tiny.qlabel_ids, s.k, **params)
    for mode in (oracle.OR, oracle.AND_PARALLEL):
        i1, d1, info = tiny_oracle.search_multi(tiny.queries, tiny.qlabel_offsets, tiny.qlabel_ids, mode, s.k,
                                                with_info=True, **params)
        assert np.array_equal(i0, i1) and np.array_equal(d0, d1)
        assert (info["n_searches"] == 1).all()


def test_parallel_and_contains_the_greedy_search_and_stays_valid(tiny, tiny_oracle):
    """The greedy policy's search (smallest list, others as predicate) is one of the
    parallel policy's searches, so the merged top-k can only be at least as close, rank by
    rank; every id still carries every label; graph-only queries run one search per label and
    scan-routed queries exactly one."""
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    rng = np.random.default_rng(9)
    nq = 300
    a = rng.integers(0, 7, size=nq)                    # the 7 largest labels are the graph lists of this workload
    b = rng.integers(0, 12, size=nq)
    qoff = np.arange(0, 2 * nq + 1, 2, dtype=np.int64)
    qids = np.stack([a, b], axis=1).reshape(-1).astype(np.int32)
    params = dict(itopk=32, width=1, iters=10, n_seeds=64)
    ig, dg, info = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, with_info=True, **params)
    ip, dp, pinfo = tiny_oracle.search_multi(tiny.queries[:nq], qoff, qids, oracle.AND_PARALLEL, s.k, with_info=True,
                                             **params)
    S, T = tiny_oracle.S, s.T
    better = 0
    for j in range(nq):
        ls = np.unique(qids[qoff[j]:qoff[j + 1]])
        for g in ip[j][ip[j] >= 0]:
            assert mem[g, ls].all()
        fin = dp[j][np.isfinite(dp[j])]
        assert (np.diff(fin) >= 0).all() and (ip[j][len(fin):] == -1).all()
        assert (dp[j] <= dg[j]).all()
        better += int((dp[j] < dg[j]).any())
        all_graph = (S[ls] >= T).all()
        assert pinfo["n_searches"][j] == (len(ls) if all_graph and (S[ls] > 0).all() else int((S[ls] > 0).all()))
    assert better > 5                                  # the policy exists because it finds closer points
    gt, _ = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, force_scan=True)
    assert recall_at_k(ip, gt) >= recall_at_k(ig, gt)


def test_or_is_at_least_as_close_as_every_single_label_search(tiny, tiny_oracle):
    s = tiny.spec
    nq = 200
    qoff, qids = _multi_label_queries(nq, s.n_labels, 11, lo=2, hi=3)
    params = dict(itopk=32, width=1, iters=10, n_seeds=64)
    io, do = tiny_oracle.search_multi(tiny.queries[:nq], qoff, qids, oracle.OR, s.k, **params)
    for t in range(2):                                  # first and second label of every query, searched alone
        one = np.array([qids[qoff[j] + min(t, qoff[j + 1] - qoff[j] - 1)] for j in range(nq)], dtype=np.int32)
        i1, d1 = tiny_oracle.search(tiny.queries[:nq], np.arange(nq + 1), one, s.k, **params)
        assert (do <= d1).all()
    assert all(len(np.unique(r[r >= 0])) == (r >= 0).sum() for r in io)


def test_multi_search_rejects_bad_arguments(tiny, tiny_oracle):
    with pytest.raises(ValueError):
        tiny_oracle.search_multi(tiny.queries[:4], np.arange(5), np.zeros(4, dtype=np.int32), 7, 10)
    with pytest.raises(ValueError):
        tiny_oracle.search_multi(tiny.queries[:4], np.arange(5), np.full(4, 10 ** 6, dtype=np.int32), oracle.OR, 10)


# ------------------------------------------------------------------ pruned graphs (rank-based pruning + reverse edges)

def _one_label_index(X, R, D, dtype):
    """All points carry label 0 (one graph list, local id == global id)."""
    n = len(X)
    off = np.arange(n + 1, dtype=np.int64)
    ids = np.zeros(n, dtype=np.int32)
    return OracleIndex(np.ascontiguousarray(X.astype(dtype)), off, ids, 1, D + 1, R, knn_degree=D)


def _rules_in_python(X, R, D):
    """The three steps written out a second time with Python sets and tuple sorts (uint8 data: exact distances)."""
    n = len(X)
    Xi = X.astype(np.int64)
    d = ((Xi[:, None, :] - Xi[None, :, :]) ** 2).sum(-1)
    np.fill_diagonal(d, np.iinfo(np.int64).max)
    knn = [sorted(range(n), key=lambda c: (d[x, c], c))[:D] for x in range(n)]
    F = []
    for x in range(n):
        keyed = []
        for j, y in enumerate(knn[x]):
            c = sum(1 for i in range(j) for r in range(j) if knn[knn[x][i]][r] == y)
            keyed.append((c, j, y))
        F.append([y for _, _, y in sorted(keyed)[:R]])
    proposals = {y: [] for y in range(n)}
    for x in range(n):
        for p, y in enumerate(F[x]):
            proposals[y].append((p, x))
    G = []
    for y in range(n):
        row = list(F[y][:R // 2])
        back = [x for _, x in sorted(proposals[y])[:R]]
        row += [x for x in back if x not in row][:R - R // 2]
        row += [v for v in F[y][R // 2:] if v not in row][:R - len(row)]
        G.append(row)
    return np.array(knn), np.array(F), np.array(G)


def test_pruned_graph_equals_the_rules_written_out_in_python():
    rng = np.random.default_rng(5)
    X = rng.integers(0, 256, size=(150, 16)).astype(np.uint8)
    for R, D in ((4, 8), (6, 9), (5, 5)):
        ix = _one_label_index(X, R, D, np.uint8)
        _, F, G = _rules_in_python(X, R, D)
        assert np.array_equal(ix.G_HS, G), (R, D)
        for j in (0, 17, 149):
            assert np.array_equal(ix.pruned_row(0, j, D), F[j])


def test_pruned_graph_of_points_on_a_line_is_the_chain():
    # positions 0, 1, 2, ...: the degree-4 row of an interior x is [x-1, x+1, x-2, x+2] (ties to the
    # lower id); x-2 is reached through x-1 and x+2 through x+1, so pruning to R = 2 leaves
    # [x-1, x+1]; x-1 proposes x at position 1 and x+1 proposes x at position 0, hence B[x] = [x+1, x-1]
    # and the merged row is [x-1, x+1]: worked by hand from the three steps.
    n = 40
    X = np.zeros((n, 16), dtype=np.float32)
    X[:, 0] = np.arange(n)
    ix = _one_label_index(X, 2, 4, np.float32)
    G = ix.G_HS
    for x in range(4, n - 4):
        assert G[x].tolist() == [x - 1, x + 1], x


def test_pruned_graph_invariants(tiny):
    s = tiny.spec
    R, D = s.graph_degree, 2 * s.graph_degree
    pruned = OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, R, knn_degree=D)
    wide = OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, D)   # exact degree-D rows
    G, KNN = pruned.G_HS, wide.G_HS
    S, O = pruned.S, pruned.O_HS
    for l in np.flatnonzero(O >= 0)[:6]:
        base, nl = int(O[l]), int(S[l])
        g, knn = G[base:base + nl], KNN[base:base + nl]
        assert g.min() >= 0 and g.max() < nl
        assert not (g == np.arange(nl)[:, None]).any()                      # no self loops
        assert all(len(set(r.tolist())) == R for r in g)                    # R distinct neighbours
        assert np.array_equal(g[:, 0], knn[:, 0])                           # the nearest neighbour has no detour
        fwd = [set(r.tolist()) for r in knn]
        for y in range(nl):
            assert set(g[y, :R // 2].tolist()) <= fwd[y]                    # kept forward edges come from the kNN row
            for x in g[y, R // 2:]:
                assert int(x) in fwd[y] or y in fwd[int(x)]                 # the rest: forward, or reverse of a kNN edge
        # the single-row routine agrees with the whole-graph build on the part that is always kept
        for j in (0, nl // 2, nl - 1):
            assert np.array_equal(pruned.pruned_row(l, j, D)[:R // 2], g[j, :R // 2])


def test_pruned_build_rejects_bad_arguments(tiny):
    s = tiny.spec
    with pytest.raises(ValueError):
        OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree,
                    knn_degree=s.graph_degree - 1)
    with pytest.raises(ValueError):
        OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, 20, 16, knn_degree=32)   # T < D + 1
    with pytest.raises(ValueError):
        OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree, lazy_graph=True,
                    knn_degree=2 * s.graph_degree)


def test_selectivity_aware_and_routing_is_exact_below_the_limit_and_unchanged_above(tiny, tiny_oracle):
    """and_scan_limit (optional routing, Section 4.3.2 / the greedy policy's ceiling in Section 5.3): an AND query whose
    smallest list is a graph list of at most that many points gets the exact filtered top-k of Def. 1 (written
    separately in numpy); every other query -- single label, AND on a scan list, AND on a longer graph list -- is
    answered exactly as without the limit."""
    s = tiny.spec
    mem = membership(tiny.label_offsets, tiny.label_ids, s.n_labels)
    S = tiny_oracle.S
    rng = np.random.default_rng(19)
    nq = 240
    a = rng.integers(0, 9, size=nq).astype(np.int32)            # the nine most frequent labels: graph lists and the first scan lists
    b = rng.integers(0, 9, size=nq).astype(np.int32)
    single = rng.random(nq) < 0.25
    cnt = np.where(single, 1, 2)
    qoff = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(cnt, out=qoff[1:])
    qids = np.empty(qoff[-1], dtype=np.int32)
    qids[qoff[:-1]] = a
    qids[qoff[:-1][~single] + 1] = b[~single]
    params = dict(itopk=32, width=1, iters=6, n_seeds=32)
    limit = 1000                                                 # graph lists hold 500 .. 3,427 points: some below, some above
    base_i, base_d, base_info = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, with_info=True, **params)
    ids, dists, info = tiny_oracle.search(tiny.queries[:nq], qoff, qids, s.k, with_info=True, and_scan_limit=limit, **params)
    n_exact = 0
    for j in range(nq):
        labs = np.unique(qids[qoff[j]:qoff[j + 1]])
        smallest = S[labs].min()
        if len(labs) > 1 and s.T <= smallest <= limit:
            assert info["method"][j] == 3 and base_info["method"][j] == 2
            wi, wd = filtered_knn(tiny.vectors, mem, tiny.queries[j], list(labs), s.k)
            assert np.array_equal(ids[j], wi) and np.array_equal(dists[j].astype(np.float64), wd)
            n_exact += 1
        else:
            assert info["method"][j] == base_info["method"][j]
            assert np.array_equal(ids[j], base_i[j]) and np.array_equal(dists[j], base_d[j])
    assert n_exact > 20 and (info["method"] == 2).sum() > 20
    # the greedy search misses some of what the exact route finds (the reason for the route)
    changed = sum(not np.array_equal(ids[j], base_i[j]) for j in range(nq))
    assert changed > 0
