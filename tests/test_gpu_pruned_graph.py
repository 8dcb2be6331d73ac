"""GPU parity for graphs built with VF_GRAPH_PRUNED (rank-based pruning + reverse edges): integer work on
ranks and ids, so rows and the searches over them must equal the oracle's bit for bit."""
import numpy as np
import pytest

from oracle import OracleIndex
from paper_2506_00812_amd.workloads import make_workload
from tests.gpu_util import assert_close_with_ties, assert_exact, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vf():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2506_00812_amd import binding
    binding.load_library()
    return binding


def _build_both(vf, w, D):
    import torch
    s = w.spec
    X = torch.from_numpy(w.vectors).cuda()
    ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree, graph_kind=vf.GRAPH_PRUNED,
                        knn_degree=D)
    ixo = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree,
                      knn_degree=D if D else (2 * s.graph_degree if w.vectors.dtype == np.uint8 else 48))
    return ix, ixo


def _rows_equal(ix, ixo, R):
    G = ix.export("G_HS").reshape(-1, R)
    bad = np.flatnonzero((G != ixo.G_HS).any(axis=1))
    assert len(bad) == 0, f"{len(bad)} of {len(G)} rows differ, first {bad[:3]}: {G[bad[0]]} vs {ixo.G_HS[bad[0]]}"


@pytest.mark.parametrize("D", [0, 24, 16])   # 0: the default 2 R; 16 = R: pruning only reorders
def test_pruned_graph_uint8_rows_and_search(vf, tiny, D):
    import torch
    s = tiny.spec
    ix, ixo = _build_both(vf, tiny, D)
    for name in ("S", "O_HS", "M_HS"):
        assert np.array_equal(ix.export(name), getattr(ixo, name)), name
    _rows_equal(ix, ixo, s.graph_degree)
    Q = torch.from_numpy(tiny.queries).cuda()
    for params in (dict(itopk=32, width=1, iters=8, n_seeds=64), dict(itopk=64, width=2, iters=20, n_seeds=0)):
        ids, d = vf.search(ix, Q, tiny.qlabel_offsets, tiny.qlabel_ids, s.k, **params)
        torch.cuda.synchronize()
        io, do = ixo.search(tiny.queries, tiny.qlabel_offsets, tiny.qlabel_ids, s.k, **params)
        assert_exact(to_np(ids), to_np(d), io, do, f"pruned uint8 D={D} {params}")


def test_pruned_graph_float_rows_and_search(vf):
    import torch
    w = make_workload("c2", n=30_000, nq=1500, n_labels=60, n_clusters=64, T=800, graph_degree=32)
    s = w.spec
    ix, ixo = _build_both(vf, w, 0)      # float32 default: degree-48 graphs
    _rows_equal(ix, ixo, s.graph_degree)
    Q = torch.from_numpy(w.queries).cuda()
    params = dict(itopk=32, width=1, iters=8, n_seeds=256)
    ids, d = vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, 10, **params)
    torch.cuda.synchronize()
    io, do, info = ixo.search(w.queries, w.qlabel_offsets, w.qlabel_ids, 10, with_info=True, **params)
    g = info["method"] == 2
    assert g.sum() > 300
    assert_exact(to_np(ids)[g], to_np(d)[g], io[g], do[g], "pruned float graph path")
    assert_close_with_ties(to_np(ids)[~g], to_np(d)[~g], io[~g], do[~g], 1e-4, "float scan path")


def test_pruned_build_rejects_bad_arguments(vf, tiny):
    import torch
    s = tiny.spec
    X = torch.from_numpy(tiny.vectors).cuda()
    for kw in (dict(graph_kind=vf.GRAPH_PRUNED, knn_degree=s.graph_degree - 1),     # D < R
               dict(graph_kind=vf.GRAPH_PRUNED, knn_degree=65),                     # beyond the self-join's candidates
               dict(graph_kind=vf.GRAPH_KNN, knn_degree=32),                        # D without pruning
               dict(graph_kind=7)):
        with pytest.raises(vf.VecflowError):
            vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree, **kw)
    with pytest.raises(vf.VecflowError):                                            # T < D + 1
        vf.build_index(X, tiny.label_offsets, tiny.label_ids, s.n_labels, 20, 16, graph_kind=vf.GRAPH_PRUNED)
