"""Parity at the full size of the two large configurations, in the launch configuration and at the operating
points bench.py reports for them: the YFCC-like one (1e7 x 192 uint8, 200,000 labels, 100,000 queries of
which 30 % are two-label ANDs, T = 2,000) and the multi-label stress one (5e6 x 96 float32, 10,000 labels,
100,000 two-label AND queries, T = 5,000).  The whole batch runs on the GPU; sampled queries are compared
with the oracle, which builds the graph rows it needs lazily by brute force over the list (lists of up to
7.8 million vectors), independently of the GPU.  Each step prints a line: an index build at this size takes
minutes."""
import sys
import time

import numpy as np
import pytest

from oracle import OracleIndex
from paper_2506_00812_amd.workloads import make_workload
from tests.gpu_util import assert_close_with_ties, assert_exact, to_np

pytestmark = pytest.mark.gpu

C3_PARAMS = dict(itopk=32, width=1, iters=32, n_seeds=16384)
C5_PARAMS = dict(itopk=32, width=1, iters=16, n_seeds=32768)


class Steps:
    """Progress lines on the real stdout (pytest's capture suspended), one per completed step."""

    def __init__(self, capsys, tag):
        self.capsys, self.tag, self.t0 = capsys, tag, time.time()

    def __call__(self, what):
        with self.capsys.disabled():
            sys.stdout.write(f"\n[{self.tag} +{time.time() - self.t0:5.0f}s] {what}")
            sys.stdout.flush()


def sub_csr(w, sample):
    qo = np.zeros(len(sample) + 1, dtype=np.int64)
    np.cumsum(np.diff(w.qlabel_offsets)[sample], out=qo[1:])
    ql = np.concatenate([w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j + 1]] for j in sample])
    return qo, ql


def spread_heavy(heavy, light):
    """Order a sample so that the expensive queries start blocks of four (the oracle hands its threads four
    consecutive queries at a time)."""
    out, light = [], list(light)
    for h in heavy:
        out.append(h)
        out.extend(light[:3])
        light = light[3:]
    return np.array(out + light, dtype=np.int64)


def test_c3_full_size_sampled_against_oracle(capsys):
    import torch
    from paper_2506_00812_amd import binding as vf
    step = Steps(capsys, "c3 1e7")
    w = make_workload("c3")
    s = w.spec
    step(f"workload drawn: {s.n} x {s.dim} {s.dtype}, {len(w.label_ids)} label draws, {s.nq} queries")
    X = torch.from_numpy(w.vectors).cuda()
    Q = torch.from_numpy(w.queries).cuda()
    ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree)
    torch.cuda.synchronize()
    st = ix.stats()
    step(f"GPU index built: {st['n_graph_labels']} graph lists ({st['n_HS']} postings), {st['n_scan_labels']} scan lists")
    ixo = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree, lazy_graph=True)
    for name in ("S", "O_HS", "O_LS", "M_HS", "M_LS"):
        assert np.array_equal(ix.export(name), getattr(ixo, name)), name
    S = ixo.S
    assert S.max() > 5_000_000 and (S >= 1_000_000).sum() >= 5
    step("oracle posting lists built and equal to the GPU's")

    ids, dists = vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, s.k, **C3_PARAMS)   # whole batch, as bench.py runs it
    torch.cuda.synchronize()
    ids, dists = to_np(ids), to_np(dists)
    step("GPU search of the whole batch done")
    # the same batch with the selection fused into the seed kernel (runs of keys instead of the 5.9 GB distance
    # matrix): every row must come out the same
    ix.tune("seed_select", 1)
    ids2, dists2 = vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, s.k, **C3_PARAMS)
    torch.cuda.synchronize()
    ix.tune("seed_select", 0)
    assert np.array_equal(to_np(ids2), ids) and np.array_equal(to_np(dists2), dists)
    del ids2, dists2
    step("seed kernel with fused selection: same results")

    nlab = np.diff(w.qlabel_offsets)
    first = w.qlabel_ids[w.qlabel_offsets[:-1]]
    rng = np.random.default_rng(31)
    single = nlab == 1
    heavy = rng.choice(np.flatnonzero(single & (S[first] > 1_000_000)), size=4, replace=False)
    mid = rng.choice(np.flatnonzero(single & (S[first] >= s.T) & (S[first] <= 1_000_000)), size=6, replace=False)
    scan = rng.choice(np.flatnonzero(single & (S[first] < s.T)), size=6, replace=False)
    two = rng.choice(np.flatnonzero(nlab == 2), size=10, replace=False)
    sample = spread_heavy(heavy, np.concatenate([mid, scan, two]))
    qo, ql = sub_csr(w, sample)
    io, do, info = ixo.search(w.queries[sample], qo, ql, s.k, with_info=True, **C3_PARAMS)
    step(f"oracle searched {len(sample)} sampled queries (lazy rows over lists of up to {S[first[heavy]].max()} vectors)")
    and_rows = nlab[sample] == 2
    assert and_rows.sum() >= 8 and (info["method"][and_rows] == 2).sum() >= 2
    assert (info["method"] == 2).sum() >= 12 and (info["method"] == 1).sum() >= 6
    assert_exact(ids[sample], dists[sample], io, do, "c3 full size, sampled")

    # exact mode (the recall ground truth) on the same sample
    gi, gd = vf.search_exact(ix, Q[torch.from_numpy(sample).cuda()].contiguous(), qo, ql, s.k)
    eo, ed = ixo.search(w.queries[sample], qo, ql, s.k, force_scan=True)
    assert_exact(to_np(gi), to_np(gd), eo, ed, "c3 full size, exact")
    step("exact mode equal")

    # properties of every row of the batch
    finite = ids >= 0
    asc = np.where(finite, dists, np.inf)
    assert (asc[:, 1:] >= asc[:, :-1]).all()
    assert np.isinf(dists[~finite]).all()
    M_HS, M_LS, O_HS, O_LS = ixo.M_HS, ixo.M_LS, ixo.O_HS, ixo.O_LS
    for j in range(0, s.nq, 997):
        for l in w.qlabel_ids[w.qlabel_offsets[j]:w.qlabel_offsets[j + 1]]:
            lst = M_HS[O_HS[l]:O_HS[l] + S[l]] if O_HS[l] >= 0 else M_LS[O_LS[l]:O_LS[l] + S[l]]
            assert np.isin(ids[j][finite[j]], lst).all()
        r = ids[j][finite[j]]
        assert len(np.unique(r)) == len(r)
        d = ((w.vectors[r].astype(np.int64) - w.queries[j].astype(np.int64)[None, :]) ** 2).sum(axis=1)
        assert np.array_equal(d.astype(np.float32), dists[j][finite[j]])
    step("whole-batch properties hold")


def test_c5_full_size_and_queries_sampled_against_oracle(capsys):
    import oracle
    import torch
    from paper_2506_00812_amd import binding as vf
    step = Steps(capsys, "c5 5e6")
    w = make_workload("c5")
    s = w.spec
    step(f"workload drawn: {s.n} x {s.dim} {s.dtype}, {s.nq} two-label AND queries")
    X = torch.from_numpy(w.vectors).cuda()
    Q = torch.from_numpy(w.queries).cuda()
    ix = vf.build_index(X, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree)
    torch.cuda.synchronize()
    st = ix.stats()
    step(f"GPU index built: {st['n_graph_labels']} graph lists ({st['n_HS']} postings), {st['n_scan_labels']} scan lists")
    ixo = OracleIndex(w.vectors, w.label_offsets, w.label_ids, s.n_labels, s.T, s.graph_degree, lazy_graph=True)
    for name in ("S", "O_HS", "O_LS", "M_HS", "M_LS"):
        assert np.array_equal(ix.export(name), getattr(ixo, name)), name
    step("oracle posting lists built and equal to the GPU's")

    ids, dists = vf.search(ix, Q, w.qlabel_offsets, w.qlabel_ids, s.k, **C5_PARAMS)
    idp, ddp = vf.search_multi(ix, Q, w.qlabel_offsets, w.qlabel_ids, vf.AND_PARALLEL, s.k, **C5_PARAMS)
    torch.cuda.synchronize()
    ids, dists, idp, ddp = to_np(ids), to_np(dists), to_np(idp), to_np(ddp)
    step("GPU searches of the whole batch done (greedy and parallel policy)")

    S = ixo.S
    la, lb = w.qlabel_ids[w.qlabel_offsets[:-1]], w.qlabel_ids[w.qlabel_offsets[:-1] + 1]
    smallest = np.minimum(S[la], S[lb])
    rng = np.random.default_rng(32)
    gq, sq = np.flatnonzero(smallest >= s.T), np.flatnonzero(smallest < s.T)
    assert len(gq) > 1000 and len(sq) > 1000
    big = np.flatnonzero(smallest >= 200_000)
    heavy = rng.choice(big, size=min(4, len(big)), replace=False)
    sample = spread_heavy(heavy, np.concatenate([rng.choice(gq, size=12, replace=False), rng.choice(sq, size=8, replace=False)]))
    qo, ql = sub_csr(w, sample)
    io, do, info = ixo.search(w.queries[sample], qo, ql, s.k, with_info=True, **C5_PARAMS)
    step(f"oracle searched {len(sample)} sampled queries, greedy policy")
    g = info["method"] == 2
    assert g.sum() >= 12 and (~g).sum() >= 8
    assert_exact(ids[sample][g], dists[sample][g], io[g], do[g], "c5 full size greedy AND, graph")
    assert_close_with_ties(ids[sample][~g], dists[sample][~g], io[~g], do[~g], 1e-4, "c5 full size greedy AND, scan")
    ip, dp = ixo.search_multi(w.queries[sample], qo, ql, oracle.AND_PARALLEL, s.k, **C5_PARAMS)
    step("oracle searched the sample with the parallel policy")
    assert_exact(idp[sample][g], ddp[sample][g], ip[g], dp[g], "c5 full size parallel AND, graph")
    assert_close_with_ties(idp[sample][~g], ddp[sample][~g], ip[~g], dp[~g], 1e-4, "c5 full size parallel AND, scan")

    # every returned id carries both labels (through the exported posting lists), rows ascend
    M_HS, M_LS, O_HS, O_LS = ixo.M_HS, ixo.M_LS, ixo.O_HS, ixo.O_LS
    for res_i, res_d in ((ids, dists), (idp, ddp)):
        finite = res_i >= 0
        asc = np.where(finite, res_d, np.inf)
        assert (asc[:, 1:] >= asc[:, :-1]).all()
        for j in range(0, s.nq, 1999):
            for l in (la[j], lb[j]):
                lst = M_HS[O_HS[l]:O_HS[l] + S[l]] if O_HS[l] >= 0 else M_LS[O_LS[l]:O_LS[l] + S[l]]
                assert np.isin(res_i[j][finite[j]], lst).all()
    step("whole-batch properties hold")
