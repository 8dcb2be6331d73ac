"""CPU tests of the host half of a search call (no GPU): ClassifyQueries of Alg. 2, the smallest-list choice of
Section 4.3.2 and the work list of the scan path, through the library's host-only entry point, against the
oracle's routing and against what the work list must satisfy by construction."""
import numpy as np
import pytest

from paper_2506_00812_amd import binding as vf


def _random_batch(rng, n_labels, nq, max_labels=4):
    cnt = rng.integers(1, max_labels + 1, size=nq)
    off = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(cnt, out=off[1:])
    ids = rng.integers(0, n_labels, size=off[-1]).astype(np.int32)
    return off, ids


def _sizes(rng, n_labels, T):
    S = np.where(rng.random(n_labels) < 0.3, rng.integers(T, 6 * T, size=n_labels), rng.integers(0, T, size=n_labels))
    S[rng.integers(0, n_labels, size=3)] = 0          # unknown-but-in-range labels
    S[1], S[2] = T, T - 1                             # the boundary: |C_l| = T is a graph list
    S[3] = S[4] = 77                                  # a tie between two lists
    return S.astype(np.int32)


def test_routing_matches_the_definitions_and_the_paper_example():
    # Section 4.3.2: lists of 10,000 / 1,000 / 5,000 points -> the 1,000-point list is searched
    r = vf.debug_route([10_000, 1_000, 5_000], 2_000, [0, 3], [0, 1, 2])
    assert r["searched"][0] == 1 and r["method"][0] == 1 and r["n_others"][0] == 2
    r = vf.debug_route([10_000, 1_000, 5_000], 1_000, [0, 3], [2, 1, 0])
    assert r["searched"][0] == 1 and r["method"][0] == 2          # |C_l| = T -> graph
    rng = np.random.default_rng(1)
    T = 300
    S = _sizes(rng, 60, T)
    off, ids = _random_batch(rng, 60, 500)
    ids[off[7]:off[8]] = 3                                          # duplicates of one label
    two = int(np.flatnonzero(np.diff(off) >= 2)[0])
    ids[off[two]:off[two] + 2] = [4, 3]                             # equal sizes: the lower label id is searched
    r = vf.debug_route(S, T, off, ids)
    for j in range(500):
        labs = np.unique(ids[off[j]:off[j + 1]])
        if (S[labs] == 0).any():
            assert r["searched"][j] == -1 and r["method"][j] == 0
            continue
        best = min(labs, key=lambda l: (S[l], l))                   # ties go to the lower label id
        assert r["searched"][j] == best
        assert r["method"][j] == (2 if S[best] >= T else 1)
        assert r["n_others"][j] == len(labs) - 1
    # graph queries come out grouped by ascending label, stable in query order
    gq = r["graph_queries"]
    keys = [(r["searched"][j], j) for j in gq]
    assert keys == sorted(keys)
    assert sorted(gq) == sorted(np.flatnonzero(r["method"] == 2))


def test_routing_matches_the_oracle_on_the_tiny_workload(tiny, tiny_oracle):
    s = tiny.spec
    rng = np.random.default_rng(2)
    off, ids = _random_batch(rng, s.n_labels, 400, max_labels=3)
    _, _, info = tiny_oracle.search(tiny.queries[:400], off, ids, 1, itopk=32, width=1, iters=0, with_info=True)
    r = vf.debug_route(tiny_oracle.S, s.T, off, ids)
    assert np.array_equal(r["method"], info["method"])
    assert np.array_equal(r["searched"], info["route_label"])


@pytest.mark.parametrize("tile_rows,seg_groups", [(16, 16), (32, 4), (1, 1), (5, 64)])
def test_scan_work_list_covers_every_tile_and_list_exactly_once(tile_rows, seg_groups):
    rng = np.random.default_rng(3)
    T = 9000
    S = _sizes(rng, 40, T)
    S[5] = T - 1                                                     # a list that needs the most segments
    off, ids = _random_batch(rng, 40, 1500, max_labels=2)
    ids[off[:-1][::3]] = 5                                           # and many queries on it
    r = vf.debug_route(S, T, off, ids, tile_rows=tile_rows, seg_groups=seg_groups)
    scan_q = np.flatnonzero(r["method"] == 1)
    assert sorted(r["scan_rows"]) == sorted(scan_q)                  # every scan query owns exactly one tile row
    items, merges = r["items"], r["merges"]
    # expected layout of the scan partition
    O_LS, GO_LS, n_ls, n_grp = {}, {}, 0, 0
    for l in range(len(S)):
        if 0 < S[l] < T:
            O_LS[l], GO_LS[l] = n_ls, n_grp
            n_ls += S[l]
            n_grp += (S[l] + 31) // 32
    by_map = {v: k for k, v in O_LS.items()}
    tiles = {}
    for group0, map_off, entry0, n, q_begin, q_count, self_base, part_row in items:
        l = by_map[map_off]
        assert self_base == -1 and 1 <= q_count <= tile_rows
        assert (r["searched"][r["scan_rows"][q_begin:q_begin + q_count]] == l).all()    # a tile holds one label's queries
        assert entry0 % 32 == 0 and group0 == GO_LS[l] + entry0 // 32
        tiles.setdefault((q_begin, q_count, l), []).append((entry0, n, part_row))
    covered_rows = 0
    used_part = []
    for (q_begin, q_count, l), segs in tiles.items():
        covered_rows += q_count
        segs.sort()
        assert len(segs) <= 64
        pos = 0
        for entry0, n, part_row in segs:                              # segments tile the list without gap or overlap
            assert entry0 == pos and n > 0
            pos += n
            assert (part_row == -1) == (len(segs) == 1)
            if part_row >= 0:
                used_part.extend(range(part_row, part_row + q_count))
        assert pos == S[l]
        if len(segs) > 1:
            assert all(n == segs[0][1] for _, n, _ in segs[:-1]) and segs[0][1] % 32 == 0
            assert segs[0][1] // 32 >= min(seg_groups, (S[l] + 31) // 32)
    assert covered_rows == len(scan_q)
    assert sorted(used_part) == list(range(r["part_rows"]))           # partial rows are dense and disjoint
    # one merge item per query of a multi-segment tile, pointing at that query's rows
    multi = {(q_begin, q_count, l): segs for (q_begin, q_count, l), segs in tiles.items() if len(segs) > 1}
    assert len(merges) == sum(q for (_, q, _) in multi)
    seen = set()
    for map_off, q, part_row, stride, nseg in merges:
        l = by_map[map_off]
        (q_begin, q_count, _), segs = next((k, v) for k, v in multi.items()
                                           if k[2] == l and q in r["scan_rows"][k[0]:k[0] + k[1]])
        row = list(r["scan_rows"][q_begin:q_begin + q_count]).index(q)
        assert part_row == segs[0][2] + row and stride == q_count and nseg == len(segs)
        seen.add(q)
    assert len(seen) == len(merges)
    assert r["max_nseg"] == max([len(v) for v in tiles.values()] + [1])


def test_routing_rejects_bad_batches():
    S = np.array([5, 0, 7], dtype=np.int32)
    with pytest.raises(vf.VecflowError, match="at least one label"):
        vf.debug_route(S, 4, [0, 0], np.zeros(0, dtype=np.int32))
    with pytest.raises(vf.VecflowError, match="outside"):
        vf.debug_route(S, 4, [0, 1], [3])
    with pytest.raises(vf.VecflowError, match="more than 8"):
        vf.debug_route(np.arange(1, 20, dtype=np.int32), 4, [0, 9], np.arange(9))
