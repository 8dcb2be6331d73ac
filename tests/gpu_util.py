"""Helpers shared by the GPU parity tests."""
import numpy as np


def to_np(t):
    return t.detach().cpu().numpy()


def assert_exact(ids_g, d_g, ids_o, d_o, what=""):
    bad = np.flatnonzero((ids_g != ids_o).any(axis=1) | (d_g.view(np.uint32) != d_o.view(np.uint32)).any(axis=1))
    assert len(bad) == 0, f"{what}: {len(bad)} of {len(ids_g)} rows differ, first {bad[:5]}: " \
                          f"gpu {ids_g[bad[0]]} {d_g[bad[0]]} oracle {ids_o[bad[0]]} {d_o[bad[0]]}"


def assert_close_with_ties(ids_g, d_g, ids_o, d_o, rtol=1e-4, what=""):
    """float scan path: distances within rtol (relative); id sets equal except where
    the differing entries tie, within rtol, with the last distance both sides kept."""
    assert ids_g.shape == ids_o.shape
    for j in range(len(ids_g)):
        vg, vo = ids_g[j] >= 0, ids_o[j] >= 0
        assert vg.sum() == vo.sum(), f"{what} row {j}: result counts differ"
        n = int(vg.sum())
        if n == 0:
            continue
        dg, do = d_g[j][:n].astype(np.float64), d_o[j][:n].astype(np.float64)
        assert np.all(np.abs(dg - do) <= rtol * np.maximum(do, 1e-30)), f"{what} row {j}: distances {dg} vs {do}"
        assert np.all(np.diff(dg) >= -rtol * dg[1:]), f"{what} row {j}: not sorted"
        if np.array_equal(ids_g[j], ids_o[j]):
            continue
        for a, da, b, db in ((ids_g[j][:n], dg, ids_o[j][:n], do), (ids_o[j][:n], do, ids_g[j][:n], dg)):
            for i in np.flatnonzero(~np.isin(a, b)):
                assert abs(da[i] - db[-1]) <= rtol * db[-1], f"{what} row {j}: id {a[i]} is not a boundary tie"
        common = np.intersect1d(ids_g[j][:n], ids_o[j][:n])
        for c in common:
            x, y = dg[ids_g[j][:n] == c][0], do[ids_o[j][:n] == c][0]
            assert abs(x - y) <= rtol * max(y, 1e-30)
