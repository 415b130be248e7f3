"""The seeded input generators: structure of what they emit, and determinism."""
import numpy as np
import pytest

import workloads as wl

SMALL = {
    "tiny": {},
    "citation": dict(n=3000, p_in=3e-3, p_out=2e-4),
    "collaboration": dict(n=4000),
    "protein": dict(n=1500, knn=24),
    "rmat": dict(scale=11, edge_factor=8),
}


@pytest.mark.parametrize("name", wl.CONFIGS)
def test_graph_is_symmetric_binary_csr(name):
    g = wl.make_graph(name, **SMALL[name])
    assert g.rowptr.dtype == np.int64 and g.colidx.dtype == np.int32
    assert g.rowptr[0] == 0 and g.rowptr[-1] == len(g.colidx) and len(g.rowptr) == g.n + 1
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    assert not np.any(rows == g.colidx), "self-loops must be removed"
    assert g.colidx.min() >= 0 and g.colidx.max() < g.n
    key = rows.astype(np.int64) * g.n + g.colidx
    assert np.all(np.diff(key) > 0), "columns sorted and unique within rows"
    assert np.array_equal(np.sort(g.colidx.astype(np.int64) * g.n + rows), key), "symmetric"
    g2 = wl.make_graph(name, **SMALL[name])
    assert np.array_equal(g.rowptr, g2.rowptr) and np.array_equal(g.colidx, g2.colidx)


def test_features_and_weights():
    x = wl.integer_features(100, 16, 1)
    assert x.dtype == np.float32 and x.min() >= -8 and x.max() <= 8 and np.array_equal(x, np.round(x))
    g = wl.gaussian_features(1000, 8, 1)
    assert g.dtype == np.float32 and abs(float(g.mean())) < 0.1 and abs(float(g.std()) - 1) < 0.1
    w = wl.glorot_uniform(500, 64, 1)
    assert w.shape == (500, 64) and np.abs(w).max() <= np.sqrt(6 / 564)
    assert np.array_equal(w, wl.glorot_uniform(500, 64, 1))
