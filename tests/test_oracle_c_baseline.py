"""The oracle's plain-C CSR products against the pinned numpy oracle and a closed form."""
import itertools

import numpy as np

import workloads as wl
from oracle import cbm_oracle as orc
from oracle import csr_ref


def test_c_products_match_numpy_oracle():
    g = wl.collaboration_graph(n=3000)
    X = wl.gaussian_features(g.n, 20, 3)
    np.testing.assert_allclose(csr_ref.spmm_f64(g.rowptr, g.colidx, X), orc.spmm_csr(g.rowptr, g.colidx, X),
                               rtol=1e-13, atol=1e-13)
    d = orc.degrees_with_self_loops(g.rowptr, g.colidx)
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
    np.testing.assert_allclose(csr_ref.spmm_norm_f64(g.rowptr, g.colidx, d, X), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(csr_ref.spmm_norm_f64(g.rowptr, g.colidx, d, X, 100, 900), ref[100:900], rtol=1e-12,
                               atol=1e-13)
    s = (1.0 / np.sqrt(d)).astype(np.float32)
    got = csr_ref.spmm_norm_omp_f32(g.rowptr, g.colidx, s, X)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
    assert csr_ref.omp_threads() >= 1


def test_c_normalized_complete_graph_is_column_mean():
    n = 9
    adj = [[j for j in range(n) if j != i] for i in range(n)]
    rowptr = np.arange(0, n * (n - 1) + 1, n - 1, dtype=np.int64)
    colidx = np.array(list(itertools.chain.from_iterable(adj)), dtype=np.int32)
    X = np.random.default_rng(0).standard_normal((n, 4)).astype(np.float32)
    want = np.tile(X.astype(np.float64).mean(0), (n, 1))
    np.testing.assert_allclose(csr_ref.spmm_norm_f64(rowptr, colidx, np.full(n, n), X), want, rtol=1e-13)
