"""Pins for the CPU oracle: each check ties it to something other than itself --
a hand-worked example, closed forms, library routines, exhaustive search."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import cbm_oracle as orc


def _csr(rows, n=None):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in sorted(r)], dtype=np.int32)
    return rowptr, colidx


def _random_rows(rng, m, n, density):
    return [sorted(np.flatnonzero(rng.random(n) < density).tolist()) for _ in range(m)]


@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_example.json")) as f:
        return json.load(f)


# ----------------------------- hand-worked example ------------------------- #
def test_worked_example_distance_graph(worked):
    rowptr, colidx = _csr(worked["rows"])
    rows = orc.adjacency_lists(worked["m"], rowptr, colidx)
    W = orc.hamming_distance_graph(rows)
    assert W.tolist() == worked["hamming"]


def test_worked_example_tree_deltas_ops(worked):
    rowptr, colidx = _csr(worked["rows"])
    rows, r, dplus, dminus = orc.build_cbm(worked["m"], rowptr, colidx, alpha=0)
    g = worked["alpha0"]
    assert r.tolist() == g["r"]
    assert [list(d) for d in dplus] == g["dplus"]
    assert [list(d) for d in dminus] == g["dminus"]
    assert sum(len(d) for d in dplus) + sum(len(d) for d in dminus) == g["tree_weight"]
    ops = orc.scalar_ops(rows, r, dplus, dminus)
    assert ops.tolist() == g["scalar_ops"]
    assert ops.sum() <= g["nnz"]


def test_worked_example_products(worked):
    rowptr, colidx = _csr(worked["rows"])
    X = np.array(worked["X"], dtype=np.float32)
    want = np.array(worked["AX"], dtype=np.float64)
    rows, r, dplus, dminus = orc.build_cbm(worked["m"], rowptr, colidx, alpha=0)
    assert np.array_equal(orc.spmm_dense(orc.dense_from_csr(6, 6, rowptr, colidx), X), want)
    assert np.array_equal(orc.spmm_csr(rowptr, colidx, X), want)
    assert np.array_equal(orc.cbm_matmul(r, dplus, dminus, X), want)
    assert np.array_equal(orc.cbm_matmul_two_stage(r, dplus, dminus, X, 6), want)
    assert np.array_equal(orc.spmm_csr(rowptr, colidx, X, rows=[5, 2]), want[[5, 2]])


def test_worked_example_alpha(worked):
    rowptr, colidx = _csr(worked["rows"])
    for a, weight in worked["alpha_tree_weight"].items():
        rows, r, dplus, dminus = orc.build_cbm(worked["m"], rowptr, colidx, alpha=int(a))
        got = sum(len(d) for d in dplus) + sum(len(d) for d in dminus)
        assert got == weight, (a, got)
    _, r, _, _ = orc.build_cbm(worked["m"], rowptr, colidx, alpha=3)
    for x, want in enumerate(worked["alpha3_r"]):
        assert r[x] in (want if isinstance(want, list) else [want])


# ----------------------------- structure: library + brute force ------------ #
@pytest.mark.parametrize("seed", range(6))
def test_mst_weight_matches_scipy(seed):
    from scipy.sparse.csgraph import minimum_spanning_tree

    rng = np.random.default_rng(seed)
    m, n = 14, 10
    rows = _random_rows(rng, m, n, 0.4)
    rows[3] = list(rows[2])  # identical rows: a zero-weight edge
    rowptr, colidx = _csr(rows)
    R = orc.adjacency_lists(m, rowptr, colidx)
    W = orc.hamming_distance_graph(R)
    r = orc.mst_rooted_at_virtual(W)
    got = sum(int(W[r[x], x]) for x in range(1, m + 1))
    # scipy treats 0 as "no edge": shift every weight by +1, m edges in the tree
    T = minimum_spanning_tree(np.triu(W + 1, k=1))
    assert got == int(T.sum()) - m
    # draw rule: a compressed row always needs strictly fewer deltas than its nnz
    for x in range(1, m + 1):
        if r[x] != 0:
            assert W[r[x], x] < W[0, x]


def _brute_force_arborescence(W, keep):
    V = W.shape[0]
    best = None
    for par in itertools.product(range(V), repeat=V - 1):
        ok, cost = True, 0
        for x, y in enumerate(par, start=1):
            if y == x or not keep[y, x]:
                ok = False
                break
            cost += int(W[y, x])
        if not ok:
            continue
        for x in range(1, V):  # every vertex must reach 0
            v, steps = x, 0
            while v != 0 and steps <= V:
                v, steps = par[v - 1], steps + 1
            if v != 0:
                ok = False
                break
        if ok and (best is None or cost < best):
            best = cost
    return best


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("alpha", [0, 1, 2])
def test_arborescence_weight_matches_exhaustive_search(seed, alpha):
    rng = np.random.default_rng(100 + seed)
    m, n = 5, 6
    rows = _random_rows(rng, m, n, 0.55)
    rowptr, colidx = _csr(rows)
    R = orc.adjacency_lists(m, rowptr, colidx)
    W = orc.hamming_distance_graph(R)
    keep = orc.admissible_edges(W, alpha)
    r = orc.mca_rooted_at_virtual(W, keep)
    got = sum(int(W[r[x], x]) for x in range(1, m + 1))
    assert got == _brute_force_arborescence(W, keep)
    if alpha == 0:  # undirected MST = directed optimum when nothing useful is pruned
        r0 = orc.mst_rooted_at_virtual(W)
        assert sum(int(W[r0[x], x]) for x in range(1, m + 1)) == _brute_force_arborescence(
            W, np.ones_like(keep) & ~np.eye(m + 1, dtype=bool) & (np.arange(m + 1)[None, :] > 0))


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("alpha", [1, 3])
def test_arborescence_weight_matches_networkx(seed, alpha):
    import networkx as nx

    rng = np.random.default_rng(200 + seed)
    m, n = 16, 12
    rows = _random_rows(rng, m, n, 0.45)
    rowptr, colidx = _csr(rows)
    R = orc.adjacency_lists(m, rowptr, colidx)
    W = orc.hamming_distance_graph(R)
    keep = orc.admissible_edges(W, alpha)
    r = orc.mca_rooted_at_virtual(W, keep)
    G = nx.DiGraph()
    for y in range(m + 1):
        for x in range(1, m + 1):
            if keep[y, x]:
                G.add_edge(y, x, weight=int(W[y, x]))
    T = nx.minimum_spanning_arborescence(G)
    assert sum(int(W[r[x], x]) for x in range(1, m + 1)) == sum(d["weight"] for _, _, d in T.edges(data=True))
    # alpha rule on every non-virtual tree edge; per-row cost never above nnz
    for x in range(1, m + 1):
        if r[x] != 0:
            assert W[r[x], x] <= W[0, x] - alpha
            assert 1 + W[r[x], x] <= W[0, x]


@pytest.mark.parametrize("alpha", [0, 2])
@pytest.mark.parametrize("self_loops", [False, True])
def test_round_trip_and_properties(alpha, self_loops):
    rng = np.random.default_rng(7)
    m = n = 24
    rows = _random_rows(rng, m, n, 0.3)
    rows[5] = []
    rows[9] = list(rows[8])
    rowptr, colidx = _csr(rows)
    R, r, dplus, dminus = orc.build_cbm(m, rowptr, colidx, alpha=alpha, add_self_loops=self_loops)
    assert orc.decompress(r, dplus, dminus) == R                      # Eq. (2)
    nnz = sum(len(a) for a in R)
    nd = sum(len(d) for d in dplus) + sum(len(d) for d in dminus)
    assert nd <= nnz                                                   # Property 1
    ops = orc.scalar_ops(R, r, dplus, dminus)
    assert all(ops[x] <= len(R[x]) for x in range(1, m + 1))           # Property 2, per row
    assert len(orc.topological_order(r)) == m                          # m tree edges, all reach 0
    X = rng.integers(-8, 9, size=(n, 3)).astype(np.float32)
    want = np.array([[sum(X[j, k] for j in R[x]) for k in range(3)] for x in range(1, m + 1)])
    assert np.array_equal(orc.cbm_matmul(r, dplus, dminus, X), want)
    assert np.array_equal(orc.cbm_matmul_two_stage(r, dplus, dminus, X, n), want)


def test_lower_triangular_is_cumsum():
    m = 20
    rows = [list(range(i + 1)) for i in range(m)]
    rowptr, colidx = _csr(rows)
    R, r, dplus, dminus = orc.build_cbm(m, rowptr, colidx)
    assert sum(len(d) for d in dplus) == m and sum(len(d) for d in dminus) == 0
    assert [int(r[x]) for x in range(1, m + 1)] == list(range(m))     # the chain 0 -> 1 -> ... -> m
    X = np.random.default_rng(1).integers(-8, 9, size=(m, 4)).astype(np.float32)
    want = np.cumsum(X.astype(np.float64), axis=0)
    assert np.array_equal(orc.cbm_matmul(r, dplus, dminus, X), want)
    assert np.array_equal(orc.spmm_csr(rowptr, colidx, X), want)


def test_identical_rows_cost_one_op_each():
    m, row = 9, [1, 4, 5, 7]
    rowptr, colidx = _csr([row] * m)
    R, r, dplus, dminus = orc.build_cbm(m, rowptr, colidx)
    assert sum(len(d) for d in dplus) + sum(len(d) for d in dminus) == len(row)
    assert orc.scalar_ops(R, r, dplus, dminus).sum() == len(row) + (m - 1)


def test_huge_alpha_is_plain_csr():
    rng = np.random.default_rng(3)
    m, n = 12, 9
    rows = _random_rows(rng, m, n, 0.5)
    rowptr, colidx = _csr(rows)
    R, r, dplus, dminus = orc.build_cbm(m, rowptr, colidx, alpha=10 ** 6)
    assert all(r[x] == 0 for x in range(1, m + 1))
    assert [list(d) for d in dplus[1:]] == rows and not any(dminus)


# ----------------------------- products: closed forms ---------------------- #
def _graph_csr(n, edges):
    adj = [set() for _ in range(n)]
    for u, v in edges:
        adj[u].add(v)
        adj[v].add(u)
    return _csr([sorted(a) for a in adj])


def test_normalized_complete_graph_is_column_mean():
    n = 7
    rowptr, colidx = _graph_csr(n, itertools.combinations(range(n), 2))
    X = np.random.default_rng(0).standard_normal((n, 5)).astype(np.float32)
    want = np.tile(X.astype(np.float64).mean(axis=0), (n, 1))
    np.testing.assert_allclose(orc.spmm_csr_normalized(rowptr, colidx, X), want, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(orc.normalized_dense(orc.dense_from_csr(n, n, rowptr, colidx)) @ X, want,
                               rtol=1e-14, atol=1e-15)


def test_normalized_cycle_is_three_point_average():
    n = 11
    rowptr, colidx = _graph_csr(n, [(i, (i + 1) % n) for i in range(n)])
    X = np.random.default_rng(1).standard_normal((n, 3)).astype(np.float64)
    want = (np.roll(X, 1, axis=0) + X + np.roll(X, -1, axis=0)) / 3.0
    np.testing.assert_allclose(orc.spmm_csr_normalized(rowptr, colidx, X), want, rtol=1e-14, atol=1e-15)


def test_normalized_path_graph_by_hand():
    # path 0-1-2: d = (2,3,2); row 0 of A_hat X = x0/2 + x1/sqrt(6); row 1 = x0/sqrt6 + x1/3 + x2/sqrt6
    rowptr, colidx = _graph_csr(3, [(0, 1), (1, 2)])
    X = np.array([[6.0], [6.0], [12.0]])
    got = orc.spmm_csr_normalized(rowptr, colidx, X)
    want = np.array([[3 + 6 / math.sqrt(6)], [18 / math.sqrt(6) + 2], [6 / math.sqrt(6) + 6]])
    np.testing.assert_allclose(got, want, rtol=1e-15)
    assert orc.degrees_with_self_loops(rowptr, colidx).tolist() == [2, 3, 2]


def test_normalized_eigenvector_symmetry_and_existing_diagonal():
    rng = np.random.default_rng(5)
    n = 30
    edges = [(int(u), int(v)) for u, v in rng.integers(0, n, size=(70, 2)) if u != v]
    rowptr, colidx = _graph_csr(n, edges)
    d = orc.degrees_with_self_loops(rowptr, colidx).astype(np.float64)
    v = np.sqrt(d)[:, None]
    np.testing.assert_allclose(orc.spmm_csr_normalized(rowptr, colidx, v), v, rtol=1e-13)  # A_hat D^1/2 1 = D^1/2 1
    a, b = rng.standard_normal((n, 1)), rng.standard_normal((n, 1))
    lhs = (a * orc.spmm_csr_normalized(rowptr, colidx, b)).sum()
    rhs = (orc.spmm_csr_normalized(rowptr, colidx, a) * b).sum()
    assert abs(lhs - rhs) < 1e-12
    # a diagonal entry already in A is not counted twice (A + I read as A v I)
    rows = [[0, 1], [0]]
    rp, ci = _csr(rows)
    assert orc.degrees_with_self_loops(rp, ci).tolist() == [2, 2]
    np.testing.assert_allclose(orc.normalized_dense(orc.dense_from_csr(2, 2, rp, ci)), [[0.5, 0.5], [0.5, 0.5]])
    np.testing.assert_allclose(orc.spmm_csr_normalized(rp, ci, np.array([[2.0], [4.0]])), [[3.0], [3.0]])


def test_normalized_cbm_form_matches_definition():
    rng = np.random.default_rng(11)
    n = 26
    edges = [(int(u), int(v)) for u, v in rng.integers(0, n, size=(90, 2)) if u != v]
    rowptr, colidx = _graph_csr(n, edges)
    X = rng.standard_normal((n, 4)).astype(np.float32)
    A_hat = orc.normalized_dense(orc.dense_from_csr(n, n, rowptr, colidx))
    want = A_hat @ X.astype(np.float64)
    np.testing.assert_allclose(orc.spmm_csr_normalized(rowptr, colidx, X), want, rtol=1e-13, atol=1e-14)
    d = orc.degrees_with_self_loops(rowptr, colidx)
    for alpha in (0, 2):
        _, r, dplus, dminus = orc.build_cbm(n, rowptr, colidx, alpha=alpha, add_self_loops=True)
        got = orc.cbm_matmul_normalized(r, dplus, dminus, d, X)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_regular_graph_normalized_is_exact_on_integers():
    # 3-regular circulant: d = 4, d^-1/2 = 1/2 exactly, so A_hat X = (A v I) X / 4 with no rounding
    n = 16
    rowptr, colidx = _graph_csr(n, [(i, (i + 1) % n) for i in range(n)] + [(i, (i + 8) % n) for i in range(8)])
    X = np.random.default_rng(2).integers(-8, 9, size=(n, 4)).astype(np.float32)
    want = (np.roll(X, 1, 0) + np.roll(X, -1, 0) + np.roll(X, 8, 0) + X).astype(np.float64) / 4.0
    assert np.array_equal(orc.spmm_csr_normalized(rowptr, colidx, X), want)


def test_linearity_on_integers():
    rng = np.random.default_rng(4)
    m, n = 15, 12
    rowptr, colidx = _csr(_random_rows(rng, m, n, 0.4))
    _, r, dplus, dminus = orc.build_cbm(m, rowptr, colidx)
    X, Z = (rng.integers(-8, 9, size=(n, 3)).astype(np.float32) for _ in range(2))
    lhs = orc.cbm_matmul(r, dplus, dminus, 3 * X - 2 * Z)
    assert np.array_equal(lhs, 3 * orc.cbm_matmul(r, dplus, dminus, X) - 2 * orc.cbm_matmul(r, dplus, dminus, Z))


# ----------------------------- GCN ----------------------------------------- #
def test_gcn2_against_dense_definition_and_closed_form():
    rng = np.random.default_rng(9)
    n, f, h, c = 18, 7, 5, 3
    edges = [(int(u), int(v)) for u, v in rng.integers(0, n, size=(40, 2)) if u != v]
    rowptr, colidx = _graph_csr(n, edges)
    X = rng.standard_normal((n, f)).astype(np.float32)
    W0 = rng.standard_normal((f, h)).astype(np.float32)
    W1 = rng.standard_normal((h, c)).astype(np.float32)
    A_hat = orc.normalized_dense(orc.dense_from_csr(n, n, rowptr, colidx))
    Xd, W0d, W1d = (a.astype(np.float64) for a in (X, W0, W1))
    want = A_hat @ np.maximum(A_hat @ Xd @ W0d, 0.0) @ W1d           # Eq. (1), left to right
    np.testing.assert_allclose(orc.gcn2(rowptr, colidx, X, W0, W1), want, rtol=1e-12, atol=1e-13)
    # complete graph, non-negative inputs: every output row = mean(X) W0 W1 (ReLU inactive)
    rowptr, colidx = _graph_csr(6, itertools.combinations(range(6), 2))
    X, W0, W1 = np.abs(X[:6]), np.abs(W0), W1
    want = np.tile(X.astype(np.float64).mean(0) @ W0.astype(np.float64) @ W1.astype(np.float64), (6, 1))
    np.testing.assert_allclose(orc.gcn2(rowptr, colidx, X, W0, W1), want, rtol=1e-12)


# ----------------------------- mean and GIN aggregators -------------------- #
def test_mean_and_gin_closed_forms():
    # complete graph without self loops: mean over the other n-1 rows; GIN = column sum + eps x_i
    n, eps = 7, 0.25
    rowptr, colidx = _graph_csr(n, itertools.combinations(range(n), 2))
    X = np.random.default_rng(2).standard_normal((n, 4))
    tot = X.sum(axis=0)
    np.testing.assert_allclose(orc.spmm_csr_mean(rowptr, colidx, X), (tot[None, :] - X) / (n - 1), rtol=1e-13)
    np.testing.assert_allclose(orc.spmm_csr_gin(rowptr, colidx, X, eps), tot[None, :] + eps * X, rtol=1e-13,
                               atol=1e-14)
    # cycle: two-point average; GIN with eps = -1 is the plain product
    n = 9
    rowptr, colidx = _graph_csr(n, [(i, (i + 1) % n) for i in range(n)])
    X = np.random.default_rng(3).integers(-8, 9, size=(n, 3)).astype(np.float64)
    assert np.array_equal(orc.spmm_csr_mean(rowptr, colidx, X), (np.roll(X, 1, 0) + np.roll(X, -1, 0)) / 2.0)
    assert np.array_equal(orc.spmm_csr_gin(rowptr, colidx, X, -1.0), orc.spmm_csr(rowptr, colidx, X))
    assert np.array_equal(orc.spmm_csr_gin(rowptr, colidx, X, 1.0), np.roll(X, 1, 0) + np.roll(X, -1, 0) + 2 * X)


def test_mean_and_gin_against_dense_definition():
    rng = np.random.default_rng(12)
    n = 21
    rows = _random_rows(rng, n, n, 0.25)
    rows[4] = []                                    # an empty row: mean gives zeros, GIN gives (1+eps) x_i
    rowptr, colidx = _csr(rows, n)
    A = orc.dense_from_csr(n, n, rowptr, colidx)
    X = rng.standard_normal((n, 5))
    deg = A.sum(axis=1)
    Dinv = np.diag([1.0 / d if d else 0.0 for d in deg])
    np.testing.assert_allclose(orc.spmm_csr_mean(rowptr, colidx, X), Dinv @ A @ X, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(orc.spmm_csr_gin(rowptr, colidx, X, 0.5), (A + 1.5 * np.eye(n)) @ X, rtol=1e-13,
                               atol=1e-14)
    assert not orc.spmm_csr_mean(rowptr, colidx, X)[4].any()
    sub = [3, 4, 17]
    assert np.array_equal(orc.spmm_csr_mean(rowptr, colidx, X, rows=sub), orc.spmm_csr_mean(rowptr, colidx, X)[sub])
    assert np.array_equal(orc.spmm_csr_gin(rowptr, colidx, X, 0.5, rows=sub),
                          orc.spmm_csr_gin(rowptr, colidx, X, 0.5)[sub])
