"""GPU parity: libcbm (through its C ABI binding) against the CPU oracle, element
by element, on the same seeded inputs.  Integer-valued features must match
bit for bit; Gaussian features within 1e-5 row-scaled max-norm relative error."""
import numpy as np
import pytest

import workloads as wl
from oracle import cbm_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2409_02208_amd as cbm

    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch, cbm


def row_scaled_error(got: np.ndarray, ref: np.ndarray, scale_from: np.ndarray = None) -> float:
    """max_i ( max_j |got - ref|[i,j] / max_j |ref|[i,j] ); rows whose reference is all zero must be exact.
    ``scale_from`` supplies the row scale when ``ref`` went through a ReLU: the rounding error of a row is
    relative to its pre-activation magnitude, which the clipping may have removed from ``ref``."""
    got = got.astype(np.float64)
    diff = np.abs(got - ref).max(axis=1) if ref.size else np.zeros(0)
    scale = np.abs(ref if scale_from is None else scale_from).max(axis=1) if ref.size else np.zeros(0)
    zero = scale == 0
    assert np.all(diff[zero] == 0), "rows with an all-zero reference must be exactly zero"
    return float((diff[~zero] / scale[~zero]).max()) if np.any(~zero) else 0.0


def _csr(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in sorted(r)], dtype=np.int32)
    return rowptr, colidx


def _run(env, fn_name, h, X, m, poison=True):
    torch, cbm = env
    Xd = torch.from_numpy(X).cuda()
    Y = torch.full((m, X.shape[1]), float("nan"), device="cuda") if poison else torch.empty((m, X.shape[1]), device="cuda")
    getattr(cbm, fn_name)(h, Xd, Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


SMALL = {
    "tiny": {},
    "citation": dict(n=6000, p_in=1.5e-3, p_out=1e-4),
    "collaboration": dict(n=20000),
    "protein": dict(n=6000, knn=60),
    "rmat": dict(scale=14, edge_factor=16),
}


@pytest.fixture(scope="module")
def graphs():
    return {name: wl.make_graph(name, **kw) for name, kw in SMALL.items()}


@pytest.mark.parametrize("name", wl.CONFIGS)
@pytest.mark.parametrize("k", [16, 128])
def test_spmm_integer_features_bit_exact(env, graphs, name, k):
    torch, cbm = env
    g = graphs[name]
    X = wl.integer_features(g.n, k, g.meta["seed"])
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=16)
    got = _run(env, "cbm_spmm", h, X, g.n)
    ref = orc.spmm_csr(g.rowptr, g.colidx, X)
    assert np.abs(ref).max() < 2 ** 24
    assert np.array_equal(got.astype(np.float64), ref)
    again = _run(env, "cbm_spmm", h, X, g.n)
    assert np.array_equal(got, again)


@pytest.mark.parametrize("name", wl.CONFIGS)
@pytest.mark.parametrize("k", [3, 16, 64, 112, 128, 256, 500])
def test_spmm_normalized_gaussian(env, graphs, name, k):
    torch, cbm = env
    g = graphs[name]
    X = wl.gaussian_features(g.n, k, g.meta["seed"])
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=16)
    got = _run(env, "cbm_spmm_normalized", h, X, g.n)
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
    assert row_scaled_error(got, ref) <= TOL
    got_relu = _run(env, "cbm_spmm_normalized_relu", h, X, g.n)
    assert row_scaled_error(got_relu, np.maximum(ref, 0.0), scale_from=ref) <= TOL
    plain = _run(env, "cbm_spmm", h, X, g.n)  # (A v I) X on a self-loop handle
    ref_plain = orc.spmm_csr(g.rowptr, g.colidx, X) + X.astype(np.float64)
    assert row_scaled_error(plain, ref_plain) <= TOL


@pytest.mark.parametrize("opts", [dict(alpha=2), dict(alpha=16), dict(max_depth=1), dict(max_depth=3),
                                  dict(max_depth=-1), dict(hub_cap=4), dict(max_candidates=1),
                                  dict(hub_cap=-1, max_candidates=-1, max_depth=-1)])
def test_every_valid_tree_gives_the_same_product(env, graphs, opts):
    torch, cbm = env
    for name in ("tiny", "collaboration"):
        g = graphs[name]
        X = wl.integer_features(g.n, 32, 5)
        ref = orc.spmm_csr(g.rowptr, g.colidx, X)
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, **opts)
        assert np.array_equal(_run(env, "cbm_spmm", h, X, g.n).astype(np.float64), ref)
        Xg = wl.gaussian_features(g.n, 32, 5)
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, **opts)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, Xg, g.n),
                                orc.spmm_csr_normalized(g.rowptr, g.colidx, Xg)) <= TOL


def test_regular_graph_normalized_bit_exact(env):
    # degree 3 + self-loop: d = 4, d^-1/2 = 1/2 exactly, so the normalised product of integers is exact
    torch, cbm = env
    n = 4096
    edges = [(i, (i + 1) % n) for i in range(n)] + [(i, (i + n // 2) % n) for i in range(n // 2)]
    adj = [set() for _ in range(n)]
    for u, v in edges:
        adj[u].add(v)
        adj[v].add(u)
    rowptr, colidx = _csr(adj)
    X = wl.integer_features(n, 64, 3)
    h = cbm.cbm_build(n, n, rowptr, colidx, add_self_loops=True, max_depth=16)
    got = _run(env, "cbm_spmm_normalized", h, X, n)
    assert np.array_equal(got.astype(np.float64), orc.spmm_csr_normalized(rowptr, colidx, X))


def test_lower_triangular_chain_is_cumsum(env):
    torch, cbm = env
    m = 300
    rowptr, colidx = _csr([list(range(i + 1)) for i in range(m)])
    X = wl.integer_features(m, 8, 1)
    want = np.cumsum(X.astype(np.float64), axis=0)
    for depth in (-1, 0, 4):
        h = cbm.cbm_build(m, m, rowptr, colidx, max_depth=depth)
        s = cbm.cbm_stats(h)
        # 0 = automatic: cap 16, or every row in full when the cost model finds the tree does not pay
        assert s["depth"] in ((m,) if depth == -1 else (1, 16) if depth == 0 else (4,))
        assert np.array_equal(_run(env, "cbm_spmm", h, X, m).astype(np.float64), want)


def test_split_rows_and_empty_rows(env):
    torch, cbm = env
    rng = np.random.default_rng(0)
    n = 6000
    dense_row = sorted(rng.choice(n, size=3000, replace=False).tolist())
    near = sorted(set(dense_row[:2900]) | {5, 7})  # compresses against the split row
    rows = [dense_row, near, [], [1, 2, 3], sorted(rng.choice(n, size=1025, replace=False).tolist())] + [[]] * 3
    rows += [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(0, 40, size=n - len(rows))]
    rowptr, colidx = _csr(rows)
    for k in (4, 100, 256):
        X = wl.integer_features(n, k, 2)
        h = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16)
        s = cbm.cbm_stats(h)
        assert s["num_split_rows"] >= 2
        assert np.array_equal(_run(env, "cbm_spmm", h, X, n).astype(np.float64), orc.spmm_csr(rowptr, colidx, X))
        Xg = wl.gaussian_features(n, k, 2)
        h = cbm.cbm_build(n, n, rowptr, colidx, add_self_loops=True, max_depth=16)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, Xg, n),
                                orc.spmm_csr_normalized(rowptr, colidx, Xg)) <= TOL


def test_split_rows_with_popular_columns_clustered(env):
    """Long rows whose entries crowd into the low end of the column range (popular columns next to each other, as in a
    graph that was not renumbered): the per-XCD column ranges are cut by entry count, some of them only a few columns
    wide, others empty of a given row; products against the oracle, rows of 1,024 entries and more cut into phases too."""
    torch, cbm = env
    rng = np.random.default_rng(11)
    n = 16000
    p = 1.0 / (np.arange(n) + 20.0) ** 1.2
    p /= p.sum()
    rows = [sorted(rng.choice(n, size=int(s), replace=False, p=p).tolist()) for s in rng.integers(130, 1500, size=300)]
    rows += [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(0, 30, size=n - len(rows))]
    rowptr, colidx = _csr(rows)
    for k in (16, 128, 200):
        X = wl.integer_features(n, k, 3)
        h = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16)
        assert cbm.cbm_stats(h)["num_split_rows"] >= 250
        assert np.array_equal(_run(env, "cbm_spmm", h, X, n).astype(np.float64), orc.spmm_csr(rowptr, colidx, X))
        cbm.cbm_free(h)
        Xg = wl.gaussian_features(n, k, 3)
        h = cbm.cbm_build(n, n, rowptr, colidx, add_self_loops=True)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, Xg, n),
                                orc.spmm_csr_normalized(rowptr, colidx, Xg)) <= TOL
        cbm.cbm_free(h)


@pytest.mark.parametrize("name", wl.CONFIGS)
@pytest.mark.parametrize("k", [3, 64, 128, 500])
def test_mean_and_gin_aggregators(env, graphs, name, k):
    """The GraphSAGE mean and the GIN sum as epilogues of the same kernels: Gaussian features to 1e-5,
    GIN on integer features with an exactly representable 1 + eps bit for bit; both a deep tree
    (deferred finish of internal rows) and the handle built with self loops (M = A v I)."""
    torch, cbm = env
    g = graphs[name]
    X = wl.gaussian_features(g.n, k, g.meta["seed"])
    Xi = wl.integer_features(g.n, k, g.meta["seed"])
    Xd, Xid = torch.from_numpy(X).cuda(), torch.from_numpy(Xi).cuda()
    for opts in (dict(max_depth=16), dict(alpha=2), dict(max_depth=16, add_self_loops=True)):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, **opts)
        if opts.get("add_self_loops"):
            R = orc.adjacency_lists(g.n, g.rowptr, g.colidx, add_self_loops=True)[1:]
            rowptr, colidx = _csr(R)
        else:
            rowptr, colidx = g.rowptr, g.colidx
        got = _run(env, "cbm_spmm_mean", h, X, g.n)
        assert row_scaled_error(got, orc.spmm_csr_mean(rowptr, colidx, X)) <= TOL
        Y = torch.full((g.n, k), float("nan"), device="cuda")
        cbm.cbm_spmm_gin(h, 0.25, Xd, Y)
        ref = orc.spmm_csr_gin(rowptr, colidx, X, 0.25)
        assert row_scaled_error(Y.cpu().numpy(), ref) <= TOL
        cbm.cbm_spmm_gin(h, 1.0, Xid, Y.fill_(float("nan")))
        ref = orc.spmm_csr_gin(rowptr, colidx, Xi, 1.0)
        assert np.abs(ref).max() < 2 ** 24
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref)
        cbm.cbm_free(h)


def test_mean_and_gin_on_split_and_empty_rows(env):
    torch, cbm = env
    rng = np.random.default_rng(1)
    n = 5000
    dense_row = sorted(rng.choice(n, size=2048, replace=False).tolist())   # 2048 entries: 1/2048 is exact
    near = sorted(set(dense_row[:2000]) | {5, 7})
    rows = [dense_row, near, [], [1, 2, 3, 4]] + [[]] * 2
    rows += [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(0, 40, size=n - len(rows))]
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16)
    assert cbm.cbm_stats(h)["num_split_rows"] >= 1
    for k in (4, 100, 256):
        Xi = wl.integer_features(n, k, 3)
        got = _run(env, "cbm_spmm_mean", h, Xi, n).astype(np.float64)
        ref = orc.spmm_csr_mean(rowptr, colidx, Xi)
        assert np.array_equal(got[[0, 2, 3, 4, 5]], ref[[0, 2, 3, 4, 5]])      # power-of-two and empty rows: exact
        assert row_scaled_error(got, ref) <= TOL
        Y = torch.full((n, k), float("nan"), device="cuda")
        cbm.cbm_spmm_gin(h, -0.5, torch.from_numpy(2 * Xi).cuda(), Y)          # (1 + eps) * even integer: exact
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.spmm_csr_gin(rowptr, colidx, 2 * Xi, -0.5))
    # rectangular handle: the mean is defined, GIN is not
    m2, n2 = 300, 700
    rows = [sorted(rng.choice(n2, size=int(s), replace=False).tolist()) for s in rng.integers(0, 30, size=m2)]
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(m2, n2, rowptr, colidx, max_depth=16)
    Xg = wl.gaussian_features(n2, 24, 5)
    assert row_scaled_error(_run(env, "cbm_spmm_mean", h, Xg, m2), orc.spmm_csr_mean(rowptr, colidx, Xg)) <= TOL
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_spmm_gin(h, 0.0, torch.from_numpy(Xg).cuda(), torch.empty((m2, 24), device="cuda"))
    assert e.value.status == 6


def test_transposed_handle_is_the_adjoint(env):
    """A directed graph: the handle built with transpose=True computes A^T.G (and A_hat^T.G), the backward pass of
    the product.  Checked against the dense definition and through <Y, A X> = <A^T Y, X> on integers, exactly."""
    torch, cbm = env
    rng = np.random.default_rng(17)
    n, k = 900, 24
    rows = [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(0, 60, size=n)]
    rows[0] = sorted(rng.choice(n, size=700, replace=False).tolist())          # a split row, and a hub column below
    rows = [sorted(set(r) | ({5} if i % 3 else set())) for i, r in enumerate(rows)]
    rowptr, colidx = _csr(rows)
    A = orc.dense_from_csr(n, n, rowptr, colidx)
    h = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16)
    ht = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16, transpose=True)
    X, G = wl.integer_features(n, k, 1), wl.integer_features(n, k, 2)
    Y = _run(env, "cbm_spmm", h, X, n).astype(np.float64)
    Z = _run(env, "cbm_spmm", ht, G, n).astype(np.float64)
    assert np.array_equal(Z, A.T @ G.astype(np.float64))
    assert (Y * G).sum() == (Z * X).sum()                                       # the adjoint identity, in integers
    # normalised: D stays the row sums of A v I as given
    hn = cbm.cbm_build(n, n, rowptr, colidx, max_depth=16, add_self_loops=True, transpose=True)
    Gg = wl.gaussian_features(n, k, 3)
    ref = orc.normalized_dense(A).T @ Gg.astype(np.float64)
    assert row_scaled_error(_run(env, "cbm_spmm_normalized", hn, Gg, n), ref) <= TOL
    # rectangular: (m x n)^T is n x m
    m2, n2 = 300, 500
    rowptr, colidx = _csr([sorted(rng.choice(n2, size=int(s), replace=False).tolist()) for s in rng.integers(0, 40, size=m2)])
    hr = cbm.cbm_build(m2, n2, rowptr, colidx, max_depth=16, transpose=True)
    G2 = wl.integer_features(m2, 8, 4)
    got = _run(env, "cbm_spmm", hr, G2, n2).astype(np.float64)
    assert np.array_equal(got, orc.dense_from_csr(m2, n2, rowptr, colidx).T @ G2.astype(np.float64))


def test_launches_of_many_waves_use_the_small_batch_build(env):
    """A launch of 65,536 waves or more runs the build of the kernels with batches of 4 rows; the graphs of the other
    tests in this file stay below that.  R-MAT at scale 18 with k = 128 (two work items per wave, 262,144 rows) is
    above it for the row launch, and is still small enough to check every row against the oracle."""
    torch, cbm = env
    g = wl.make_graph("rmat", scale=18, edge_factor=16)
    k = 128
    for opts in (dict(), dict(max_depth=16, alpha=0)):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, **opts)
        s = cbm.cbm_stats(h)
        assert s["num_tasks"] // 2 >= 65536
        Xi = wl.integer_features(g.n, k, 9, lo=-2, hi=2)
        ref = orc.spmm_csr(g.rowptr, g.colidx, Xi)
        assert np.abs(ref).max() < 2 ** 24
        assert np.array_equal(_run(env, "cbm_spmm", h, Xi, g.n).astype(np.float64), ref)
        Xr = np.ascontiguousarray(Xi[:, :126])        # not a multiple of four columns: the ragged variant of the same build
        assert np.array_equal(_run(env, "cbm_spmm", h, Xr, g.n).astype(np.float64), ref[:, :126])
        cbm.cbm_free(h)
    hn = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=2)
    Xg = wl.gaussian_features(g.n, k, 9)
    assert row_scaled_error(_run(env, "cbm_spmm_normalized", hn, Xg, g.n), orc.spmm_csr_normalized(g.rowptr, g.colidx, Xg)) <= TOL
    assert row_scaled_error(_run(env, "cbm_spmm_mean", hn, Xg, g.n),
                            orc.spmm_csr_mean(*_csr(orc.adjacency_lists(g.n, g.rowptr, g.colidx, add_self_loops=True)[1:]), Xg)) <= TOL


def test_rounds_scheduled_by_graph_locality(env):
    """Rounds of long work items on a square matrix are handed out per XCD in breadth-first order of the graph; a
    nearest-neighbour graph with 100 neighbours has such rounds.  Every row against the oracle, and the launch records
    must show that the per-XCD path was taken (and is not taken when switched off by a rectangular matrix)."""
    torch, cbm = env
    g = wl.make_graph("protein", n=20000, knn=100)
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=2, max_depth=16)  # a tree, whatever it costs
    cbm.cbm_profile_enable(h, True)
    for k in (64, 256, 30):
        Xg = wl.gaussian_features(g.n, k, 4)
        got = _run(env, "cbm_spmm_normalized", h, Xg, g.n)
        recs = cbm.cbm_profile_read(h)
        assert any(r["kind"] == 0 and r["per_xcd"] == 1 for r in recs), recs
        assert row_scaled_error(got, orc.spmm_csr_normalized(g.rowptr, g.colidx, Xg)) <= TOL
    cbm.cbm_profile_enable(h, False)
    Xi = wl.integer_features(g.n, 16, 4, lo=-2, hi=2)
    hp = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=2, max_depth=16)
    assert np.array_equal(_run(env, "cbm_spmm", hp, Xi, g.n).astype(np.float64), orc.spmm_csr(g.rowptr, g.colidx, Xi))


def test_product_is_independent_of_the_builder_thread_count(env, graphs):
    """Same work lists whatever the number of host threads that built them: same rounding, bit for bit."""
    torch, cbm = env
    for name in ("collaboration", "rmat"):
        g = graphs[name]
        X = torch.from_numpy(wl.gaussian_features(g.n, 48, 6)).cuda()
        ys = []
        for nt in (1, 3, 0):
            h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=1, max_depth=16, num_threads=nt)
            Y = torch.empty_like(X)
            cbm.cbm_spmm_normalized(h, X, Y)
            torch.cuda.synchronize()
            ys.append(Y)
            cbm.cbm_free(h)
        assert torch.equal(ys[0], ys[1]) and torch.equal(ys[0], ys[2])


@pytest.mark.parametrize("k", [1000, 4096, 4099])
def test_very_wide_features(env, k):
    """Many column chunks per work item, aligned and ragged."""
    torch, cbm = env
    g = wl.tiny_graph()
    X = wl.gaussian_features(g.n, k, 1)
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
    for opts in (dict(max_depth=16), dict()):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, **opts)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, X, g.n), ref) <= TOL
        cbm.cbm_free(h)


def test_degenerate_shapes(env):
    torch, cbm = env
    # empty matrix
    h = cbm.cbm_build(0, 5, np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), max_depth=16)
    X = torch.ones((5, 4), device="cuda")
    Y = torch.empty((0, 4), device="cuda")
    cbm.cbm_spmm(h, X, Y)
    # all rows empty: Y must be written with zeros
    rowptr, colidx = _csr([[]] * 7)
    h = cbm.cbm_build(7, 5, rowptr, colidx, max_depth=16)
    got = _run(env, "cbm_spmm", h, np.ones((5, 4), dtype=np.float32), 7)
    assert np.array_equal(got, np.zeros((7, 4), dtype=np.float32))
    # rectangular, k = 1 (the matrix-vector product of Eq. (6)), single row
    rng = np.random.default_rng(1)
    rows = [sorted(np.flatnonzero(rng.random(37) < 0.3).tolist()) for _ in range(90)]
    rowptr, colidx = _csr(rows)
    X = wl.integer_features(37, 1, 0)
    h = cbm.cbm_build(90, 37, rowptr, colidx, max_depth=16)
    assert np.array_equal(_run(env, "cbm_spmm", h, X, 90).astype(np.float64), orc.spmm_csr(rowptr, colidx, X))
    rowptr, colidx = _csr([[0, 2]])
    h = cbm.cbm_build(1, 3, rowptr, colidx, max_depth=16)
    X = np.array([[1, 2], [3, 4], [5, 6]], dtype=np.float32)
    assert np.array_equal(_run(env, "cbm_spmm", h, X, 1), np.array([[6, 8]], dtype=np.float32))
    # isolated node in the normalised product: A v I row is {x}, d = 1, output = input row
    rowptr, colidx = _csr([[1], [0], []])
    h = cbm.cbm_build(3, 3, rowptr, colidx, add_self_loops=True, max_depth=16)
    X = np.array([[2.0, 4.0], [6.0, 8.0], [3.0, 5.0]], dtype=np.float32)
    got = _run(env, "cbm_spmm_normalized", h, X, 3)
    np.testing.assert_allclose(got, [[4.0, 6.0], [4.0, 6.0], [3.0, 5.0]], rtol=1e-6)


def test_strided_and_misaligned_operands(env, graphs):
    torch, cbm = env
    g = graphs["collaboration"]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=16)
    k = 48
    X = wl.integer_features(g.n, k, 9)
    ref = orc.spmm_csr(g.rowptr, g.colidx, X)
    # leading dimensions larger than k (a column slice of a wider tensor)
    Xw = torch.zeros((g.n, 80), device="cuda")
    Xw[:, 8:8 + k] = torch.from_numpy(X).cuda()
    Yw = torch.full((g.n, 64), float("nan"), device="cuda")
    cbm.cbm_spmm(h, Xw[:, 8:8 + k], Yw[:, 4:4 + k])
    torch.cuda.synchronize()
    assert np.array_equal(Yw[:, 4:4 + k].cpu().numpy().astype(np.float64), ref)
    assert bool(torch.isnan(Yw[:, :4]).all()) and bool(torch.isnan(Yw[:, 4 + k:]).all())  # nothing else touched
    # pointers that are only 4-byte / 8-byte aligned select the narrower-load variants
    for off in (1, 2):
        cbm.cbm_spmm(h, Xw[:, off:off + k], Yw[:, off:off + k])
        torch.cuda.synchronize()
        want = orc.spmm_csr(g.rowptr, g.colidx, Xw[:, off:off + k].cpu().numpy())
        assert np.array_equal(Yw[:, off:off + k].cpu().numpy().astype(np.float64), want)


def test_argument_errors_on_device_handle(env, graphs):
    torch, cbm = env
    g = graphs["tiny"]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=16)  # no self-loops
    X = torch.zeros((g.n, 8), device="cuda")
    Y = torch.zeros((g.n, 8), device="cuda")
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_spmm_normalized(h, X, Y)
    assert e.value.status == 6
    with pytest.raises(cbm.CbmError) as e:  # the output may not overlap the input
        cbm.cbm_spmm(h, X, X)
    assert e.value.status == 1
    W = torch.zeros((g.n, 16), device="cuda")
    with pytest.raises(cbm.CbmError) as e:  # not even as interleaved column slices of one buffer
        cbm.cbm_spmm(h, W[:, :8], W[:, 8:])
    assert e.value.status == 1


@pytest.mark.parametrize("name", ["tiny", "collaboration", "protein", "rmat"])
@pytest.mark.parametrize("blocks", [2, 8])
def test_column_blocked_handle_gives_the_same_products(env, graphs, name, blocks):
    """Column-blocked CBM: every product of the boundary against the oracle, as for the plain format."""
    torch, cbm = env
    g = graphs[name]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=1, max_depth=16, column_blocks=blocks)
    s = cbm.cbm_stats(h)
    assert s["column_blocks"] == blocks
    Xi = wl.integer_features(g.n, 16, g.meta["seed"])
    got = _run(env, "cbm_spmm", h, Xi, g.n)
    ref = orc.spmm_csr(g.rowptr, g.colidx, Xi) + Xi.astype(np.float64)          # the handle holds A v I
    assert np.array_equal(got.astype(np.float64), ref)
    d = np.diff(g.rowptr) + 1
    for k in (3, 64, 128):
        X = wl.gaussian_features(g.n, k, g.meta["seed"])
        ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, X, g.n), ref) <= TOL
        assert row_scaled_error(_run(env, "cbm_spmm_normalized_relu", h, X, g.n), np.maximum(ref, 0.0), scale_from=ref) <= TOL
        mean = (orc.spmm_csr(g.rowptr, g.colidx, X) + X.astype(np.float64)) / d[:, None]
        assert row_scaled_error(_run(env, "cbm_spmm_mean", h, X, g.n), mean) <= TOL
        Xd = torch.from_numpy(X).cuda()
        Y = torch.full((g.n, k), float("nan"), device="cuda")
        cbm.cbm_spmm_gin(h, 0.25, Xd, Y)
        torch.cuda.synchronize()
        gin = orc.spmm_csr(g.rowptr, g.colidx, X) + 2.25 * X.astype(np.float64)   # (A v I) X + 1.25 X
        scale = orc.spmm_csr(g.rowptr, g.colidx, np.abs(X)) + 2.25 * np.abs(X).astype(np.float64)
        assert np.all(np.abs(Y.cpu().numpy() - gin) <= 1e-5 * scale)
    # the GCN driver and the per-launch records go through the same handle
    f_in, hidden, f_out = 32, 16, 8
    X = wl.gaussian_features(g.n, f_in, 3)
    W0, W1 = wl.glorot_uniform(f_in, hidden, 1), wl.glorot_uniform(hidden, f_out, 2)
    out = torch.full((g.n, f_out), float("nan"), device="cuda")
    ws = torch.empty(cbm.cbm_gcn2_workspace_bytes(h, f_in, hidden, f_out), dtype=torch.uint8, device="cuda")
    cbm.cbm_gcn2_forward(h, *(torch.from_numpy(a).cuda() for a in (X, W0, W1)), out, ws)
    torch.cuda.synchronize()
    assert row_scaled_error(out.cpu().numpy(), orc.gcn2(g.rowptr, g.colidx, X, W0, W1)) <= TOL
    cbm.cbm_profile_enable(h, True)
    _run(env, "cbm_spmm_normalized", h, wl.gaussian_features(g.n, 8, 1), g.n)
    recs = cbm.cbm_profile_read(h)
    cbm.cbm_profile_enable(h, False)
    assert recs[-1]["kind"] == 4 and all(r["milliseconds"] > 0 for r in recs)
    with pytest.raises(cbm.CbmError) as e:   # the static scratch is not for B partial rows per row
        cbm.cbm_spmm_noalloc(h, torch.zeros((g.n, 8), device="cuda"), torch.zeros((g.n, 8), device="cuda"))
    assert e.value.status == 5


@pytest.mark.parametrize("name", ["collaboration", "protein", "citation"])
def test_bundled_rounds_give_the_same_products(env, graphs, name, monkeypatch):
    """Rounds of long multi-row paths are gathered in one sweep per path (one partial sum per row of the path): every
    product against the oracle with bundling forced onto the reduced graphs, whose work items are too short for it
    otherwise; aligned and ragged widths, strided operands, a depth that leaves rows for the deferred finish."""
    torch, cbm = env
    g = graphs[name]
    monkeypatch.setenv("CBM_BUNDLE_MIN", "1")
    monkeypatch.setenv("CBM_BUNDLE_MIN_ITEMS", "1")
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=1, max_depth=16)
    hp = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=0, max_depth=16)   # (an unbounded tree would give the row limit up)
    monkeypatch.delenv("CBM_BUNDLE_MIN")
    monkeypatch.delenv("CBM_BUNDLE_MIN_ITEMS")
    s = cbm.cbm_stats(h)
    assert s["bundled_rounds"] >= 1 and cbm.cbm_stats(hp)["bundled_rounds"] >= 1 and s["num_internal"] > 0
    Xi = wl.integer_features(g.n, 16, g.meta["seed"])
    assert np.array_equal(_run(env, "cbm_spmm", hp, Xi, g.n).astype(np.float64), orc.spmm_csr(g.rowptr, g.colidx, Xi))
    d = np.diff(g.rowptr) + 1
    for k in (3, 64, 112, 130, 256):
        X = wl.gaussian_features(g.n, k, g.meta["seed"])
        ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
        assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, X, g.n), ref) <= TOL
        if k <= 64:   # narrow X shares a work item among four groups of a wave; the one-group form of the same kernel too
            monkeypatch.setenv("CBM_WIDE_MAX_WAVES", "0")
            assert row_scaled_error(_run(env, "cbm_spmm_normalized", h, X, g.n), ref) <= TOL
            assert np.array_equal(_run(env, "cbm_spmm", hp, Xi, g.n).astype(np.float64), orc.spmm_csr(g.rowptr, g.colidx, Xi))
            monkeypatch.delenv("CBM_WIDE_MAX_WAVES")
        assert row_scaled_error(_run(env, "cbm_spmm_normalized_relu", h, X, g.n), np.maximum(ref, 0.0), scale_from=ref) <= TOL
        mean = (orc.spmm_csr(g.rowptr, g.colidx, X) + X.astype(np.float64)) / d[:, None]
        assert row_scaled_error(_run(env, "cbm_spmm_mean", h, X, g.n), mean) <= TOL
        Xd = torch.from_numpy(X).cuda()
        Y = torch.full((g.n, k), float("nan"), device="cuda")
        cbm.cbm_spmm_gin(hp, 0.25, Xd, Y)
        torch.cuda.synchronize()
        gin = orc.spmm_csr(g.rowptr, g.colidx, X) + 1.25 * X.astype(np.float64)
        scale = orc.spmm_csr(g.rowptr, g.colidx, np.abs(X)) + 1.25 * np.abs(X).astype(np.float64)
        assert np.all(np.abs(Y.cpu().numpy() - gin) <= 1e-5 * scale)
    # strided operands: column slices of wider buffers
    Xw = torch.from_numpy(wl.gaussian_features(g.n, 96, 3)).cuda()
    Yw = torch.full((g.n, 80), float("nan"), device="cuda")
    cbm.cbm_spmm_normalized(h, Xw[:, 8:72], Yw[:, 4:68])
    torch.cuda.synchronize()
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, Xw[:, 8:72].cpu().numpy())
    assert row_scaled_error(Yw[:, 4:68].cpu().numpy(), ref) <= TOL
    # the same tree without bundling gives the same integer result bit for bit, and the bundled product is repeatable
    Y1 = _run(env, "cbm_spmm_normalized", h, wl.gaussian_features(g.n, 64, 9), g.n)
    Y2 = _run(env, "cbm_spmm_normalized", h, wl.gaussian_features(g.n, 64, 9), g.n)
    assert np.array_equal(Y1, Y2)


@pytest.mark.parametrize("name", ["protein", "collaboration"])
def test_order_inside_xcd_shares_does_not_change_the_product(env, graphs, name, monkeypatch):
    """Rounds scheduled by locality hand every XCD a share of the work items; the order inside a share (breadth-first,
    longest first, by length in buckets) is a scheduling choice: every row is still summed in the same order, so the
    products are the same bit for bit, and equal to the oracle's."""
    torch, cbm = env
    g = graphs[name]
    X = wl.gaussian_features(g.n, 128, g.meta["seed"])
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X)
    outs = []
    for mode in ("0", "1", "7", None):
        if mode is None:
            monkeypatch.delenv("CBM_SHARE_SORT", raising=False)
        else:
            monkeypatch.setenv("CBM_SHARE_SORT", mode)
        monkeypatch.setenv("CBM_LOCALITY_MIN", "1")     # every round of the reduced graphs goes by locality
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=1, max_depth=16)
        monkeypatch.delenv("CBM_LOCALITY_MIN")
        outs.append(_run(env, "cbm_spmm_normalized", h, X, g.n))
        assert row_scaled_error(outs[-1], ref) <= TOL
        cbm.cbm_free(h)
    assert all(np.array_equal(outs[0], o) for o in outs[1:])


def test_reserve_sizes_the_split_row_scratch_before_capture(env):
    # cbm_reserve instead of a first eager product: a handle WITH split rows is captured at once, and the replay is exact
    torch, cbm = env
    rng = np.random.default_rng(5)
    n = 3000
    rows = [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(0, 700, size=400)]
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(len(rows), n, rowptr, colidx, max_depth=16)
    assert cbm.cbm_stats(h)["num_split_rows"] > 0
    X = wl.integer_features(n, 48, 3)
    Xd = torch.from_numpy(X).cuda()
    Y = torch.full((len(rows), 48), float("nan"), device="cuda")
    cbm.cbm_reserve(h, 48)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cbm.cbm_spmm(h, Xd, Y)
    graph.replay()
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.spmm_csr(rowptr, colidx, X))
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_reserve(h, 0)
    assert e.value.status == 1


def test_gcn2_rejects_overlapping_buffers(env, graphs):
    torch, cbm = env
    g = graphs["tiny"]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=16)
    f_in, hidden, f_out = 8, 8, 8
    nb = cbm.cbm_gcn2_workspace_bytes(h, f_in, hidden, f_out)
    ws = torch.zeros(nb + g.n * f_out * 4, dtype=torch.uint8, device="cuda")
    X = torch.zeros((g.n, f_in), device="cuda")
    W0 = torch.zeros((f_in, hidden), device="cuda")
    W1 = torch.zeros((hidden, f_out), device="cuda")
    out = torch.zeros((g.n, f_out), device="cuda")
    inside = ws[:g.n * f_out * 4].view(torch.float32).view(g.n, f_out)   # lies inside the workspace
    for args in ((X, W0, W1, inside, ws), (inside, W0, W1, out, ws), (X, W0, W1, X, ws[:nb])):
        with pytest.raises(cbm.CbmError) as e:
            cbm.cbm_gcn2_forward(h, *args)
        assert e.value.status == 1
    cbm.cbm_gcn2_forward(h, X, W0, W1, out, ws[:nb])
    torch.cuda.synchronize()


@pytest.mark.parametrize("M,N,K", [(1000, 64, 500), (777, 3, 64), (513, 112, 256), (256, 256, 256), (130, 33, 7),
                                   (1, 1, 1), (300, 200, 37),
                                   # widths served by the 16-column tiles (N mod 32 in 1..16 above 32), ragged M and K too
                                   (2000, 112, 256), (1029, 100, 61), (515, 48, 128), (640, 40, 36), (300, 80, 500),
                                   (129, 65, 33), (4100, 97, 5),
                                   # as many rows as fill the chip evenly with blocks of 128 rows (fewer rows run in blocks of 64)
                                   (32768, 112, 40), (32700, 48, 36), (32768, 80, 33),
                                   # tall enough for the panel-resident kernel: one and two panels, ragged rows, K not a
                                   # multiple of 64, widths that are not a multiple of 16, leftover groups cut into tiles
                                   (70001, 112, 256), (65536, 256, 256), (9000, 64, 500), (20011, 200, 100), (8192, 16, 4),
                                   (33333, 132, 68), (12345, 20, 260), (66000, 128, 64),
                                   # leftover groups cut into chunks of two and of four tiles (with a last chunk that
                                   # overlaps its neighbour at seven tiles), three panels one after the other
                                   (78336, 128, 64), (78341, 128, 128), (91136, 128, 64), (78341, 112, 128), (91136, 112, 64),
                                   (9000, 300, 64)])
def test_dense_matmul(env, M, N, K):
    torch, cbm = env
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    Cd = torch.full((M, N), float("nan"), device="cuda")
    cbm.cbm_dense_matmul(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), Cd)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    # bound from the arithmetic: K products summed in fp32, |error| <= ~K * 2^-24 * sum|a||b|
    bound = 2.0 * K * 2.0 ** -24 * (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64))
    assert np.all(np.abs(Cd.cpu().numpy() - ref) <= bound + 1e-30)
    Ai = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
    Bi = rng.integers(-4, 5, size=(K, N)).astype(np.float32)
    cbm.cbm_dense_matmul(torch.from_numpy(Ai).cuda(), torch.from_numpy(Bi).cuda(), Cd)
    torch.cuda.synchronize()
    assert np.array_equal(Cd.cpu().numpy().astype(np.float64), Ai.astype(np.float64) @ Bi.astype(np.float64))


@pytest.mark.parametrize("M,N,K,pad_a,pad_b,pad_c,off", [(40000, 112, 256, 8, 16, 4, 4),    # panel kernel, strided, aligned
                                                          (40000, 256, 128, 4, 0, 12, 8),    # two panels side by side
                                                          (40000, 112, 256, 8, 16, 4, 1),    # slices off the 16-byte grid
                                                          (40000, 96, 64, 3, 5, 1, 0)])      # odd strides: staged kernels
def test_dense_matmul_strided_operands(env, M, N, K, pad_a, pad_b, pad_c, off):
    """A, B and C as column slices of wider buffers (leading dimensions larger than the widths), output rows poisoned:
    nothing outside C's columns may be written."""
    torch, cbm = env
    rng = np.random.default_rng(M + N + K + off)
    Aw = rng.standard_normal((M, K + pad_a + off)).astype(np.float32)
    Bw = rng.standard_normal((K, N + pad_b + off)).astype(np.float32)
    Ad, Bd = torch.from_numpy(Aw).cuda(), torch.from_numpy(Bw).cuda()
    Cw = torch.full((M, N + pad_c + off), float("nan"), device="cuda")
    A, B, C = Ad[:, off:off + K], Bd[:, off:off + N], Cw[:, off:off + N]
    cbm.cbm_dense_matmul(A, B, C)
    torch.cuda.synchronize()
    a64, b64 = Aw[:, off:off + K].astype(np.float64), Bw[:, off:off + N].astype(np.float64)
    bound = 2.0 * K * 2.0 ** -24 * (np.abs(a64) @ np.abs(b64))
    got = Cw.cpu().numpy()
    assert np.all(np.abs(got[:, off:off + N] - a64 @ b64) <= bound + 1e-30)
    outside = np.ones(got.shape[1], dtype=bool)
    outside[off:off + N] = False
    assert np.isnan(got[:, outside]).all()


@pytest.mark.parametrize("name,f_in,hidden,f_out", [("citation", 500, 64, 3), ("protein", 256, 256, 112),
                                                    ("tiny", 16, 8, 4)])
def test_gcn2_forward(env, graphs, name, f_in, hidden, f_out):
    torch, cbm = env
    g = graphs[name]
    seed = g.meta["seed"]
    X = wl.gaussian_features(g.n, f_in, seed)
    W0 = wl.glorot_uniform(f_in, hidden, seed)
    W1 = wl.glorot_uniform(hidden, f_out, seed)
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=16)
    ws = torch.empty(cbm.cbm_gcn2_workspace_bytes(h, f_in, hidden, f_out), dtype=torch.uint8, device="cuda")
    out = torch.full((g.n, f_out), float("nan"), device="cuda")
    cbm.cbm_gcn2_forward(h, *(torch.from_numpy(a).cuda() for a in (X, W0, W1)), out, ws)
    torch.cuda.synchronize()
    ref = orc.gcn2(g.rowptr, g.colidx, X, W0, W1)
    assert row_scaled_error(out.cpu().numpy(), ref) <= TOL


def test_iterated_products_ping_pong(env, graphs):
    # X_{t+1} = A X_t, ten times; each iterate is checked against the oracle fed the GPU's previous iterate
    torch, cbm = env
    g = graphs["collaboration"]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=1, max_depth=16)
    cur = torch.from_numpy(wl.gaussian_features(g.n, 32, 4)).cuda()
    nxt = torch.empty_like(cur)
    for _ in range(10):
        prev = cur.cpu().numpy()
        cbm.cbm_spmm(h, cur, nxt)
        torch.cuda.synchronize()
        assert row_scaled_error(nxt.cpu().numpy(), orc.spmm_csr(g.rowptr, g.colidx, prev)) <= TOL
        scale = float(nxt.abs().max())
        cur, nxt = nxt / scale, cur  # keep magnitudes bounded; the division is not part of the check


def test_profile_records(env, graphs):
    torch, cbm = env
    g = graphs["protein"]
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=16)
    s = cbm.cbm_stats(h)
    cbm.cbm_profile_enable(h, True)
    X = torch.from_numpy(wl.gaussian_features(g.n, 64, 1)).cuda()
    Y = torch.empty_like(X)
    cbm.cbm_spmm_normalized(h, X, Y)
    torch.cuda.synchronize()
    recs = cbm.cbm_profile_read(h)
    levels = [r for r in recs if r["kind"] == 0]
    assert len(levels) == s["rounds"] <= s["depth"]
    assert sum(r["deltas"] for r in levels) == s["num_delta_plus"] + s["num_delta_minus"]
    assert all(r["milliseconds"] > 0 for r in recs)


def test_products_can_be_captured_in_a_hip_graph(env, graphs):
    # the product calls only enqueue kernels (after the first call has sized the scratch), so a caller may
    # capture them; every replay is checked against the eager result, with eager work between replays
    torch, cbm = env
    g = graphs["collaboration"]
    k, hidden, f_out = 32, 16, 4
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=16)
    W0 = torch.from_numpy(wl.glorot_uniform(k, hidden, 1)).cuda()
    W1 = torch.from_numpy(wl.glorot_uniform(hidden, f_out, 2)).cuda()
    ws = torch.empty(cbm.cbm_gcn2_workspace_bytes(h, k, hidden, f_out), dtype=torch.uint8, device="cuda")
    X = torch.from_numpy(wl.gaussian_features(g.n, k, 1)).cuda()
    Y = torch.empty((g.n, k), device="cuda")
    out = torch.empty((g.n, f_out), device="cuda")
    cbm.cbm_spmm_normalized(h, X, Y)          # first calls outside the capture: scratch is sized here
    cbm.cbm_gcn2_forward(h, X, W0, W1, out, ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cbm.cbm_spmm_normalized(h, X, Y)
        cbm.cbm_gcn2_forward(h, X, W0, W1, out, ws)
    for it in range(4):
        X.copy_(torch.from_numpy(wl.gaussian_features(g.n, k, 10 + it)).cuda())
        Y.fill_(float("nan"))
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got_y, got_out = Y.clone(), out.clone()
        Y2 = torch.empty_like(Y)
        out2 = torch.empty_like(out)
        cbm.cbm_spmm_normalized(h, X, Y2)     # eager, between replays
        cbm.cbm_gcn2_forward(h, X, W0, W1, out2, ws)
        torch.cuda.synchronize()
        assert torch.equal(got_y, Y2) and torch.equal(got_out, out2)
    ref = orc.spmm_csr_normalized(g.rowptr, g.colidx, X.cpu().numpy())
    assert row_scaled_error(got_y.cpu().numpy(), ref) <= TOL
