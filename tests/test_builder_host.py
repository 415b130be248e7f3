"""Host logic of libcbm (no GPU): the library loads and exports the declared
symbols, the builder's tree/deltas satisfy the paper's invariants and, in exact
mode, reach the oracle's optimal tree weight; error paths return status codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2409_02208_amd as cbm
import workloads as wl
from oracle import cbm_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _csr(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in sorted(r)], dtype=np.int32)
    return rowptr, colidx


def _random_rows(rng, m, n, density):
    return [sorted(np.flatnonzero(rng.random(n) < density).tolist()) for _ in range(m)]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "cbm.h")).read()
    declared = set(re.findall(r"\b(cbm_[a-z0-9_]+)\s*\(", header))
    declared -= {"cbm_launch_record"}
    assert declared == set(cbm.EXPORTS), declared ^ set(cbm.EXPORTS)
    lib = ctypes.CDLL(cbm.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert cbm.cbm_status_string(0) == "ok"
    assert "CSR" in cbm.cbm_status_string(2)


def _check_invariants(m, n, rowptr, colidx, h, alpha, self_loops):
    s = cbm.cbm_stats(h)
    t = cbm.cbm_get_tree(h)
    rp, ci = cbm.cbm_decompress(h)
    rows = orc.adjacency_lists(m, rowptr, colidx, add_self_loops=self_loops)
    want_rp, want_ci = _csr([sorted(r) for r in rows[1:]])
    assert np.array_equal(rp, want_rp) and np.array_equal(ci, want_ci)           # Eq. (2) round trip
    nnz = int(want_rp[-1])
    assert s["nnz"] == nnz
    assert s["num_delta_plus"] == t["nplus"].sum() and s["num_delta_minus"] == t["nminus"].sum()
    assert s["num_delta_plus"] + s["num_delta_minus"] <= nnz                     # Property 1
    assert s["scalar_ops"] <= nnz                                                # Property 2
    parent, level = t["parent"], t["level"]
    assert s["num_roots"] == int((parent < 0).sum())
    for x in range(m):
        y = int(parent[x])
        nx = len(rows[x + 1])
        if y < 0:
            assert level[x] == 1 and t["nplus"][x] == nx and t["nminus"][x] == 0
            continue
        assert level[x] == level[y] + 1                                          # acyclic, reaches vertex 0
        w = len(rows[x + 1] ^ rows[y + 1])
        assert t["nplus"][x] + t["nminus"][x] == w
        assert w <= nx - max(alpha, 1)                                           # alpha rule; draws -> virtual
        assert 1 + w <= nx                                                       # Property 2, per row
    assert s["depth"] == (int(level.max()) if m else 0)
    assert (1 if m else 0) <= s["rounds"] <= max(s["depth"], 0)
    return s


@pytest.mark.parametrize("alpha", [0, 1, 3])
@pytest.mark.parametrize("self_loops", [False, True])
def test_invariants_random(alpha, self_loops):
    rng = np.random.default_rng(alpha * 2 + self_loops)
    m = n = 60
    rows = _random_rows(rng, m, n, 0.2)
    rows[4] = []
    rows[11] = list(rows[10])
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(m, n, rowptr, colidx, alpha=alpha, add_self_loops=self_loops, host_only=True, max_depth=16)
    _check_invariants(m, n, rowptr, colidx, h, alpha, self_loops)
    cbm.cbm_free(h)


@pytest.mark.parametrize("seed", range(5))
def test_exact_mode_reaches_the_minimum_spanning_tree_weight(seed):
    # hub_cap = max_candidates = max_depth = unlimited, alpha = 0: Prim on all useful edges
    rng = np.random.default_rng(40 + seed)
    m, n = 40, 30
    rows = _random_rows(rng, m, n, 0.35)
    rows[7] = list(rows[6])
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(m, n, rowptr, colidx, max_depth=-1, hub_cap=-1, max_candidates=-1, host_only=True)
    s = _check_invariants(m, n, rowptr, colidx, h, 0, False)
    R = orc.adjacency_lists(m, rowptr, colidx)
    W = orc.hamming_distance_graph(R)
    r = orc.mst_rooted_at_virtual(W)
    assert s["num_delta_plus"] + s["num_delta_minus"] == sum(int(W[r[x], x]) for x in range(1, m + 1))


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("alpha", [0, 1, 2, 4])
def test_exact_tree_is_a_minimum_cost_arborescence(seed, alpha):
    # CBM_FLAG_EXACT_TREE on the complete candidate graph: same total weight as the oracle's Chu-Liu/Edmonds
    rng = np.random.default_rng(900 + seed)
    m, n = 45, 24
    rows = _random_rows(rng, m, n, 0.4)
    rows[7] = list(rows[6])
    rows[20] = []
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(m, n, rowptr, colidx, alpha=alpha, hub_cap=-1, max_candidates=-1, exact_tree=True, host_only=True)
    s = _check_invariants(m, n, rowptr, colidx, h, alpha, False)
    R = orc.adjacency_lists(m, rowptr, colidx)
    W = orc.hamming_distance_graph(R)
    r = orc.mca_rooted_at_virtual(W, orc.admissible_edges(W, max(alpha, 1)))  # draws go to the virtual edge: strict gain
    want = sum(int(W[r[x], x]) for x in range(1, m + 1))
    assert s["num_delta_plus"] + s["num_delta_minus"] == want


def test_exact_tree_on_a_reduced_workload():
    g = wl.collaboration_graph(n=6000)
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=2, exact_tree=True, host_only=True)
    s = cbm.cbm_stats(h)
    hp = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=2, max_depth=-1, seed_roots=-1, host_only=True)
    sp = cbm.cbm_stats(hp)
    # same candidate edges: the arborescence can only be lighter than the Prim-grown tree
    assert s["num_delta_plus"] + s["num_delta_minus"] <= sp["num_delta_plus"] + sp["num_delta_minus"]
    rp, ci = cbm.cbm_decompress(h)
    rp2, ci2 = cbm.cbm_decompress(hp)
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)
    t = cbm.cbm_get_tree(h)
    comp = t["parent"] >= 0
    assert np.all(t["level"][comp] == t["level"][t["parent"][comp]] + 1) and np.all(t["level"] >= 1)


def test_depth_cap_and_pruning_options():
    g = wl.tiny_graph()
    full = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=-1, seed_roots=-1, host_only=True))
    for cap in (1, 2, 5):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=cap, seed_roots=-1, host_only=True)
        s = _check_invariants(g.n, g.n, g.rowptr, g.colidx, h, 0, False)
        assert s["depth"] <= cap
        assert s["num_delta_plus"] + s["num_delta_minus"] >= full["num_delta_plus"] + full["num_delta_minus"]
    s1 = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=1, host_only=True))
    assert s1["num_roots"] == g.n and s1["num_delta_plus"] == g.nnz and s1["num_delta_minus"] == 0  # plain CSR
    s2 = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=10 ** 6, host_only=True, max_depth=16))
    assert s2["num_roots"] == g.n and s2["depth"] == 1


def test_automatic_depth_uses_the_cost_model():
    # default options: a tree only where it pays for its extra dependent launches
    g = wl.tiny_graph()
    s = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, host_only=True))
    assert s["depth"] == 1 and s["rounds"] == 1 and s["num_roots"] == g.n      # launch-bound: plain CSR
    forced = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, max_depth=16, host_only=True))
    assert forced["depth"] > 1 and forced["num_delta_plus"] + forced["num_delta_minus"] < s["num_delta_plus"]
    g = wl.collaboration_graph(n=40000)
    s = cbm.cbm_stats(cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, host_only=True))
    assert s["depth"] > 1 and s["scalar_ops"] < 0.7 * s["nnz"]                  # bandwidth-bound: the tree pays


def test_seeded_roots():
    g = wl.protein_graph(n=3000, knn=40)
    for seeds in (-1, 0, 200):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, max_depth=8, seed_roots=seeds, host_only=True)
        s = _check_invariants(g.n, g.n, g.rowptr, g.colidx, h, 0, True)
        if seeds > 0:
            t = cbm.cbm_get_tree(h)
            assert s["num_roots"] >= seeds and all(t["parent"][i * g.n // seeds] < 0 for i in range(seeds))


def test_special_shapes():
    # lower-triangular: the chain; depth capped by default, exact when unlimited
    m = 50
    rowptr, colidx = _csr([list(range(i + 1)) for i in range(m)])
    h = cbm.cbm_build(m, m, rowptr, colidx, max_depth=-1, host_only=True)
    s = _check_invariants(m, m, rowptr, colidx, h, 0, False)
    assert s["num_delta_plus"] == m and s["num_delta_minus"] == 0 and s["depth"] == m
    assert s["rounds"] == 1 and s["num_tasks"] == 1  # the whole chain is one path: one work item, one launch
    # identical rows: one stored in full, the others cost one op each
    row = [1, 4, 5, 7]
    rowptr, colidx = _csr([row] * 9)
    s = cbm.cbm_stats(cbm.cbm_build(9, 8, rowptr, colidx, host_only=True, max_depth=16))
    assert s["num_delta_plus"] == 4 and s["num_delta_minus"] == 0 and s["scalar_ops"] == 4 + 8
    # empty matrix, empty rows, single row, rectangular
    for rows, n in ([], 5), ([[]] * 3, 4), ([[0, 2]], 3), ([[0, 1, 2, 3, 4, 5, 6], [0, 1, 2, 3, 4, 5]], 7):
        rowptr, colidx = _csr(rows)
        h = cbm.cbm_build(len(rows), n, rowptr, colidx, host_only=True, max_depth=16)
        _check_invariants(len(rows), n, rowptr, colidx, h, 0, False)


def test_long_rows_are_split_into_segments():
    rng = np.random.default_rng(0)
    n = 5000
    for size, pieces in ((900, 8), (1800, 32)):  # one piece per XCD column range; 4 sub-ranges each from 1024 entries
        rows = [sorted(rng.choice(n, size=size, replace=False).tolist()), [1, 2, 3], []]
        rowptr, colidx = _csr(rows)
        h = cbm.cbm_build(3, n, rowptr, colidx, host_only=True, max_depth=16)
        s = _check_invariants(3, n, rowptr, colidx, h, 0, False)
        assert s["num_split_rows"] == 1 and s["num_tasks"] == 2 + pieces


def test_error_paths_return_status_codes():
    rowptr, colidx = _csr([[0, 1], [1]])
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(2, 2, np.array([0, 2, 1], dtype=np.int64), colidx, host_only=True, max_depth=16)
    assert e.value.status == 2
    for bad in ([1, 0, 1], [0, 0, 1], [0, 5, 1], [-1, 1, 1]):
        with pytest.raises(cbm.CbmError) as e:
            cbm.cbm_build(2, 2, rowptr, np.array(bad, dtype=np.int32), host_only=True, max_depth=16)
        assert e.value.status == 2
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(2, 2, rowptr, colidx, alpha=-1, host_only=True, max_depth=16)
    assert e.value.status == 1
    with pytest.raises(cbm.CbmError) as e:  # self-loops need a square matrix
        cbm.cbm_build(2, 3, rowptr, colidx, add_self_loops=True, host_only=True, max_depth=16)
    assert e.value.status == 1
    lib = ctypes.CDLL(cbm.LIB_PATH)
    assert lib.cbm_build(ctypes.c_int64(2), ctypes.c_int64(2), None, None, None, None) == 1
    lib.cbm_free(None)  # NULL-safe
    # a host-only handle refuses products (no device arrays) instead of computing anything on the CPU
    h = cbm.cbm_build(2, 2, rowptr, colidx, host_only=True, max_depth=16)
    lib.cbm_spmm.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                                     ctypes.c_void_p]
    assert lib.cbm_spmm(h.ptr, 16, 4, 4, 32, 4, None) == 6
    assert lib.cbm_spmm(h.ptr, None, 4, 4, 32, 4, None) == 1
    assert lib.cbm_spmm(h.ptr, 16, 2, 4, 32, 4, None) == 1


@pytest.mark.parametrize("blocks", [2, 3, 8])
def test_column_blocked_format_round_trips_and_keeps_property_1(blocks):
    """Column-blocked CBM (one tree over the B m part-rows): decompression gives back the matrix (Eq. (2)), the delta
    count stays within nnz (Property 1 holds for the stacked matrix, whose non-zeros are those of A), the tree covers
    B m part-rows, and an option that cannot be combined is refused."""
    g = wl.make_graph("protein", n=1500, knn=30)
    for self_loops in (False, True):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=self_loops, alpha=1, max_depth=16, host_only=True,
                          column_blocks=blocks)
        s = cbm.cbm_stats(h)
        assert s["column_blocks"] == blocks and s["m"] == g.n
        rows = orc.adjacency_lists(g.n, g.rowptr, g.colidx, add_self_loops=self_loops)
        want_rp, want_ci = _csr([sorted(r) for r in rows[1:]])
        rp, ci = cbm.cbm_decompress(h)
        assert np.array_equal(rp, want_rp) and np.array_equal(ci, want_ci)
        assert s["nnz"] == int(want_rp[-1])
        assert s["num_delta_plus"] + s["num_delta_minus"] <= s["nnz"]
        t = cbm.cbm_get_tree(h)
        assert len(t["parent"]) == blocks * g.n
        assert s["num_roots"] == int((t["parent"] < 0).sum())
        # a part-row is only ever compressed against a part-row of the same column range
        x = np.flatnonzero(t["parent"] >= 0)
        assert np.array_equal(x // g.n, t["parent"][x] // g.n)
    h1 = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=1, max_depth=16, host_only=True)
    hb = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=1, max_depth=16, host_only=True, column_blocks=blocks)
    s1, sb = cbm.cbm_stats(h1), cbm.cbm_stats(hb)
    assert s1["column_blocks"] == 1
    print(blocks, (sb["num_delta_plus"] + sb["num_delta_minus"]) / sb["nnz"], (s1["num_delta_plus"] + s1["num_delta_minus"]) / s1["nnz"])
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, host_only=True, column_blocks=blocks, transpose=True)
    assert e.value.status == 1
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, host_only=True, column_blocks=-2)
    assert e.value.status == 1
    # rectangular, with empty rows and an empty block
    rowptr, colidx = _csr([[0, 1, 2, 90], [], [1, 2, 90], [5]])
    h = cbm.cbm_build(4, 100, rowptr, colidx, host_only=True, max_depth=16, column_blocks=4)
    rp, ci = cbm.cbm_decompress(h)
    assert np.array_equal(rp, rowptr) and np.array_equal(ci, colidx)


def test_tuning_knobs_from_the_environment_are_held_in_range(monkeypatch):
    """Out-of-range values of the builder's environment knobs must not reach the work lists: zero sub-ranges
    would divide by zero, and an entry count of 2^24 or more would spill into a work item's flag bits."""
    rng = np.random.default_rng(3)
    n = 5000
    rows = [sorted(rng.choice(n, size=2000, replace=False).tolist()), [1, 2, 3], []]
    rowptr, colidx = _csr(rows)
    monkeypatch.setenv("CBM_PHASES", "0")
    h = cbm.cbm_build(3, n, rowptr, colidx, host_only=True, max_depth=16)
    s = _check_invariants(3, n, rowptr, colidx, h, 0, False)
    assert s["num_split_rows"] == 1
    monkeypatch.delenv("CBM_PHASES")
    for name in ("CBM_SPLIT_MIN", "CBM_SPLIT_LEN", "CBM_PATH_MAX", "CBM_FINE_MIN"):
        monkeypatch.setenv(name, str(1 << 26))
        h = cbm.cbm_build(3, n, rowptr, colidx, host_only=True, max_depth=16)
        _check_invariants(3, n, rowptr, colidx, h, 0, False)
        monkeypatch.delenv(name)
    for name in ("CBM_SPLIT_MIN", "CBM_SPLIT_LEN"):
        monkeypatch.setenv(name, "-5")
        h = cbm.cbm_build(3, n, rowptr, colidx, host_only=True, max_depth=16)
        _check_invariants(3, n, rowptr, colidx, h, 0, False)
        monkeypatch.delenv(name)


@pytest.mark.parametrize("name,kw", [("citation", dict(n=3000, p_in=3e-3, p_out=2e-4)), ("collaboration", dict(n=3000)),
                                     ("protein", dict(n=1200, knn=20)), ("rmat", dict(scale=10, edge_factor=8))])
def test_invariants_on_reduced_workloads(name, kw):
    g = wl.make_graph(name, **kw)
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=1, host_only=True, max_depth=16)
    s = cbm.cbm_stats(h)
    rp, ci = cbm.cbm_decompress(h)
    # A v I rebuilt exactly
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    want = np.unique(np.concatenate((rows.astype(np.int64) * g.n + g.colidx, np.arange(g.n, dtype=np.int64) * (g.n + 1))))
    got = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(rp)) * g.n + ci
    assert np.array_equal(got, want)
    assert s["num_delta_plus"] + s["num_delta_minus"] <= s["nnz"] and s["scalar_ops"] <= s["nnz"]
    t = cbm.cbm_get_tree(h)
    comp = t["parent"] >= 0
    assert np.all(t["level"][comp] == t["level"][t["parent"][comp]] + 1)


@pytest.mark.parametrize("self_loops", [False, True])
def test_transposed_build_holds_the_transpose(self_loops):
    """CBM_FLAG_TRANSPOSE: the handle is the CBM of A^T (of (A v I)^T with self loops) and satisfies the same
    invariants; the transpose is checked against scipy's."""
    import scipy.sparse as sp

    rng = np.random.default_rng(21 + self_loops)
    m, n = (70, 70) if self_loops else (50, 90)
    rows = _random_rows(rng, m, n, 0.15)                 # directed: not symmetric
    rows[3] = []
    rowptr, colidx = _csr(rows)
    h = cbm.cbm_build(m, n, rowptr, colidx, alpha=1, add_self_loops=self_loops, transpose=True, host_only=True, max_depth=16)
    A = sp.csr_matrix((np.ones(len(colidx)), colidx, rowptr), shape=(m, n))
    if self_loops:
        A = ((A + sp.identity(m, format="csr")) > 0).astype(np.float64)
    At = sp.csr_matrix(A.T)
    At.sort_indices()
    s = cbm.cbm_stats(h)
    assert (s["m"], s["n"], s["nnz"]) == (n, m, At.nnz)
    _check_invariants(n, m, At.indptr.astype(np.int64), At.indices.astype(np.int32), h, 1, False)
    cbm.cbm_free(h)


@pytest.mark.parametrize("seed", range(40))
def test_invariants_random_options(seed):
    """Seeded sweep over shapes, structure and every build option: the format must decompress to the input and
    keep Properties 1 and 2, the alpha rule and the draw rule whatever the options."""
    rng = np.random.default_rng(500 + seed)
    m = int(rng.integers(1, 400))
    square = bool(rng.integers(0, 2))
    n = m if square else int(rng.integers(1, 400))
    rows, base = [], None
    for _ in range(m):
        kind = int(rng.integers(0, 8))
        if kind == 0:
            r = []
        elif kind == 1 and base is not None:
            r = list(base)
        elif kind in (2, 3) and base is not None and len(base) > 2:
            r = sorted(set(base[:-1]) | set(rng.integers(0, n, size=2).tolist()))
        elif kind == 4 and n > 150:
            r = sorted(rng.choice(n, size=int(rng.integers(130, n)), replace=False).tolist())   # long enough to be split
        else:
            r = sorted(set(rng.integers(0, n, size=int(rng.integers(1, 30))).tolist()))
        rows.append(r)
        if r and rng.random() < 0.4:
            base = r
    rowptr, colidx = _csr(rows)
    alpha = int(rng.choice([0, 1, 2, 7]))
    self_loops = square and bool(rng.integers(0, 2))
    opts = dict(max_depth=int(rng.choice([-1, 2, 5, 16])), hub_cap=int(rng.choice([0, 3, -1])),
                max_candidates=int(rng.choice([0, 1, -1])), seed_roots=int(rng.choice([0, -1, 4])),
                exact_tree=bool(rng.integers(0, 3) == 0), num_threads=int(rng.choice([0, 1, 3])))
    h = cbm.cbm_build(m, n, rowptr, colidx, alpha=alpha, add_self_loops=self_loops, host_only=True, **opts)
    s = _check_invariants(m, n, rowptr, colidx, h, alpha, self_loops)
    if opts["max_depth"] > 0 and not opts["exact_tree"]:
        assert s["depth"] <= opts["max_depth"]
    cbm.cbm_free(h)


def test_build_is_independent_of_the_thread_count():
    """The candidate search, the transpose, the seeded tree growths and the entry stream run on several host threads;
    the result must not depend on how many (same tree, same statistics, same decompressed matrix)."""
    import workloads as wl

    g = wl.make_graph("collaboration", n=30000)
    ref = None
    for nt in (1, 2, 5, 0):
        h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=2, add_self_loops=True, host_only=True, max_depth=16,
                          num_threads=nt)
        t = cbm.cbm_get_tree(h)
        s = cbm.cbm_stats(h)
        s.pop("build_seconds")
        cur = (t, s, cbm.cbm_decompress(h))
        if ref is None:
            ref = cur
        else:
            assert all(np.array_equal(ref[0][k], cur[0][k]) for k in ref[0])
            assert ref[1] == cur[1]
            assert np.array_equal(ref[2][0], cur[2][0]) and np.array_equal(ref[2][1], cur[2][1])
        cbm.cbm_free(h)
