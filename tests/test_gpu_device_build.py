"""The builder's GPU side (CBM_FLAG_DEVICE_BUILD: candidate search and delta lists on the GPU) against the host
builder: both follow one selection rule with one tie-break and write the delta lists in one order, so the
compression tree, the delta lists and the products must be identical, not merely equivalent."""
import numpy as np
import pytest

import workloads as wl
from oracle import cbm_oracle as orc

pytestmark = pytest.mark.gpu

SMALL = {
    "tiny": {},
    "citation": dict(n=6000, p_in=1.5e-3, p_out=1e-4),
    "collaboration": dict(n=20000),
    "protein": dict(n=6000, knn=60),
    "rmat": dict(scale=14, edge_factor=16),
}


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2409_02208_amd as cbm

    assert torch.cuda.is_available()
    return torch, cbm


def _csr(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in sorted(r)], dtype=np.int32)
    return rowptr, colidx


def _same_tree(cbm, m, n, rowptr, colidx, **opts):
    hh = cbm.cbm_build(m, n, rowptr, colidx, host_search=True, **opts)
    hd = cbm.cbm_build(m, n, rowptr, colidx, device_build=True, **opts)
    th, td = cbm.cbm_get_tree(hh), cbm.cbm_get_tree(hd)
    for key in ("parent", "nplus", "nminus", "level"):
        assert np.array_equal(th[key], td[key]), (key, opts)
    sh, sd = cbm.cbm_stats(hh), cbm.cbm_stats(hd)
    for key in ("num_delta_plus", "num_delta_minus", "depth", "rounds", "num_tasks", "scalar_ops", "bytes_cbm"):
        assert sh[key] == sd[key], (key, opts)
    # the delta lists made on the GPU rebuild the matrix (Eq. (2)) exactly as the host's do
    (rph, cih), (rpd, cid) = cbm.cbm_decompress(hh), cbm.cbm_decompress(hd)
    assert np.array_equal(rph, rpd) and np.array_equal(cih, cid)
    return hh, hd


@pytest.mark.parametrize("name", wl.CONFIGS)
def test_device_candidates_give_the_host_tree(env, name):
    torch, cbm = env
    g = wl.make_graph(name, **SMALL[name])
    for opts in (dict(max_depth=16), dict(max_depth=16, add_self_loops=True, alpha=2), dict(max_depth=-1, alpha=4),
                 dict(max_depth=16, hub_cap=8), dict(max_depth=16, hub_cap=-1, max_candidates=3),
                 dict(max_depth=16, max_candidates=16, alpha=1)):
        hh, hd = _same_tree(cbm, g.n, g.n, g.rowptr, g.colidx, **opts)
        if opts.get("add_self_loops"):
            X = torch.from_numpy(wl.gaussian_features(g.n, 32, 7)).cuda()
            Yh, Yd = torch.empty_like(X), torch.empty_like(X)
            cbm.cbm_spmm_normalized(hh, X, Yh)
            cbm.cbm_spmm_normalized(hd, X, Yd)
            torch.cuda.synchronize()
            assert torch.equal(Yh, Yd)
        cbm.cbm_free(hh)
        cbm.cbm_free(hd)


def test_device_candidates_on_degenerate_inputs(env):
    torch, cbm = env
    rng = np.random.default_rng(5)
    n = 3000
    hub = sorted(rng.choice(n, size=2500, replace=False).tolist())            # a row longer than any cap
    rows = [hub, sorted(set(hub[:2400]) | {1, 2}), [], [], [7], [7], [7, 8], list(range(40)), list(range(1, 41))]
    rows += [[0] + sorted(rng.choice(np.arange(1, n), size=int(s), replace=False).tolist())   # column 0 is a hub column
             for s in rng.integers(0, 30, size=n - len(rows))]
    rowptr, colidx = _csr(rows)
    for opts in (dict(max_depth=16), dict(max_depth=16, hub_cap=64), dict(max_depth=-1, hub_cap=-1),
                 dict(max_depth=16, alpha=3, max_candidates=1)):
        hh, hd = _same_tree(cbm, n, n, rowptr, colidx, **opts)
        Xi = wl.integer_features(n, 16, 3)
        Y = torch.full((n, 16), float("nan"), device="cuda")
        cbm.cbm_spmm(hd, torch.from_numpy(Xi).cuda(), Y)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), orc.spmm_csr(rowptr, colidx, Xi))
    # rectangular, one row, no rows
    m2, n2 = 500, 90
    rowptr, colidx = _csr([sorted(rng.choice(n2, size=int(s), replace=False).tolist()) for s in rng.integers(0, 40, size=m2)])
    _same_tree(cbm, m2, n2, rowptr, colidx, max_depth=16)
    _same_tree(cbm, 1, 5, *_csr([[1, 3]]), max_depth=16)
    h = cbm.cbm_build(0, 5, np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), device_build=True)
    assert cbm.cbm_stats(h)["m"] == 0


def test_device_deltas_of_a_transposed_directed_matrix(env):
    torch, cbm = env
    rng = np.random.default_rng(9)
    m, n = 4000, 2500
    base = [sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in rng.integers(5, 60, size=200)]
    rows = []
    for i in range(m):   # near-copies of a few base rows: a deep tree with both kinds of delta
        r = set(base[int(rng.integers(len(base)))])
        r ^= set(rng.choice(n, size=3, replace=False).tolist())
        rows.append(sorted(r))
    rowptr, colidx = _csr(rows)
    for opts in (dict(max_depth=16), dict(max_depth=-1, transpose=True), dict(max_depth=16, alpha=2, transpose=True)):
        hh, hd = _same_tree(cbm, m, n, rowptr, colidx, **opts)
        s = cbm.cbm_stats(hd)
        assert s["num_delta_minus"] > 0 and s["depth"] > 2
        mm, nn = (n, m) if opts.get("transpose") else (m, n)
        X = torch.from_numpy(wl.gaussian_features(nn, 24, 3)).cuda()
        Yh = torch.full((mm, 24), float("nan"), device="cuda")
        Yd = torch.full((mm, 24), float("nan"), device="cuda")
        cbm.cbm_spmm(hh, X, Yh)
        cbm.cbm_spmm(hd, X, Yd)
        torch.cuda.synchronize()
        assert torch.equal(Yh, Yd)


def test_device_build_argument_errors(env):
    torch, cbm = env
    g = wl.tiny_graph()
    with pytest.raises(cbm.CbmError) as e:      # the device search keeps at most 16 candidates per row
        cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, device_build=True, max_candidates=-1, max_depth=16)
    assert e.value.status == 1
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, device_build=True, host_only=True, max_depth=16)
    assert e.value.status == 1
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, device_build=True, host_search=True, max_depth=16)
    assert e.value.status == 1
