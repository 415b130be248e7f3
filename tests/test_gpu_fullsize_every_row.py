"""GPU parity at full size on EVERY output row: the products bench.py times (R-MAT at k = 128 and 64, the protein
graph at k = 256 and 112, each of the ten iterates of the collaboration chain at k = 128) against the oracle's plain-C
CSR products (fp64 accumulation, pinned to the numpy oracle in test_oracle_c_baseline.py), element by element,
1e-5 row-scaled.  The sampled numpy check of test_gpu_fullsize.py stays beside it."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import workloads as wl
from oracle import csr_ref

pytestmark = pytest.mark.gpu

TOL = 1e-5
BLOCK = 32768   # rows per call of the C oracle
WORKERS = 16    # the C routines release the interpreter lock: row blocks run side by side on the host cores


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2409_02208_amd as cbm

    assert torch.cuda.is_available()
    return torch, cbm


_graphs = {}


def graph(name):
    if name not in _graphs:
        _graphs.clear()   # one full-size graph in memory at a time
        _graphs[name] = wl.make_graph(name)
        print(f"{name}: n={_graphs[name].n} nnz={_graphs[name].nnz}", flush=True)
    return _graphs[name]


def every_row_error(g, X, got, normalized):
    """max over ALL rows of max_j |got - ref| / max_j |ref| against the C oracle; rows whose reference is zero must be zero."""
    d = np.diff(g.rowptr) + 1  # the generators emit no self-loops

    def block(b):
        e = min(g.n, b + BLOCK)
        ref = (csr_ref.spmm_norm_f64(g.rowptr, g.colidx, d, X, b, e) if normalized
               else csr_ref.spmm_f64(g.rowptr, g.colidx, X, b, e))
        diff = np.abs(got[b:e].astype(np.float64) - ref).max(axis=1)
        scale = np.abs(ref).max(axis=1)
        zero = scale == 0
        assert np.all(diff[zero] == 0), "rows with an all-zero reference must be exactly zero"
        return float((diff[~zero] / scale[~zero]).max()) if np.any(~zero) else 0.0

    with ThreadPoolExecutor(max_workers=WORKERS) as ex:
        return max(ex.map(block, range(0, g.n, BLOCK)))


@pytest.mark.parametrize("name,k,alpha", [("rmat", 128, 2), ("rmat", 64, 2), ("protein", 256, 2), ("protein", 112, 2)])
def test_normalized_product_every_row(env, name, k, alpha):
    torch, cbm = env
    g = graph(name)
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, add_self_loops=True, alpha=alpha)   # as bench.py builds it
    X = wl.gaussian_features(g.n, k, g.meta["seed"])
    Y = torch.full((g.n, k), float("nan"), device="cuda")
    cbm.cbm_spmm_normalized(h, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    del Y
    cbm.cbm_free(h)
    assert not np.isnan(got).any(), "every row of Y must be written"
    err = every_row_error(g, X, got, normalized=True)
    print(f"{name} k={k}: max row-scaled error over all {g.n} rows {err:.2e}", flush=True)
    assert err <= TOL, (name, k, err)


def test_collaboration_chain_every_iterate_every_row(env):
    """X_(t+1) = A X_t, ten products at k = 128: every iterate against the oracle applied to the GPU's previous
    iterate (so rounding does not compound between iterates), every row."""
    torch, cbm = env
    g = graph("collaboration")
    k = 128
    h = cbm.cbm_build(g.n, g.n, g.rowptr, g.colidx, alpha=2)
    s = cbm.cbm_stats(h)
    assert s["depth"] > 1 and s["num_delta_plus"] + s["num_delta_minus"] < s["nnz"]   # the chain runs through a real tree
    a = torch.from_numpy(wl.gaussian_features(g.n, k, 5)).cuda()
    b = torch.empty_like(a)
    prev = a.cpu().numpy()
    worst = 0.0
    for it in range(10):
        b.fill_(float("nan"))
        cbm.cbm_spmm(h, a, b)
        torch.cuda.synchronize()
        got = b.cpu().numpy()
        assert np.isfinite(got).all()
        err = every_row_error(g, prev, got, normalized=False)
        worst = max(worst, err)
        assert err <= TOL, (it, err)
        prev = got
        a, b = b, a
    print(f"collaboration chain: worst iterate error {worst:.2e}", flush=True)
    cbm.cbm_free(h)
