"""Seeded sweep over random shapes and options: every product entry point against the oracle on matrices whose
structure mixes what the kernels treat differently (empty rows, duplicate rows, near-duplicates that form deep
chains, rows long enough to be split, hub columns), with odd k, strided operands and every build option."""
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

    assert torch.cuda.is_available()
    return torch, cbm


def _matrix(rng, m, n):
    rows = []
    base = None
    for i in range(m):
        kind = rng.integers(0, 10)
        if kind == 0 or n == 0:
            r = set()
        elif kind == 1 and base is not None:
            r = set(base)                                             # duplicate of an earlier row
        elif kind in (2, 3, 4) and base is not None and len(base) > 2:
            r = set(base)                                             # a few columns away from an earlier row
            for c in rng.choice(sorted(r), size=min(len(r) - 1, int(rng.integers(1, 4))), replace=False):
                r.discard(int(c))
            r |= set(rng.integers(0, n, size=int(rng.integers(0, 4))).tolist())
        elif kind == 5 and n > 400:
            r = set(rng.choice(n, size=int(rng.integers(130, min(n, 1500))), replace=False).tolist())   # a split row
        else:
            r = set(rng.integers(0, n, size=int(rng.integers(1, 40))).tolist())
        if rng.random() < 0.5 and n > 0:
            r.add(0)                                                  # column 0 is a hub column
        rows.append(sorted(r))
        if r and rng.random() < 0.3:
            base = sorted(r)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in r], dtype=np.int32)
    return rowptr, colidx


def _err(got, ref, ref_abs):
    """Forward error against the sum of magnitudes: max |got - ref| / (|M| |X|), element by element; where that sum
    is zero the result must be exactly zero.  (With k as small as 1 a row's own magnitude can cancel to nothing, so
    the row-scaled measure of the other parity tests says little here.)"""
    diff = np.abs(got.astype(np.float64) - ref)
    assert np.all(diff[ref_abs == 0] == 0)
    nz = ref_abs > 0
    return float((diff[nz] / ref_abs[nz]).max()) if nz.any() else 0.0


@pytest.mark.parametrize("seed", range(80))
def test_random_configuration(env, seed):
    torch, cbm = env
    rng = np.random.default_rng(1000 + seed)
    square = seed % 3 != 0
    m = int(rng.integers(1, 2500))
    n = m if square else int(rng.integers(1, 2500))
    k = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 48, 100, 128, 130, 256, 300]))
    rowptr, colidx = _matrix(rng, m, n)
    opts = dict(alpha=int(rng.choice([0, 1, 2, 5])), max_depth=int(rng.choice([-1, 2, 3, 16, 16, 16])),
                hub_cap=int(rng.choice([0, 0, 4, -1])), max_candidates=int(rng.choice([0, 0, 1, 16])),
                seed_roots=int(rng.choice([0, -1, 3])), device_build=bool(rng.integers(0, 2)),
                exact_tree=bool(rng.integers(0, 4) == 0))
    self_loops = square and bool(rng.integers(0, 2))
    print(f"seed={seed} m={m} n={n} k={k} nnz={len(colidx)} self_loops={self_loops} {opts}", flush=True)
    h = cbm.cbm_build(m, n, rowptr, colidx, add_self_loops=self_loops, **opts)
    if self_loops:
        R = orc.adjacency_lists(m, rowptr, colidx, add_self_loops=True)[1:]
        rp = np.zeros(m + 1, dtype=np.int64)
        rp[1:] = np.cumsum([len(r) for r in R])
        ci = np.array([c for r in R for c in sorted(r)], dtype=np.int32)
    else:
        rp, ci = rowptr, colidx
    # strided operands: X and Y are column slices of wider buffers (leading dimension > k, maybe misaligned)
    pad = int(rng.choice([0, 1, 4]))
    Xi = wl.integer_features(n, k, seed)
    Xg = wl.gaussian_features(n, k, seed)
    Xbuf = torch.zeros((n, k + pad), device="cuda")
    Ybuf = torch.full((m, k + pad), float("nan"), device="cuda")
    X, Y = Xbuf[:, pad:], Ybuf[:, pad:]

    def run(fn, Xh, *args):
        X.copy_(torch.from_numpy(Xh))
        Ybuf.fill_(float("nan"))
        fn(h, *args, X, Y)
        torch.cuda.synchronize()
        if pad:
            assert bool(torch.isnan(Ybuf[:, :pad]).all()), "wrote outside the k columns"
        return Y.cpu().numpy()

    ref = orc.spmm_csr(rp, ci, Xi)
    assert np.abs(ref).max(initial=0) < 2 ** 24
    assert np.array_equal(run(cbm.cbm_spmm, Xi).astype(np.float64), ref)
    assert _err(run(cbm.cbm_spmm_mean, Xg), orc.spmm_csr_mean(rp, ci, Xg), orc.spmm_csr_mean(rp, ci, np.abs(Xg))) <= TOL
    if square:
        assert np.array_equal(run(cbm.cbm_spmm_gin, Xi, 1.0).astype(np.float64), orc.spmm_csr_gin(rp, ci, Xi, 1.0))
    if self_loops:
        want = orc.spmm_csr_normalized(rowptr, colidx, Xg)
        mag = orc.spmm_csr_normalized(rowptr, colidx, np.abs(Xg))
        assert _err(run(cbm.cbm_spmm_normalized, Xg), want, mag) <= TOL
        got = run(cbm.cbm_spmm_normalized_relu, Xg).astype(np.float64)
        assert (np.abs(got - np.maximum(want, 0.0)) <= TOL * mag).all()
    cbm.cbm_free(h)
