"""cbm_spmm_noalloc (the entry point for callers that cannot allocate) against cbm_spmm, through the C ABI:
same result bit for bit, on two calls in a row that share the library's static scratch, the second smaller."""
import numpy as np
import pytest

import workloads as wl
from oracle import cbm_oracle as orc

pytestmark = pytest.mark.gpu


def _csr(rows):
    rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c in sorted(r)], dtype=np.int32)
    return rowptr, colidx


def _hub_matrix(seed, m, n, longest):
    """Mostly short rows plus a tenth of long ones (their delta lists are split into segments: scratch rows)."""
    rng = np.random.default_rng(seed)
    sizes = np.where(rng.random(m) < 0.1, rng.integers(200, longest, size=m), rng.integers(0, 40, size=m))
    return _csr([sorted(rng.choice(n, size=int(s), replace=False).tolist()) for s in sizes])


def test_noalloc_matches_spmm_on_two_calls_in_a_row():
    import torch

    import paper_2409_02208_amd as cbm

    assert torch.cuda.is_available(), "this test needs the MI355X"
    cases = []
    for seed, m, n, longest, k in ((11, 3000, 5000, 3000, 96), (12, 700, 1500, 900, 18)):   # the second is smaller
        rowptr, colidx = _hub_matrix(seed, m, n, longest)
        h = cbm.cbm_build(m, n, rowptr, colidx, max_depth=16)
        assert cbm.cbm_stats(h)["num_split_rows"] > 0
        Xi, Xg = wl.integer_features(n, k, seed), wl.gaussian_features(n, k, seed)
        cases.append((m, n, k, rowptr, colidx, h, Xi, Xg))

    # a product on another handle first, so that the kernels' code is already on the GPU when memory is compared
    rp0, ci0 = _csr([[0, 1], [1], []])
    h0 = cbm.cbm_build(3, 2, rp0, ci0, max_depth=16)
    cbm.cbm_spmm(h0, torch.zeros((2, 96), device="cuda"), torch.zeros((3, 96), device="cuda"))
    cbm.cbm_spmm(h0, torch.zeros((2, 18), device="cuda"), torch.zeros((3, 18), device="cuda"))
    torch.cuda.synchronize()

    got = []
    for m, n, k, rowptr, colidx, h, Xi, Xg in cases:        # the two calls in a row, nothing between them
        Xd = [torch.from_numpy(a).cuda() for a in (Xi, Xg)]
        Y = [torch.full((m, k), float("nan"), device="cuda") for _ in range(2)]
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        for x, y in zip(Xd, Y):
            cbm.cbm_spmm_noalloc(h, x, y)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "cbm_spmm_noalloc changed the free device memory"
        got.append([y.cpu().numpy() for y in Y])
    for (m, n, k, rowptr, colidx, h, Xi, Xg), (yi, yg) in zip(cases, got):
        want = []
        for X in (Xi, Xg):
            Y = torch.full((m, k), float("nan"), device="cuda")
            cbm.cbm_spmm(h, torch.from_numpy(X).cuda(), Y)
            torch.cuda.synchronize()
            want.append(Y.cpu().numpy())
        assert np.array_equal(yi, want[0]) and np.array_equal(yg, want[1])          # same kernels, same order of sums
        assert np.array_equal(yi.astype(np.float64), orc.spmm_csr(rowptr, colidx, Xi))  # and the oracle, bit for bit
        ref = orc.spmm_csr(rowptr, colidx, Xg)
        scale = np.abs(ref).max(axis=1)
        ok = scale > 0
        assert (np.abs(yg - ref).max(axis=1)[ok] / scale[ok]).max() <= 1e-5
        assert np.all(yg[~ok] == 0)


def test_noalloc_rejects_what_the_static_scratch_cannot_hold():
    import torch

    import paper_2409_02208_amd as cbm

    rng = np.random.default_rng(13)
    m, n, k = 700, 4000, 4096
    rowptr, colidx = _csr([sorted(rng.choice(n, size=2000, replace=False).tolist()) for _ in range(m)])
    h = cbm.cbm_build(m, n, rowptr, colidx, max_depth=1)   # every row in full: 32 segments each
    X = torch.zeros((n, k), device="cuda")
    Y = torch.zeros((m, k), device="cuda")
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_spmm_noalloc(h, X, Y)
    assert e.value.status == 5
    cbm.cbm_spmm_noalloc(h, X[:, :64], Y[:, :64])   # the same handle at a width that fits
    cbm.cbm_profile_enable(h, True)
    with pytest.raises(cbm.CbmError) as e:
        cbm.cbm_spmm_noalloc(h, X[:, :64], Y[:, :64])
    assert e.value.status == 6
    cbm.cbm_profile_enable(h, False)
    torch.cuda.synchronize()
