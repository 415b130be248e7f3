"""Seeded synthetic graphs standing in for the paper's datasets (Table 1), which
are not available offline.  Five recipes; every graph is undirected,
symmetrised, deduplicated, free of self-loops, and returned as a binary CSR
pattern (int64 row offsets, sorted int32 column indices, no value array).

Every recipe takes ``n`` (and the other size knobs) as arguments so tests can
run the same construction at reduced size; ``make_graph(name)`` uses the full
sizes.  Only input generation lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 240902208

CONFIGS = ("tiny", "citation", "collaboration", "protein", "rmat")


@dataclass
class Graph:
    name: str
    n: int
    rowptr: np.ndarray  # int64, n + 1
    colidx: np.ndarray  # int32, nnz, sorted within each row
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def csr_from_edges(n: int, src: np.ndarray, dst: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Symmetrise, drop self-loops and duplicates, return (rowptr, colidx)."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    shift = max(1, int(n - 1).bit_length())
    keys = np.concatenate(((src << shift) | dst, (dst << shift) | src))
    del src, dst
    keys = np.unique(keys)
    rows = keys >> shift
    colidx = (keys & ((1 << shift) - 1)).astype(np.int32)
    del keys
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=rowptr[1:])
    return rowptr, colidx


def _finish(name: str, n: int, src, dst, seed: int, **meta) -> Graph:
    rowptr, colidx = csr_from_edges(n, src, dst)
    deg = np.diff(rowptr)
    meta.update(seed=seed, nnz=int(rowptr[-1]), undirected_edges=int(rowptr[-1]) // 2,
                max_degree=int(deg.max()) if n else 0, avg_degree=float(deg.mean()) if n else 0.0)
    return Graph(name, n, rowptr, colidx, meta)


# --------------------------------------------------------------------------- #
def tiny_graph(n: int = 1024, communities: int = 8, core: int = 16, frac: float = 0.6,
               extra: int = 2, seed: int = BASE_SEED + 0) -> Graph:
    """Planted communities: each node links to a random ``frac`` of its
    community's core set plus ``extra`` uniform random nodes."""
    rng = _rng(seed)
    csize = n // communities
    pick = int(round(frac * core))
    src, dst = [], []
    for c in range(communities):
        members = np.arange(c * csize, (c + 1) * csize if c < communities - 1 else n)
        cores = rng.choice(members, size=min(core, len(members)), replace=False)
        for u in members:
            src.append(np.full(min(pick, len(cores)), u))
            dst.append(rng.choice(cores, size=min(pick, len(cores)), replace=False))
    src.append(np.repeat(np.arange(n), extra))
    dst.append(rng.integers(0, n, size=n * extra))
    return _finish("tiny", n, np.concatenate(src), np.concatenate(dst), seed,
                   recipe=f"{communities} communities, core {core}, {pick} core links + {extra} random")


# --------------------------------------------------------------------------- #
def citation_graph(n: int = 19717, blocks: int = 3, p_in: float = 4e-4, p_out: float = 2e-5,
                   copy_frac: float = 0.3, copy_keep: float = 0.8,
                   seed: int = BASE_SEED + 1) -> Graph:
    """Stochastic block model followed by copy-model rewiring: ``copy_frac`` of
    the nodes each copy ``copy_keep`` of one random neighbour's adjacency."""
    rng = _rng(seed)
    bounds = np.linspace(0, n, blocks + 1).astype(np.int64)
    src, dst = [], []
    for a in range(blocks):
        na = bounds[a + 1] - bounds[a]
        for b in range(a, blocks):
            nb = bounds[b + 1] - bounds[b]
            pairs = na * (na - 1) // 2 if a == b else na * nb
            cnt = rng.binomial(pairs, p_in if a == b else p_out)
            src.append(bounds[a] + rng.integers(0, na, size=cnt))
            dst.append(bounds[b] + rng.integers(0, nb, size=cnt))
    src, dst = np.concatenate(src), np.concatenate(dst)
    rowptr, colidx = csr_from_edges(n, src, dst)
    # copy step, against the adjacency as it stood before any copying
    copiers = rng.choice(n, size=int(round(copy_frac * n)), replace=False)
    csrc, cdst = [], []
    for u in copiers:
        nb = colidx[rowptr[u]:rowptr[u + 1]]
        if len(nb) == 0:
            continue
        v = nb[rng.integers(0, len(nb))]
        adj = colidx[rowptr[v]:rowptr[v + 1]]
        take = adj[rng.random(len(adj)) < copy_keep]
        csrc.append(np.full(len(take), u))
        cdst.append(take)
    if csrc:
        src = np.concatenate([src] + csrc)
        dst = np.concatenate([dst] + cdst)
    return _finish("citation", n, src, dst, seed,
                   recipe=f"SBM {blocks} blocks p_in={p_in} p_out={p_out}, {copy_frac:.0%} copy {copy_keep:.0%}")


# --------------------------------------------------------------------------- #
def _zipf_sizes(rng: np.random.Generator, count: int, a: float, lo: int, hi: int) -> np.ndarray:
    support = np.arange(lo, hi + 1)
    p = support.astype(np.float64) ** (-a)
    p /= p.sum()
    return rng.choice(support, size=count, p=p)


def collaboration_graph(n: int = 235868, mean_memberships: float = 3.0, zipf_a: float = 2.0,
                        lo: int = 2, hi: int = 50, seed: int = BASE_SEED + 2) -> Graph:
    """Union of random cliques (hyperedges): every node draws Poisson(mean)
    memberships; the shuffled membership stubs are cut into cliques whose sizes
    follow a Zipf law truncated to [lo, hi]."""
    rng = _rng(seed)
    stubs = np.repeat(np.arange(n, dtype=np.int64), rng.poisson(mean_memberships, size=n))
    rng.shuffle(stubs)
    mean_size = float((np.arange(lo, hi + 1) ** (1.0 - zipf_a)).sum()
                      / (np.arange(lo, hi + 1) ** (-zipf_a)).sum())
    sizes = _zipf_sizes(rng, int(len(stubs) / mean_size * 1.2) + 16, zipf_a, lo, hi)
    ends = np.cumsum(sizes)
    ncl = int(np.searchsorted(ends, len(stubs), side="right"))
    sizes, ends = sizes[:ncl], ends[:ncl]
    starts = ends - sizes
    src, dst = [], []
    for s in np.unique(sizes):
        sel = starts[sizes == s]
        members = stubs[sel[:, None] + np.arange(s)[None, :]]  # (cliques, s)
        iu, ju = np.triu_indices(int(s), k=1)
        src.append(members[:, iu].ravel())
        dst.append(members[:, ju].ravel())
    return _finish("collaboration", n, np.concatenate(src), np.concatenate(dst), seed,
                   cliques=ncl,
                   recipe=f"cliques Zipf({zipf_a}) in [{lo},{hi}], Poisson({mean_memberships}) memberships")


# --------------------------------------------------------------------------- #
def protein_graph(n: int = 132534, knn: int = 300, seed: int = BASE_SEED + 3, workers: int = -1) -> Graph:
    """Geometric graph: uniform points in the unit cube, each linked to its
    ``knn`` nearest neighbours, then symmetrised."""
    from scipy.spatial import cKDTree

    rng = _rng(seed)
    pts = rng.random((n, 3))
    kk = min(knn, n - 1)
    tree = cKDTree(pts)
    src, dst = [], []
    step = 16384
    for s in range(0, n, step):
        _, nb = tree.query(pts[s:s + step], k=kk + 1, workers=workers)
        nb = nb[:, 1:] if kk >= 1 else nb[:, :0]
        src.append(np.repeat(np.arange(s, min(n, s + step), dtype=np.int64), kk))
        dst.append(nb.astype(np.int64).ravel())
    return _finish("protein", n, np.concatenate(src), np.concatenate(dst), seed,
                   recipe=f"{knn}-nearest-neighbour graph of uniform points in the unit cube")


# --------------------------------------------------------------------------- #
def rmat_graph(scale: int = 21, edge_factor: int = 32, abcd=(0.57, 0.19, 0.19, 0.05),
               seed: int = BASE_SEED + 4, permute: bool = True) -> Graph:
    """R-MAT: ``edge_factor * 2**scale`` directed samples, symmetrised and
    deduplicated.  Vertex labels are shuffled (``permute``) so hub rows are not
    contiguous in memory."""
    rng = _rng(seed)
    n = 1 << scale
    m = edge_factor * n
    a, b, c, _ = abcd
    t_ab = np.uint32(min(2 ** 32 - 1, round(a * 2 ** 32)))
    t_abc = np.uint32(min(2 ** 32 - 1, round((a + b) * 2 ** 32)))
    t_abcd = np.uint32(min(2 ** 32 - 1, round((a + b + c) * 2 ** 32)))
    src = np.zeros(m, dtype=np.int32)
    dst = np.zeros(m, dtype=np.int32)
    chunk = 1 << 23
    for s in range(0, m, chunk):
        e = min(m, s + chunk)
        u = np.zeros(e - s, dtype=np.int32)
        v = np.zeros(e - s, dtype=np.int32)
        for _level in range(scale):
            r = rng.integers(0, 2 ** 32, size=e - s, dtype=np.uint32)
            ubit = r >= t_abc                              # quadrants c, d: lower half
            vbit = ((r >= t_ab) & (r < t_abc)) | (r >= t_abcd)  # quadrants b, d: right half
            u = (u << 1) | ubit
            v = (v << 1) | vbit
        src[s:e], dst[s:e] = u, v
    if permute:
        perm = rng.permutation(n).astype(np.int32)
        src, dst = perm[src], perm[dst]
    return _finish("rmat", n, src, dst, seed,
                   recipe=f"R-MAT scale {scale} edge factor {edge_factor} abcd={abcd} permute={permute}")


# --------------------------------------------------------------------------- #
def make_graph(name: str, **overrides) -> Graph:
    """Full-size graph of one of the five named configurations."""
    fn = {"tiny": tiny_graph, "citation": citation_graph, "collaboration": collaboration_graph,
          "protein": protein_graph, "rmat": rmat_graph}[name]
    return fn(**overrides)
