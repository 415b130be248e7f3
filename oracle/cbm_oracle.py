"""CPU oracle for the Compressed Binary Matrix (CBM) product.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library must compute.  It shares no code with the library, is never imported
by it, and may be imported only by tests, the smoke check and the benchmark's
CPU-baseline leg.  All floating point is fp64 unless a caller rounds the result.

Notation follows the paper: A is an m x n binary matrix whose row a_x is a sorted
list of column indices; vertex 0 of the distance graph is the virtual null row,
so matrix row i (0-based) is vertex i + 1; r_x is the vertex that row x is
compressed against (r_x = 0 means "stored in full").

Parity pins (see tests/test_oracle_*.py): a hand-worked example, dense brute
force, closed forms (complete graph, cycle, lower-triangular/cumsum, the
eigen-identity of the normalised adjacency, neighbour mean / GIN sum on the
complete graph and the cycle), library MST / arborescence weights,
and exhaustive enumeration of all arborescences on tiny inputs.  Every function
below is covered by at least one of them; none is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------- #
# O1: the plain definition on a dense 0/1 matrix (tiny inputs only)
# --------------------------------------------------------------------------- #


def dense_from_csr(m: int, n: int, rowptr, colidx) -> np.ndarray:
    """A as a dense m x n array of 0.0/1.0 (Section 2: rows are adjacency lists)."""
    A = np.zeros((m, n), dtype=np.float64)
    for i in range(m):
        for p in range(int(rowptr[i]), int(rowptr[i + 1])):
            A[i, int(colidx[p])] = 1.0
    return A


def spmm_dense(A: np.ndarray, X: np.ndarray) -> np.ndarray:
    """C = A.B by the textbook definition (Section 2.2, operands of Algorithm 1)."""
    return A.astype(np.float64) @ X.astype(np.float64)


def normalized_dense(A: np.ndarray) -> np.ndarray:
    """A_hat = D^-1/2 (A + I) D^-1/2 (Eq. (1) and the text under it).

    Reading taken where the paper is silent: A + I is the set union A v I (a
    diagonal entry already present stays 1), and D holds the row sums of A v I,
    the renormalisation of the GCN paper it cites, so no degree is zero.
    """
    m, n = A.shape
    if m != n:
        raise ValueError("the normalised adjacency needs a square matrix")
    At = np.maximum(A.astype(np.float64), np.eye(n))
    d = At.sum(axis=1)
    s = 1.0 / np.sqrt(d)
    return (s[:, None] * At) * s[None, :]


# --------------------------------------------------------------------------- #
# O2: row-by-row sums over the adjacency lists, fp64 accumulation
# --------------------------------------------------------------------------- #


def spmm_csr(rowptr, colidx, X: np.ndarray, rows=None) -> np.ndarray:
    """Y[i,:] = sum_{j in a_i} X[j,:]; ``rows`` selects a subset of output rows."""
    rows = range(len(rowptr) - 1) if rows is None else rows
    Y = np.zeros((len(rows), X.shape[1]), dtype=np.float64)
    for o, i in enumerate(rows):
        cols = colidx[int(rowptr[i]):int(rowptr[i + 1])]
        if len(cols):
            Y[o] = X[cols].sum(axis=0, dtype=np.float64)
    return Y


def degrees_with_self_loops(rowptr, colidx) -> np.ndarray:
    """d_i = |a_i v {i}|: row sums of A v I."""
    n = len(rowptr) - 1
    d = np.zeros(n, dtype=np.int64)
    for i in range(n):
        cols = colidx[int(rowptr[i]):int(rowptr[i + 1])]
        d[i] = len(cols) + (0 if np.any(cols == i) else 1)
    return d


def spmm_csr_normalized(rowptr, colidx, X: np.ndarray, rows=None, d=None) -> np.ndarray:
    """Y[i,:] = d_i^-1/2 * sum_{j in a_i v {i}} d_j^-1/2 X[j,:] (Eq. (1) text)."""
    n = len(rowptr) - 1
    if d is None:
        d = degrees_with_self_loops(rowptr, colidx)
    s = 1.0 / np.sqrt(d.astype(np.float64))
    rows = range(n) if rows is None else rows
    Y = np.zeros((len(rows), X.shape[1]), dtype=np.float64)
    for o, i in enumerate(rows):
        cols = np.asarray(colidx[int(rowptr[i]):int(rowptr[i + 1])], dtype=np.int64)
        if not np.any(cols == i):
            cols = np.concatenate((cols, [i]))
        Y[o] = s[i] * (s[cols, None] * X[cols].astype(np.float64)).sum(axis=0)
    return Y


def spmm_csr_mean(rowptr, colidx, X: np.ndarray, rows=None) -> np.ndarray:
    """Y[i,:] = mean_{j in a_i} X[j,:], a zero row where a_i is empty: the mean
    aggregator of the GraphSAGE layer (one of the layers Section 1 names as built
    on the same product)."""
    rows = range(len(rowptr) - 1) if rows is None else rows
    Y = np.zeros((len(rows), X.shape[1]), dtype=np.float64)
    for o, i in enumerate(rows):
        cols = colidx[int(rowptr[i]):int(rowptr[i + 1])]
        if len(cols):
            Y[o] = X[cols].sum(axis=0, dtype=np.float64) / len(cols)
    return Y


def spmm_csr_gin(rowptr, colidx, X: np.ndarray, eps: float, rows=None) -> np.ndarray:
    """Y[i,:] = (1 + eps) X[i,:] + sum_{j in a_i} X[j,:]: the aggregator of the GIN
    layer (Section 1 names it among the layers built on the same product)."""
    rows = range(len(rowptr) - 1) if rows is None else rows
    Y = np.zeros((len(rows), X.shape[1]), dtype=np.float64)
    for o, i in enumerate(rows):
        cols = colidx[int(rowptr[i]):int(rowptr[i + 1])]
        Y[o] = (1.0 + float(eps)) * X[i].astype(np.float64)
        if len(cols):
            Y[o] += X[cols].sum(axis=0, dtype=np.float64)
    return Y


# --------------------------------------------------------------------------- #
# O3: the CBM format and Algorithm 1, literally
# --------------------------------------------------------------------------- #


def adjacency_lists(m: int, rowptr, colidx, add_self_loops: bool = False) -> list:
    """rows[v] for v = 0..m: rows[0] is the null row, rows[i+1] = a_i as a frozenset."""
    rows = [frozenset()]
    for i in range(m):
        s = set(int(c) for c in colidx[int(rowptr[i]):int(rowptr[i + 1])])
        if add_self_loops:
            s.add(i)
        rows.append(frozenset(s))
    return rows


def hamming_distance_graph(rows: list) -> np.ndarray:
    """W[y,x] = number of deltas to turn row y into row x, for all vertex pairs
    of the extended distance graph (Section 2, "Minimizing the number of deltas"
    and "Worst-case guarantees").  Through the list intersection of Lemma 2.1:
    w = nnz(a_x) + nnz(a_y) - 2 |a_x n a_y|; with the null row as vertex 0 this
    gives W[0,x] = nnz(a_x)."""
    V = len(rows)
    W = np.zeros((V, V), dtype=np.int64)
    for y in range(V):
        for x in range(V):
            W[y, x] = len(rows[x]) + len(rows[y]) - 2 * len(rows[x] & rows[y])
    return W


def admissible_edges(W: np.ndarray, alpha: int) -> np.ndarray:
    """Directed edge mask after pruning (Section 2.2, "Edge Pruning"): edge (y,x)
    goes when W[y,x] > nnz(a_x) - alpha.  Reading taken: edges leaving the virtual
    vertex are exempt (the same paragraph relies on them all being present);
    no edge enters vertex 0 and there are no self-edges."""
    V = W.shape[0]
    nnz = W[0]
    keep = W <= (nnz[None, :] - alpha)
    keep[0, :] = True
    keep[:, 0] = False
    keep[np.arange(V), np.arange(V)] = False
    return keep


def mst_rooted_at_virtual(W: np.ndarray) -> np.ndarray:
    """Chain of compression for alpha = 0: a minimum spanning tree of the
    undirected extended distance graph, rooted at vertex 0 (Section 2).  Kruskal
    with the draw rule of Section 2.2: among equal weights an edge leaving the
    virtual vertex goes first; remaining draws by (smaller endpoint, larger
    endpoint).  Returns r[0..m] with r[0] = -1."""
    V = W.shape[0]
    edges = []
    for y in range(V):
        for x in range(y + 1, V):
            edges.append((int(W[y, x]), 0 if y == 0 else 1, y, x))
    edges.sort()
    comp = list(range(V))

    def find(v):
        while comp[v] != v:
            comp[v] = comp[comp[v]]
            v = comp[v]
        return v

    nbrs = [[] for _ in range(V)]
    for _w, _nv, y, x in edges:
        fy, fx = find(y), find(x)
        if fy != fx:
            comp[fy] = fx
            nbrs[y].append(x)
            nbrs[x].append(y)
    r = np.full(V, -2, dtype=np.int64)
    r[0] = -1
    frontier = [0]
    while frontier:
        nxt = []
        for y in frontier:
            for x in nbrs[y]:
                if r[x] == -2:
                    r[x] = y
                    nxt.append(x)
        frontier = nxt
    assert not np.any(r == -2)
    return r


def mca_rooted_at_virtual(W: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """Chain of compression for alpha > 0: a minimum cost arborescence of the
    pruned, now directed, distance graph rooted at vertex 0 (Section 2.2, "Edge
    Pruning").  Chu-Liu/Edmonds by cycle contraction on a dense cost matrix.
    Draw rule: total weight first, then as few non-virtual edges as possible
    (cost (V+1) * w + [y != 0])."""
    V = W.shape[0]
    INF = float("inf")
    cost = [[INF] * V for _ in range(V)]
    for y in range(V):
        for x in range(1, V):
            if y != x and keep[y, x]:
                cost[y][x] = (V + 1) * int(W[y, x]) + (0 if y == 0 else 1)
    parent = _edmonds(cost, 0)
    r = np.asarray(parent, dtype=np.int64)
    r[0] = -1
    return r


def _edmonds(cost, root):
    """Minimum arborescence of a dense digraph; cost[y][x] = inf means no edge.
    Returns parent[] (parent[root] = root).  Recursive contraction."""
    V = len(cost)
    INF = float("inf")
    best = [root] * V
    for x in range(V):
        if x == root:
            continue
        by = min((y for y in range(V) if y != x), key=lambda y: (cost[y][x], y))
        if cost[by][x] == INF:
            raise ValueError("vertex unreachable from the root")
        best[x] = by
    # look for a cycle among the chosen in-edges
    color = [0] * V
    cycle = None
    for s in range(V):
        if color[s]:
            continue
        path, v = [], s
        while v != root and color[v] == 0:
            color[v] = 1
            path.append(v)
            v = best[v]
        if v != root and color[v] == 1:
            cycle = path[path.index(v):]
        for p in path:
            color[p] = 2
        if cycle:
            break
    if cycle is None:
        return best
    incycle = set(cycle)
    others = [v for v in range(V) if v not in incycle]
    newid = {v: i for i, v in enumerate(others)}
    c = len(others)  # the contracted vertex
    ncost = [[INF] * (c + 1) for _ in range(c + 1)]
    enter = {}  # (outside y) -> cycle vertex its edge into c really enters
    leave = {}  # (outside x) -> cycle vertex the edge from c really leaves
    for y in others:
        for x in others:
            if y != x:
                ncost[newid[y]][newid[x]] = cost[y][x]
        bx, bc = None, INF
        for x in cycle:  # entering the cycle at x drops x's chosen in-edge
            if cost[y][x] < INF:
                red = cost[y][x] - cost[best[x]][x]
                if red < bc:
                    bx, bc = x, red
        if bx is not None:
            ncost[newid[y]][c] = bc
            enter[y] = bx
        bx, bc = None, INF
        for x in cycle:
            if cost[x][y] < bc:
                bx, bc = x, cost[x][y]
        if bx is not None:
            ncost[c][newid[y]] = bc
            leave[y] = bx
    sub = _edmonds(ncost, newid[root])
    parent = list(best)  # cycle edges stay, except the one displaced below
    for x in others:
        if x == root:
            continue
        p = sub[newid[x]]
        parent[x] = leave[x] if p == c else others[p]
    y = others[sub[c]]
    parent[enter[y]] = y
    parent[root] = root
    return parent


def topological_order(r: np.ndarray) -> list:
    """Vertices 1..m, every vertex after the vertex it is compressed against."""
    V = len(r)
    children = [[] for _ in range(V)]
    for x in range(1, V):
        children[int(r[x])].append(x)
    order, frontier = [], [0]
    while frontier:
        nxt = []
        for y in frontier:
            for x in children[y]:
                order.append(x)
                nxt.append(x)
        frontier = nxt
    if len(order) != V - 1:
        raise ValueError("not a tree rooted at the virtual vertex")
    return order


def delta_lists(rows: list, r: np.ndarray):
    """Delta+ = a_x \\ a_y and Delta- = a_y \\ a_x for every tree edge (y,x) = (r_x, x)
    (Eq. (2)); sorted lists, index 0 unused."""
    V = len(rows)
    dplus = [[] for _ in range(V)]
    dminus = [[] for _ in range(V)]
    for x in topological_order(r):
        y = int(r[x])
        dplus[x] = sorted(rows[x] - rows[y])
        dminus[x] = sorted(rows[y] - rows[x])
    return dplus, dminus


def decompress(r: np.ndarray, dplus: list, dminus: list) -> list:
    """Rebuild every row from its parent: a_x = (a_y u Delta+) \\ Delta- (Eq. (2))."""
    V = len(r)
    rows = [None] * V
    rows[0] = frozenset()
    for x in topological_order(r):
        rows[x] = frozenset((set(rows[int(r[x])]) | set(dplus[x])) - set(dminus[x]))
    return rows


def cbm_matmul(r: np.ndarray, dplus: list, dminus: list, B: np.ndarray) -> np.ndarray:
    """Algorithm 1: for every tree edge (y,x) in topological order and every
    column k, C[x,k] = C[y,k] + Delta+ . b_k - Delta- . b_k, where the null row's
    product is zero.  All p columns are processed and C is pure output (the
    printed loop bound and the listing of C as an input are read as typos)."""
    V = len(r)
    p = B.shape[1]
    C = np.zeros((V, p), dtype=np.float64)  # row 0 belongs to the null row
    Bd = B.astype(np.float64)
    for x in topological_order(r):
        y = int(r[x])
        for k in range(p):
            acc = C[y, k]
            for j in dplus[x]:
                acc += Bd[j, k]
            for j in dminus[x]:
                acc -= Bd[j, k]
            C[x, k] = acc
    return C[1:]


def cbm_matmul_two_stage(r, dplus, dminus, B: np.ndarray, n: int) -> np.ndarray:
    """The two-stage form (Section 2.2, "Leveraging High Performance SpMM
    kernels"): C := A'.B with the delta matrix A' (+1 on Delta+, -1 on Delta-),
    then c_x := c_x + c_y along the tree in topological order."""
    V = len(r)
    Ap = np.zeros((V, n), dtype=np.float64)
    for x in range(1, V):
        for j in dplus[x]:
            Ap[x, j] = 1.0
        for j in dminus[x]:
            Ap[x, j] = -1.0
    C = Ap @ B.astype(np.float64)
    for x in topological_order(r):
        C[x] = C[x] + C[int(r[x])]
    return C[1:]


def cbm_matmul_normalized(r, dplus, dminus, d: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Normalised extension (Section 2.2, "Extending SpMM with CBM ..."): the CBM
    is that of A v I; each delta on column j carries weight d_j^-1/2 (the
    column-scaled matrix (A + I) D^-1/2); rows are scaled by d_x^-1/2 in the update
    step.  Reading taken: a row's scale is applied only after its children have
    read its unscaled sum, so scaling is done last here."""
    V = len(r)
    s = 1.0 / np.sqrt(np.asarray(d, dtype=np.float64))
    Bd = B.astype(np.float64)
    C = np.zeros((V, B.shape[1]), dtype=np.float64)
    for x in topological_order(r):
        acc = C[int(r[x])].copy()
        for j in dplus[x]:
            acc += s[j] * Bd[j]
        for j in dminus[x]:
            acc -= s[j] * Bd[j]
        C[x] = acc
    return s[:, None] * C[1:]


def scalar_ops(rows: list, r: np.ndarray, dplus: list, dminus: list) -> np.ndarray:
    """Scalar operations per row of a matrix-vector product (Section 2.2, text
    after Eq. (5)): nnz(a_x) for a row stored in full, 1 + |Delta+| + |Delta-| for a
    compressed one.  Index 0 unused."""
    V = len(r)
    ops = np.zeros(V, dtype=np.int64)
    for x in range(1, V):
        ops[x] = len(rows[x]) if r[x] == 0 else 1 + len(dplus[x]) + len(dminus[x])
    return ops


def build_cbm(m: int, rowptr, colidx, alpha: int = 0, add_self_loops: bool = False):
    """Whole construction: distance graph -> pruning -> MST (alpha = 0) or MCA
    (alpha > 0) -> delta lists.  Returns (rows, r, dplus, dminus)."""
    rows = adjacency_lists(m, rowptr, colidx, add_self_loops)
    W = hamming_distance_graph(rows)
    if alpha == 0:
        r = mst_rooted_at_virtual(W)
    else:
        r = mca_rooted_at_virtual(W, admissible_edges(W, alpha))
    dplus, dminus = delta_lists(rows, r)
    return rows, r, dplus, dminus


# --------------------------------------------------------------------------- #
# O4: two-layer GCN inference (Eq. (1))
# --------------------------------------------------------------------------- #


def gcn2(rowptr, colidx, X, W0, W1) -> np.ndarray:
    """A_hat . relu(A_hat . X . W0) . W1 evaluated as Z0 = X W0, H = relu(A_hat Z0),
    Z1 = H W1, out = A_hat Z1 (sigma = ReLU, no bias: Eq. (1) has none)."""
    d = degrees_with_self_loops(rowptr, colidx)
    Z0 = X.astype(np.float64) @ W0.astype(np.float64)
    H = np.maximum(spmm_csr_normalized(rowptr, colidx, Z0, d=d), 0.0)
    Z1 = H @ W1.astype(np.float64)
    return spmm_csr_normalized(rowptr, colidx, Z1, d=d)
