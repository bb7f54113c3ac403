"""Graph generators and plain graph statistics used to choose target nodes.

All graphs are returned as a symmetric CSR (row i lists the neighbours of i,
ascending, no duplicates, no self-loops): row_ptr int64[N+1], col int32[nnz].
"""
import numpy as np


def csr_from_undirected_edges(num_nodes, src, dst):
    """Symmetrise, drop self-loops, de-duplicate, sort rows."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    a = np.concatenate([src, dst])
    b = np.concatenate([dst, src])
    code = np.unique(a * np.int64(num_nodes) + b)
    rows = code // num_nodes
    cols = (code % num_nodes).astype(np.int32)
    counts = np.bincount(rows, minlength=num_nodes)
    row_ptr = np.zeros(num_nodes + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, cols


def tiny_graph():
    """8 nodes, 12 undirected edges, every node within two hops of node 0."""
    edges = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 4), (1, 5), (2, 5), (2, 6),
             (3, 6), (3, 7), (4, 5), (6, 7)]
    s, d = zip(*edges)
    return (8,) + csr_from_undirected_edges(8, s, d)


def barabasi_albert(num_nodes, m, rng):
    """Preferential attachment: each new node attaches to m distinct earlier
    nodes chosen with probability proportional to degree."""
    targets = list(range(m))
    repeated = []
    src, dst = [], []
    for v in range(m, num_nodes):
        src.extend([v] * m)
        dst.extend(targets)
        repeated.extend(targets)
        repeated.extend([v] * m)
        chosen = set()
        while len(chosen) < m:
            chosen.add(repeated[int(rng.integers(len(repeated)))])
        targets = sorted(chosen)
    return (num_nodes,) + csr_from_undirected_edges(num_nodes, src, dst)


def rmat(scale, edge_factor, rng, a=0.57, b=0.19, c=0.19):
    """Recursive-matrix generator, cleaned Graph500-style (symmetrised,
    self-loops dropped, duplicates merged)."""
    num_nodes = 1 << scale
    m = edge_factor * num_nodes
    src = np.zeros(m, dtype=np.int64)
    dst = np.zeros(m, dtype=np.int64)
    ab, abc = a + b, a + b + c
    for _ in range(scale):
        u = rng.random(m)
        src = (src << 1) | (u >= ab)
        dst = (dst << 1) | (((u >= a) & (u < ab)) | (u >= abc))
    return (num_nodes,) + csr_from_undirected_edges(num_nodes, src, dst)


def khop_ball(row_ptr, col, v, hops):
    """Nodes within `hops` hops of v (boolean membership array, ball sizes)."""
    n = len(row_ptr) - 1
    inside = np.zeros(n, dtype=bool)
    inside[v] = True
    frontier = np.array([v], dtype=np.int64)
    sizes = [1]
    for _ in range(hops):
        if len(frontier) == 0:
            sizes.append(sizes[-1])
            continue
        starts, ends = row_ptr[frontier], row_ptr[frontier + 1]
        lens = ends - starts
        idx = np.repeat(starts - np.cumsum(np.r_[0, lens[:-1]]), lens) + np.arange(lens.sum())
        nb = np.unique(col[idx])
        nb = nb[~inside[nb]]
        inside[nb] = True
        frontier = nb.astype(np.int64)
        sizes.append(int(inside.sum()))
    return inside, sizes


def induced_undirected_edge_count(row_ptr, col, inside):
    """Number of unordered node pairs joined by an edge with both ends inside."""
    nodes = np.flatnonzero(inside)
    starts, ends = row_ptr[nodes], row_ptr[nodes + 1]
    lens = ends - starts
    if lens.sum() == 0:
        return 0
    idx = np.repeat(starts - np.cumsum(np.r_[0, lens[:-1]]), lens) + np.arange(lens.sum())
    return int(inside[col[idx]].sum()) // 2


def fanout_capped_subgraph(row_ptr, col, root, fans):
    """Neighbourhood sampling with a deterministic fan-out cap: from `root`, hop h keeps, for every node
    reached at hop h-1, its first fans[h-1] neighbours in CSR order. Returns the graph made of exactly the
    kept edges (symmetrised, nodes renumbered in ascending order of their old ids) and the root's new id."""
    src_all, dst_all = [], []
    seen = np.zeros(len(row_ptr) - 1, dtype=bool)
    seen[root] = True
    frontier = np.array([root], dtype=np.int64)
    for f in fans:
        if len(frontier) == 0:
            break
        starts = row_ptr[frontier]
        lens = np.minimum(row_ptr[frontier + 1] - starts, f)
        idx = np.repeat(starts - np.cumsum(np.r_[0, lens[:-1]]), lens) + np.arange(lens.sum())
        nb = col[idx].astype(np.int64)
        src_all.append(np.repeat(frontier, lens))
        dst_all.append(nb)
        new = np.unique(nb)
        new = new[~seen[new]]
        seen[new] = True
        frontier = new
    src = np.concatenate(src_all)
    dst = np.concatenate(dst_all)
    nodes = np.flatnonzero(seen)
    num = len(nodes)
    rp, ci = csr_from_undirected_edges(num, np.searchsorted(nodes, src), np.searchsorted(nodes, dst))
    return num, rp, ci, int(np.searchsorted(nodes, root))
