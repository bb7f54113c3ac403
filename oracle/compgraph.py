"""Computational graph of a target node and the players of the game.

The computational graph is the target's 1..L-hop neighbourhood and the edges
among those nodes (paper, background section on GNNs); the players of the game
are its edges (overview, step 1).  Row i of the input CSR lists the
in-neighbours of i (messages flow j -> i), so the neighbourhood is grown along
rows.  Self-loop entries are never players.

Local node order: ascending (hop distance, global id).  Player order:
undirected - unordered pairs {a < b} ascending by (a, b) in global ids;
directed - entries (dst, src) ascending by (dst, src).
"""
import numpy as np


def extract(row_ptr, col, target, hops, undirected=True):
    N = len(row_ptr) - 1
    dist = np.full(N, -1, dtype=np.int64)
    dist[target] = 0
    frontier = [int(target)]
    for h in range(1, hops + 1):
        nxt = []
        for i in frontier:
            for j in col[row_ptr[i]:row_ptr[i + 1]]:
                j = int(j)
                if dist[j] < 0:
                    dist[j] = h
                    nxt.append(j)
        frontier = nxt
    members = np.flatnonzero(dist >= 0)
    order = np.lexsort((members, dist[members]))
    node_gid = members[order].astype(np.int64)
    hop = dist[node_gid].astype(np.int64)
    local = np.full(N, -1, dtype=np.int64)
    local[node_gid] = np.arange(len(node_gid))
    ball = [int((hop <= h).sum()) for h in range(hops + 1)]

    psrc, pdst = [], []
    for a in members:                        # ascending global id
        a = int(a)
        row = col[row_ptr[a]:row_ptr[a + 1]]
        for b in row:                        # rows are sorted ascending
            b = int(b)
            if b == a or dist[b] < 0:
                continue
            if undirected:
                if b > a:
                    back = col[row_ptr[b]:row_ptr[b + 1]]
                    if a not in back:
                        raise ValueError("CSR is not symmetric: undirected players need both directions")
                    psrc.append(a)
                    pdst.append(b)
                else:
                    back = col[row_ptr[b]:row_ptr[b + 1]]
                    if a not in back:
                        raise ValueError("CSR is not symmetric: undirected players need both directions")
            else:
                psrc.append(b)               # message b -> a
                pdst.append(a)
    psrc = np.asarray(psrc, dtype=np.int64)
    pdst = np.asarray(pdst, dtype=np.int64)
    return {
        "target": int(target), "hops": hops, "undirected": undirected,
        "node_gid": node_gid, "hop": hop, "ball": ball,
        "num_nodes": len(node_gid), "num_players": len(psrc),
        "edge_src": psrc, "edge_dst": pdst,           # global ids, player order
        "lsrc": local[psrc] if len(psrc) else psrc,   # local ids
        "ldst": local[pdst] if len(pdst) else pdst,
        "target_local": 0,
    }
