"""Top-k explanation sub-graph and the two fidelity scores of the paper's evaluation section:
  Fidelity+ = | f(G_c) - f(G_c \\ G_s) |      (drop the k most important edges)
  Fidelity- = | f(G_c) - f(G_s) |            (keep only the k most important edges)
where G_s holds the k edges with the largest Shapley values (step 5 of the overview: rank and
select). Ranking is by descending phi, ties broken by the lower player index."""
import numpy as np


def top_k_players(phi, k):
    phi = np.asarray(phi)
    order = np.lexsort((np.arange(len(phi)), -phi.astype(np.float64)))
    return order[:max(0, min(int(k), len(phi)))]


def top_k_masks(phi, ks):
    """bool[2*len(ks), n]: row 2t = G_s for ks[t], row 2t+1 = G_c without G_s."""
    n = len(phi)
    out = np.zeros((2 * len(ks), n), dtype=bool)
    for t, k in enumerate(ks):
        out[2 * t, top_k_players(phi, k)] = True
        out[2 * t + 1] = ~out[2 * t]
    return out


def fidelity(f, phi, ks):
    """f: oracle.gcn.ValueFunction. Returns (fid_plus[len(ks)], fid_minus[len(ks)])."""
    n = len(phi)
    full = f(np.ones(n, dtype=bool))
    masks = top_k_masks(phi, ks)
    plus = np.array([abs(full - f(masks[2 * t + 1])) for t in range(len(ks))])
    minus = np.array([abs(full - f(masks[2 * t])) for t in range(len(ks))])
    return plus, minus
