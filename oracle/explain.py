"""End-to-end explanation by the oracle: computational graph -> sampled
coalitions -> GCN value of every coalition -> constrained weighted least
squares -> one score per edge (the five steps of the paper's overview)."""
import numpy as np

from . import compgraph, gat as gat_model, gcn, sampling, solve


def explain(row_ptr, col, X, weights, target, n_samples, seed, biases=None,
            hops=None, undirected=True, score="prob", solver="lstsq",
            tol=1e-10, max_iter=None, dense_adjacency=False, bf16=False, gat=None, weighting="class",
            saturate=False):
    """`gat`: a model dictionary for oracle.gat (then `weights`/`biases` are ignored); otherwise a GCN."""
    L = len(gat["W"]) if gat is not None else len(weights)
    hops = L if hops is None or hops == 0 else hops
    cg = compgraph.extract(row_ptr, col, target, hops, undirected)
    n = cg["num_players"]
    out = {"cg": cg, "n": n}
    if n == 0:
        out.update(phi=np.zeros(0), k=0)
        return out
    if gat is not None:
        f = gat_model.ValueFunction(cg, X, gat, score)
    else:
        f = gcn.ValueFunction(cg, X, weights, biases, score, dense=dense_adjacency, bf16=bf16)
    if n == 1:
        f0, f1 = f(np.zeros(1, bool)), f(np.ones(1, bool))
        out.update(phi=np.array([f1 - f0]), k=2, y=np.array([f0, f1]), pred_class=f.pred_class)
        return out
    if n_samples < 4:
        raise ValueError("n_samples must be at least 4")
    Z, w, sz = sampling.sample(n, n_samples, seed, int(target) & 0xFFFFFFFF, weighting=weighting, saturate=saturate)
    bits = sampling.unpack_rows(Z, n)
    y = f.batch(bits)
    if solver == "lstsq":
        phi = solve.solve_lstsq(bits, w, y)
        it, rel = 0, 0.0
    elif solver == "kkt":
        phi = solve.solve_kkt(bits, w, y)
        it, rel = 0, 0.0
    else:
        phi, it, rel = solve.solve_cgls(bits, w, y, tol=tol, max_iter=max_iter)
    out.update(phi=phi, k=len(w), Z=Z, w=w, sz=sz, y=y, pred_class=f.pred_class,
               iterations=it, rel_residual=rel)
    return out
