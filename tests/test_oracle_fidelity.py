"""Pins for the oracle's top-k selection and fidelity scores (the paper's evaluation metrics)."""
import numpy as np
import pytest

from oracle import compgraph, fidelity, gcn
from synth import make_workload


def test_top_k_order_and_ties():
    phi = np.array([0.1, 0.5, 0.5, -0.2, 0.0, 0.5], dtype=np.float32)
    assert list(fidelity.top_k_players(phi, 0)) == []
    assert list(fidelity.top_k_players(phi, 2)) == [1, 2]           # ties -> lower index first
    assert list(fidelity.top_k_players(phi, 4)) == [1, 2, 5, 0]
    assert list(fidelity.top_k_players(phi, 99)) == [1, 2, 5, 0, 4, 3]
    m = fidelity.top_k_masks(phi, [2])
    assert list(np.flatnonzero(m[0])) == [1, 2] and list(np.flatnonzero(m[1])) == [0, 3, 4, 5]


def test_fidelity_special_cases_follow_the_definitions():
    w = make_workload("c1")
    cg = compgraph.extract(w.row_ptr, w.col, 0, 2)
    f = gcn.ValueFunction(cg, w.features, w.weights, dense=True)
    n = cg["num_players"]
    phi = np.random.default_rng(0).standard_normal(n).astype(np.float32)
    full, empty = f(np.ones(n, bool)), f(np.zeros(n, bool))
    plus, minus = fidelity.fidelity(f, phi, [0, n, 3])
    # G_s empty: nothing removed / nothing kept;  G_s = G_c: everything removed / everything kept
    assert plus[0] == 0.0 and minus[0] == pytest.approx(abs(full - empty))
    assert plus[1] == pytest.approx(abs(full - empty)) and minus[1] == 0.0
    top3 = fidelity.top_k_players(phi, 3)
    keep = np.zeros(n, bool)
    keep[top3] = True
    assert plus[2] == pytest.approx(abs(full - f(~keep))) and minus[2] == pytest.approx(abs(full - f(keep)))


def test_exact_shapley_ranking_finds_the_decisive_edge():
    # path target(0) - 1 - 2 plus a pendant 3 on node 0 whose features are zero: with a 1-layer model
    # only the edges at the target matter, and the edge to the feature-carrying neighbour dominates
    from oracle import shapley
    from synth import csr_from_undirected_edges
    rp, ci = csr_from_undirected_edges(4, [0, 1, 0], [1, 2, 3])
    X = np.zeros((4, 3))
    X[1] = [3.0, -1.0, 2.0]
    W = [np.eye(3)]
    cg = compgraph.extract(rp, ci, 0, 2)
    f = gcn.ValueFunction(cg, X, W, score="logit", dense=True)
    n = cg["num_players"]
    phi = shapley.exact_shapley(shapley.all_values(f, n), n)
    pairs = list(zip(cg["edge_src"], cg["edge_dst"]))
    assert fidelity.top_k_players(phi, 1)[0] == pairs.index((0, 1))
    plus, minus = fidelity.fidelity(f, phi, [1])
    assert plus[0] == pytest.approx(abs(f(np.ones(n, bool)) - 0.0))   # without (0,1) the target sees only zeros
