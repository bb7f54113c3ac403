"""Pins for the oracle's computational graph, GCN value function, exact Shapley
values and the equality of enumerated Kernel-SHAP with them."""
import numpy as np
import pytest

from oracle import compgraph, explain, gcn, sampling, shapley, solve
from synth import csr_from_undirected_edges, make_workload


def _graph(n, edges):
    s, d = zip(*edges)
    return csr_from_undirected_edges(n, s, d)


def test_extraction_order_players_and_balls():
    w = make_workload("c1")
    cg = compgraph.extract(w.row_ptr, w.col, 0, 2)
    assert cg["ball"] == [1, 4, 8]
    assert list(cg["node_gid"]) == [0, 1, 2, 3, 4, 5, 6, 7]
    assert list(cg["hop"]) == [0, 1, 1, 1, 2, 2, 2, 2]
    pairs = list(zip(cg["edge_src"], cg["edge_dst"]))
    assert pairs == [(0, 1), (0, 2), (0, 3), (1, 2), (1, 4), (1, 5), (2, 5), (2, 6),
                     (3, 6), (3, 7), (4, 5), (6, 7)]
    one_hop = compgraph.extract(w.row_ptr, w.col, 0, 1)
    assert one_hop["ball"] == [1, 4]
    assert list(zip(one_hop["edge_src"], one_hop["edge_dst"])) == [(0, 1), (0, 2), (0, 3), (1, 2)]
    directed = compgraph.extract(w.row_ptr, w.col, 0, 1, undirected=False)
    got = list(zip(directed["edge_dst"], directed["edge_src"]))
    assert got == sorted(got) and len(got) == 8


def test_extraction_local_order_is_hop_then_global_id():
    rp, ci = _graph(7, [(6, 0), (6, 3), (0, 5), (3, 1), (5, 2), (1, 2)])
    cg = compgraph.extract(rp, ci, 6, 2)
    assert list(cg["node_gid"]) == [6, 0, 3, 1, 5]
    assert list(cg["hop"]) == [0, 1, 1, 2, 2]
    assert list(zip(cg["edge_src"], cg["edge_dst"])) == [(0, 5), (0, 6), (1, 3), (3, 6)]


def test_asymmetric_csr_is_rejected_for_undirected_players():
    row_ptr = np.array([0, 1, 1], dtype=np.int64)
    col = np.array([1], dtype=np.int32)
    with pytest.raises(ValueError):
        compgraph.extract(row_ptr, col, 0, 1)
    cg = compgraph.extract(row_ptr, col, 0, 1, undirected=False)
    assert cg["num_players"] == 1


def test_symmetric_normalisation_hand_example():
    # path a-b-c, one layer, W = [1]: out_a = x_a/2 + x_b/sqrt(2*3)
    rp, ci = _graph(3, [(0, 1), (1, 2)])
    cg = compgraph.extract(rp, ci, 0, 2)
    X = np.array([[1.0], [2.0], [4.0]])
    A = gcn.adjacency_dense(cg, np.ones(2, bool))
    out = gcn.forward(A, X, [np.array([[1.0]])])
    assert out[0, 0] == pytest.approx(1 / 2 + 2 / np.sqrt(6))
    assert out[1, 0] == pytest.approx(1 / np.sqrt(6) + 2 / 3 + 4 / np.sqrt(6))
    # dropping edge (b, c) renormalises b: d_b = 2
    A = gcn.adjacency_dense(cg, np.array([True, False]))
    out = gcn.forward(A, X, [np.array([[1.0]])])
    assert out[0, 0] == pytest.approx(1 / 2 + 2 / 2)
    assert out[2, 0] == pytest.approx(4.0)


def test_empty_coalition_is_a_plain_mlp_on_the_target():
    w = make_workload("c2_small")
    cg = compgraph.extract(w.row_ptr, w.col, w.targets[0], 3)
    f = gcn.ValueFunction(cg, w.features, w.weights)
    h = w.features[w.targets[0]].astype(np.float64)
    for l, W in enumerate(w.weights):
        h = h @ W.astype(np.float64)
        if l < len(w.weights) - 1:
            h = np.maximum(h, 0)
    assert np.allclose(f.logits(np.zeros(cg["num_players"], bool)), h, rtol=1e-12, atol=1e-12)


def test_regular_graph_full_coalition_is_mean_aggregation():
    n = 9
    rp, ci = _graph(n, [(i, (i + 1) % n) for i in range(n)])
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, 5))
    W = [rng.standard_normal((5, 4))]
    cg = compgraph.extract(rp, ci, 0, 4)
    assert cg["num_nodes"] == n and cg["num_players"] == n
    f = gcn.ValueFunction(cg, X, W)
    expect = ((X[0] + X[1] + X[n - 1]) / 3.0) @ W[0]
    assert np.allclose(f.logits(np.ones(n, bool)), expect)


def test_dense_and_sparse_adjacency_agree():
    w = make_workload("c2_small")
    cg = compgraph.extract(w.row_ptr, w.col, w.targets[0], 3)
    fd = gcn.ValueFunction(cg, w.features, w.weights, dense=True)
    fs = gcn.ValueFunction(cg, w.features, w.weights, dense=False)
    rng = np.random.default_rng(0)
    for _ in range(5):
        m = rng.random(cg["num_players"]) < rng.random()
        assert fd(m) == pytest.approx(fs(m), rel=1e-12, abs=1e-14)
    # directed players
    cgd = compgraph.extract(w.row_ptr, w.col, w.targets[0], 2, undirected=False)
    fd = gcn.ValueFunction(cgd, w.features, w.weights[:2], dense=True)
    fs = gcn.ValueFunction(cgd, w.features, w.weights[:2], dense=False)
    m = rng.random(cgd["num_players"]) < 0.5
    assert fd(m) == pytest.approx(fs(m), rel=1e-12)


def test_relabelling_nodes_leaves_the_value_unchanged():
    w = make_workload("c1")
    rng = np.random.default_rng(5)
    perm = rng.permutation(8)                  # new id of old node i
    cg = compgraph.extract(w.row_ptr, w.col, 0, 2)
    olds, oldd = cg["edge_src"], cg["edge_dst"]
    rp2, ci2 = csr_from_undirected_edges(8, perm[olds], perm[oldd])
    X2 = np.empty_like(w.features)
    X2[perm] = w.features
    cg2 = compgraph.extract(rp2, ci2, int(perm[0]), 2)
    f1 = gcn.ValueFunction(cg, w.features, w.weights)
    f2 = gcn.ValueFunction(cg2, X2, w.weights)
    key2 = {(min(a, b), max(a, b)): j for j, (a, b) in enumerate(zip(cg2["edge_src"], cg2["edge_dst"]))}
    for _ in range(6):
        m1 = rng.random(12) < 0.5
        m2 = np.zeros(12, bool)
        for j in np.flatnonzero(m1):
            a, b = int(perm[olds[j]]), int(perm[oldd[j]])
            m2[key2[(min(a, b), max(a, b))]] = True
        assert f1(m1) == pytest.approx(f2(m2), rel=1e-12)


def test_exact_shapley_linear_game_and_efficiency():
    rng = np.random.default_rng(1)
    n = 7
    a = rng.standard_normal(n)
    vals = shapley.all_values(lambda m: 0.3 + a[m].sum(), n)
    assert np.allclose(shapley.exact_shapley(vals, n), a)
    vals = rng.standard_normal(1 << n)
    phi = shapley.exact_shapley(vals, n)
    assert phi.sum() == pytest.approx(vals[-1] - vals[0])


def test_exact_shapley_two_player_hand_example():
    # f(00)=0, f(01)=1 (player 0), f(10)=3 (player 1), f(11)=10
    vals = np.array([0.0, 1.0, 3.0, 10.0])
    phi = shapley.exact_shapley(vals, 2)
    assert phi[0] == pytest.approx(0.5 * (1 - 0) + 0.5 * (10 - 3))
    assert phi[1] == pytest.approx(0.5 * (3 - 0) + 0.5 * (10 - 1))


def test_null_players_outside_the_receptive_field():
    # 2-layer model, graph extracted to 3 hops: edge (3,4) joins two nodes at
    # distance 3, so it cannot influence the target; edge (2,3) changes the
    # degree of node 2 (distance 2), which does.
    rp, ci = _graph(5, [(0, 1), (1, 2), (2, 3), (2, 4), (3, 4)])
    rng = np.random.default_rng(2)
    X = rng.standard_normal((5, 6))
    W = [rng.standard_normal((6, 5)), rng.standard_normal((5, 3))]
    cg = compgraph.extract(rp, ci, 0, 3)
    f = gcn.ValueFunction(cg, X, W, dense=True)
    n = cg["num_players"]
    phi = shapley.exact_shapley(shapley.all_values(f, n), n)
    pairs = list(zip(cg["edge_src"], cg["edge_dst"]))
    assert phi[pairs.index((3, 4))] == 0.0
    assert abs(phi[pairs.index((2, 3))]) > 1e-6
    # Kernel-SHAP under enumeration reproduces the zero
    out = explain.explain(rp, ci, X, W, 0, 1 << n, 1, hops=3)
    assert abs(out["phi"][pairs.index((3, 4))]) < 1e-9      # fp32-stored weights


def test_symmetric_players_get_equal_values():
    # star around the target with identical leaf features: all edges are interchangeable
    rp, ci = _graph(6, [(0, i) for i in range(1, 6)])
    rng = np.random.default_rng(4)
    X = np.tile(rng.standard_normal((1, 4)), (6, 1))
    X[0] = rng.standard_normal(4)
    W = [rng.standard_normal((4, 4)), rng.standard_normal((4, 3))]
    cg = compgraph.extract(rp, ci, 0, 2)
    f = gcn.ValueFunction(cg, X, W, dense=True)
    phi = shapley.exact_shapley(shapley.all_values(f, 5), 5)
    assert np.allclose(phi, phi[0], rtol=1e-12, atol=1e-15)
    out = explain.explain(rp, ci, X, W, 0, 32, 1)
    assert np.allclose(out["phi"], phi[0], rtol=1e-9)


def test_enumerated_kernel_shap_equals_exact_shapley_on_the_tiny_config():
    w = make_workload("c1")
    out = explain.explain(w.row_ptr, w.col, w.features, w.weights, 0, w.n_samples, w.seed)
    assert out["n"] == 12 and out["k"] == 4096
    f = gcn.ValueFunction(out["cg"], w.features, w.weights, dense=True)
    exact = shapley.exact_shapley(shapley.all_values(f, 12), 12)
    # weights are stored in fp32, which bounds the agreement
    assert np.abs(out["phi"] - exact).max() < 1e-8
    assert out["phi"].sum() == pytest.approx(out["y"][1] - out["y"][0], abs=1e-14)
    for solver in ("kkt", "cgls"):
        o2 = explain.explain(w.row_ptr, w.col, w.features, w.weights, 0, w.n_samples, w.seed, solver=solver)
        assert np.abs(o2["phi"] - exact).max() < 1e-8


@pytest.mark.parametrize("score", ["prob", "logit"])
def test_enumerated_kernel_shap_equals_exact_shapley_random_graphs(score):
    rng = np.random.default_rng(11)
    for trial in range(3):
        nn = 6
        edges = set()
        while len(edges) < 8:
            a, b = rng.integers(nn, size=2)
            if a != b:
                edges.add((min(a, b), max(a, b)))
        rp, ci = _graph(nn, sorted(edges))
        X = rng.standard_normal((nn, 5))
        W = [rng.standard_normal((5, 4)), rng.standard_normal((4, 3))]
        b = [rng.standard_normal(4), rng.standard_normal(3)]
        out = explain.explain(rp, ci, X, W, 0, 1 << 10, trial, biases=b, score=score)
        n = out["n"]
        if n < 2:
            continue
        f = gcn.ValueFunction(out["cg"], X, W, b, score=score, dense=True)
        exact = shapley.exact_shapley(shapley.all_values(f, n), n)
        assert np.abs(out["phi"] - exact).max() < 1e-8


def test_directed_players_enumerated_kernel_shap_equals_exact():
    w = make_workload("c1")
    out = explain.explain(w.row_ptr, w.col, w.features, w.weights, 0, 1 << 8, 3, hops=1, undirected=False)
    n = out["n"]
    assert n == 8
    f = gcn.ValueFunction(out["cg"], w.features, w.weights, dense=True)
    exact = shapley.exact_shapley(shapley.all_values(f, n), n)
    assert np.abs(out["phi"] - exact).max() < 1e-8


def test_sampled_estimate_approaches_exact_shapley():
    w = make_workload("c1")
    cg = compgraph.extract(w.row_ptr, w.col, 0, 2)
    f = gcn.ValueFunction(cg, w.features, w.weights, dense=True)
    vals = shapley.all_values(f, 12)
    exact = shapley.exact_shapley(vals, 12)
    errs = []
    for ns in (64, 1024):
        e = []
        for seed in range(6):
            Z, wt, sz = sampling.sample(12, ns, seed, 0)
            bits = sampling.unpack_rows(Z, 12)
            idx = (bits.astype(np.int64) << np.arange(12)).sum(axis=1)
            phi = solve.solve_lstsq(bits, wt, vals[idx])
            assert phi.sum() == pytest.approx(vals[-1] - vals[0], abs=1e-12)
            e.append(np.abs(phi - exact).max())
        errs.append(np.mean(e))
    assert errs[1] < 0.5 * errs[0]
    assert errs[1] < 0.05 * np.abs(exact).max() + 1e-3


def test_uniform_weighting_is_the_importance_sampling_form_of_the_same_estimator():
    """weighting="uniform": rows are already allocated in proportion to rho_s, so weight 1 per row is the
    importance-sampling estimator. Pins: the allocation is untouched and the table is 1 on every class
    that has rows; a linear game is still recovered exactly; the estimate approaches exact Shapley at
    the same rate as the default; enumerated plans keep the exact kernel weights."""
    a = sampling.allocation(30, 2000)
    u = sampling.allocation(30, 2000, "uniform")
    assert np.array_equal(a["b"], u["b"])
    has_rows = np.diff(u["b"], prepend=0)[1:] > 0
    assert np.array_equal(u["wtab"][1:], has_rows.astype(np.float32))
    # where the allocation is exact the default weight is the same constant T / (2K) for every class
    # (a pair class of mass 2 rho_s gets K 2 rho_s / T pairs, each with one row of size s; the middle class
    # of an even n has mass rho_s and two rows per pair): uniform
    # weights differ from it only by that common factor and by the rounding of the allocation
    K = a["K"]
    ratio = a["wtab"][1:][has_rows] * 2 * K / a["T"]
    q = np.diff(a["b"], prepend=0)[1:][has_rows]
    assert np.all(np.abs(ratio - 1.0) <= 1.2 / q + 1e-6)
    e = sampling.allocation(10, 1 << 10, "uniform")
    assert e["enumerate"] and np.array_equal(e["wtab"], sampling.allocation(10, 1 << 10)["wtab"])
    with pytest.raises(ValueError):
        sampling.allocation(30, 2000, "other")

    rng = np.random.default_rng(0)
    coef = rng.normal(size=14)
    Z, wt, sz = sampling.sample(14, 400, 3, 0, weighting="uniform")
    bits = sampling.unpack_rows(Z, 14)
    assert set(np.unique(wt[2:])) == {np.float32(1.0)} and wt[0] == 0 and wt[1] == 0
    phi = solve.solve_lstsq(bits, wt, 0.3 + bits @ coef)
    assert np.abs(phi - coef).max() < 1e-10

    w = make_workload("c1")
    cg = compgraph.extract(w.row_ptr, w.col, 0, 2)
    f = gcn.ValueFunction(cg, w.features, w.weights, dense=True)
    vals = shapley.all_values(f, 12)
    exact = shapley.exact_shapley(vals, 12)
    err = {}
    for mode in ("class", "uniform"):
        for ns in (64, 1024):
            e = []
            for seed in range(6):
                Z, wt, sz = sampling.sample(12, ns, seed, 0, weighting=mode)
                bits = sampling.unpack_rows(Z, 12)
                idx = (bits.astype(np.int64) << np.arange(12)).sum(axis=1)
                e.append(np.abs(solve.solve_lstsq(bits, wt, vals[idx]) - exact).max())
            err[mode, ns] = np.mean(e)
    assert err["uniform", 1024] < 0.5 * err["uniform", 64]
    assert 0.5 < err["uniform", 1024] / err["class", 1024] < 2.0


def test_bf16_rounding_is_nearest_even():
    # bfloat16 keeps 8 significand bits: spacing 2^-7 in [1, 2)
    assert gcn.round_bf16(1.0) == 1.0
    assert gcn.round_bf16(1.0 + 2.0 ** -8) == 1.0                    # tie -> even
    assert gcn.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6    # tie -> even (up)
    assert gcn.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert gcn.round_bf16(-3.1415927) == -3.140625
    x = np.random.default_rng(0).standard_normal(1000)
    r = gcn.round_bf16(x)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8 * (1 + 1e-6))
    assert np.array_equal(gcn.round_bf16(r), r)


def test_bf16_mode_stays_close_to_full_precision():
    w = make_workload("c2_small")
    cg = compgraph.extract(w.row_ptr, w.col, w.targets[0], 3)
    f64 = gcn.ValueFunction(cg, w.features, w.weights)
    f16 = gcn.ValueFunction(cg, w.features, w.weights, bf16=True)
    rng = np.random.default_rng(1)
    for _ in range(4):
        m = rng.random(cg["num_players"]) < 0.5
        assert abs(f64(m) - f16(m)) < 2e-2
        assert f64(m) != f16(m)


def test_bf16_diagnostic_mode_operand_placement_hand_worked():
    """Two nodes joined by one edge, widths 1 -> 1 -> 1, X = (1, 2), W_1 = 1 + 2^-6 + 2^-8, W_2 = 3 + 2^-7 + 2^-12.
    Full coalition: A^ = [[1/2, 1/2], [1/2, 1/2]]. Layer 1 is NOT rounded: A^ X = 1.5 at both nodes,
    h = 1.5 * 1.01953125 = 1.529296875. Layer 2 rounds both operands: bfloat16 spacing is 2^-7 in [1, 2), so
    A^ H = h -> 1.53125 (0.00195 away; 1.5234375 is 0.00586 away); spacing 2^-6 in [2, 4), so
    W_2 = 3.00805664 -> 3.015625 (0.00757 away; 3.0 is 0.00806 away); logit = 1.53125 * 3.015625 = 4.61767578125.
    Rounding layer 1 as well would give 4.5941162109375, leaving the activations unrounded 4.611785888671875,
    leaving W_2 unrounded 4.606086730957031, no rounding 4.6002116203308105: each misplacement fails.
    Empty coalition: A^ = I, h = 1.01953125 = 1 + 2.5 * 2^-7, a tie that goes to the even neighbour 1.015625;
    logit = 1.015625 * 3.015625 = 3.062744140625."""
    from oracle import cfast
    row_ptr = np.array([0, 1, 2], dtype=np.int64)
    col = np.array([1, 0], dtype=np.int32)
    X = np.array([[1.0], [2.0]])
    weights = [np.array([[1.0 + 2.0 ** -6 + 2.0 ** -8]]), np.array([[3.0 + 2.0 ** -7 + 2.0 ** -12]])]
    cg = compgraph.extract(row_ptr, col, 0, 2)
    assert cg["num_players"] == 1 and cg["num_nodes"] == 2
    f = gcn.ValueFunction(cg, X, weights, score="logit", bf16=True)
    assert f(np.array([True])) == 4.61767578125
    assert f(np.array([False])) == 3.062744140625
    plain = gcn.ValueFunction(cg, X, weights, score="logit")
    assert abs(plain(np.array([True])) - 4.6002116203308105) < 1e-14
    Z = np.array([[1], [0]], dtype=np.uint64)
    y, _, _ = cfast.gcn_values(cg, X, weights, Z, score="logit", bf16=True)
    assert y[0] == 4.61767578125 and y[1] == 3.062744140625
