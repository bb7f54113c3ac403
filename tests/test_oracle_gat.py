"""Pins for the GAT value function of the oracle (oracle/gat.py).

The layer follows Velickovic et al. (the GAT the paper cites for its second model
family).  Each test fixes it to something other than its own formula:
  * no active edge        -> attention is 1 on the self term: a plain two-layer perceptron;
  * zero attention vectors -> uniform attention: the row-normalised (A + I) mean aggregation;
  * one neighbour, scalars -> the logistic closed form, worked by hand below;
  * attention asymmetry    -> exchanging the roles of a_src and a_dst must change the result
                              in the way the hand-worked case says;
  * relabelling the nodes leaves the value unchanged;
  * edges that cannot reach the target within L layers are exact null players (brute-force Shapley).
"""
import math

import numpy as np

from oracle import compgraph, gat, shapley
from synth import graphs


def _model(rng, d0, heads, widths, slope=0.2, bias=False):
    W, a_s, a_d, b = [], [], [], []
    din = d0
    L = len(heads)
    for l in range(L):
        W.append(rng.normal(size=(din, heads[l] * widths[l])) * 0.4)
        a_s.append(rng.normal(size=(heads[l], widths[l])) * 0.7)
        a_d.append(rng.normal(size=(heads[l], widths[l])) * 0.7)
        out = widths[l] if l == L - 1 else heads[l] * widths[l]
        b.append(rng.normal(size=out) * 0.1 if bias else None)
        din = heads[l] * widths[l]
    return dict(W=W, a_src=a_s, a_dst=a_d, bias=b if bias else None, heads=list(heads), slope=slope)


def _tiny_cg(hops=2):
    _, row_ptr, col = graphs.tiny_graph()
    return row_ptr, col, compgraph.extract(row_ptr, col, 0, hops, True)


def test_empty_coalition_is_a_perceptron():
    rng = np.random.default_rng(1)
    row_ptr, col, cg = _tiny_cg()
    X = rng.normal(size=(8, 5))
    m = _model(rng, 5, (3, 2), (4, 6), bias=True)
    f = gat.ValueFunction(cg, X, m, score="logit")
    z = f.logits(np.zeros(cg["num_players"], bool))
    x = X[cg["node_gid"][cg["target_local"]]]
    h = x @ m["W"][0] + m["bias"][0]
    h = np.where(h > 0, h, np.exp(np.minimum(h, 0)) - 1.0)
    o = (h @ m["W"][1]).reshape(2, 6).mean(axis=0) + m["bias"][1]
    assert np.allclose(z, o, rtol=0, atol=1e-13)


def test_zero_attention_is_mean_aggregation():
    rng = np.random.default_rng(2)
    row_ptr, col, cg = _tiny_cg()
    V, n = cg["num_nodes"], cg["num_players"]
    X = rng.normal(size=(8, 4))
    m = _model(rng, 4, (2, 1), (3, 5))
    for l in range(2):
        m["a_src"][l][:] = 0.0
        m["a_dst"][l][:] = 0.0
    active = rng.random(n) < 0.6
    A = np.eye(V)
    for j in np.flatnonzero(active):
        A[cg["ldst"][j], cg["lsrc"][j]] = 1.0
        A[cg["lsrc"][j], cg["ldst"][j]] = 1.0
    M = A / A.sum(axis=1, keepdims=True)
    Xc = X[cg["node_gid"]]
    h = M @ (Xc @ m["W"][0])
    h = np.where(h > 0, h, np.expm1(np.minimum(h, 0)))
    want = (M @ (h @ m["W"][1]))[cg["target_local"]]
    got = gat.ValueFunction(cg, X, m, score="logit").logits(active)
    assert np.allclose(got, want, rtol=0, atol=1e-13)


def test_two_nodes_by_hand():
    """One edge 1 -> 0 (undirected player), one layer, one head of width 1, scalar features.
    z_i = w x_i.  Receiver 0: e_00 = lrelu((a_d + a_s) z_0), e_01 = lrelu(a_d z_0 + a_s z_1);
    alpha_01 = 1 / (1 + exp(e_00 - e_01)); out_0 = (1 - alpha_01) z_0 + alpha_01 z_1."""
    cg = dict(num_nodes=2, num_players=1, lsrc=np.array([1]), ldst=np.array([0]), undirected=True,
              node_gid=np.array([0, 1]), target_local=0)
    x0, x1, w, a_s, a_d, slope = 0.5, -2.0, 1.5, 0.8, -0.3, 0.2
    z0, z1 = w * x0, w * x1                       # 0.75, -3.0
    e00 = (a_d + a_s) * z0                        # 0.375 > 0
    e01 = a_d * z0 + a_s * z1                     # -0.225 - 2.4 = -2.625 -> slope * = -0.525
    assert e00 > 0 and e01 < 0
    e01 = slope * e01
    al = 1.0 / (1.0 + math.exp(e00 - e01))
    want = (1 - al) * z0 + al * z1
    m = dict(W=[np.array([[w]])], a_src=[np.array([[a_s]])], a_dst=[np.array([[a_d]])], bias=None, heads=[1], slope=slope)
    f = gat.ValueFunction(cg, np.array([[x0], [x1]]), m, score="logit")
    got = f.logits(np.array([True]))[0]
    assert abs(got - want) < 1e-15
    # exchanging the two halves of the attention vector gives the other closed form
    m2 = dict(m, a_src=[np.array([[a_d]])], a_dst=[np.array([[a_s]])])
    e01b = a_s * z0 + a_d * z1                    # 0.6 + 0.9 = 1.5
    alb = 1.0 / (1.0 + math.exp(e00 - e01b))
    got2 = gat.ValueFunction(cg, np.array([[x0], [x1]]), m2, score="logit").logits(np.array([True]))[0]
    assert abs(got2 - ((1 - alb) * z0 + alb * z1)) < 1e-15
    assert abs(got - got2) > 0.1
    # without the edge the node keeps its own value
    assert abs(f.logits(np.array([False]))[0] - z0) < 1e-15


def test_directed_player_only_feeds_its_destination():
    cg = dict(num_nodes=2, num_players=1, lsrc=np.array([0]), ldst=np.array([1]), undirected=False,
              node_gid=np.array([0, 1]), target_local=0)
    m = dict(W=[np.array([[1.0]])], a_src=[np.array([[0.3]])], a_dst=[np.array([[0.1]])], bias=None, heads=[1], slope=0.2)
    f = gat.ValueFunction(cg, np.array([[2.0], [5.0]]), m, score="logit")
    assert f.logits(np.array([True]))[0] == 2.0          # node 0 receives nothing from the edge 0 -> 1


def test_relabelling_nodes_changes_nothing():
    rng = np.random.default_rng(3)
    row_ptr, col, cg = _tiny_cg()
    X = rng.normal(size=(8, 6))
    m = _model(rng, 6, (4, 2), (3, 4), bias=True)
    active = rng.random(cg["num_players"]) < 0.5
    base = gat.ValueFunction(cg, X, m)(active)
    perm = rng.permutation(cg["num_nodes"])
    inv = np.argsort(perm)
    cg2 = dict(cg)
    cg2["lsrc"] = inv[cg["lsrc"]]
    cg2["ldst"] = inv[cg["ldst"]]
    cg2["node_gid"] = cg["node_gid"][perm]
    cg2["target_local"] = int(inv[cg["target_local"]])
    assert abs(gat.ValueFunction(cg2, X, m)(active) - base) < 1e-14


def test_attention_rows_sum_to_one_and_heads_are_independent():
    rng = np.random.default_rng(4)
    row_ptr, col, cg = _tiny_cg()
    X = rng.normal(size=(8, 4))
    conn = gat.connectivity(cg, rng.random(cg["num_players"]) < 0.5)
    Xc = X[cg["node_gid"]]
    m = _model(rng, 4, (2,), (3,))
    # constant value rows: any convex combination returns the constant, so the output equals it for every head
    Wc = np.zeros((4, 6))
    out = gat.layer(conn, np.ones((cg["num_nodes"], 4)), Wc + 0.25, m["a_src"][0], m["a_dst"][0], None, 2, last=True)
    assert np.allclose(out, 1.0, atol=1e-14)
    # a head's output does not depend on the other head's parameters
    full = gat.layer(conn, Xc, m["W"][0], m["a_src"][0], m["a_dst"][0], None, 2, last=False)
    W2 = m["W"][0].copy()
    W2[:, 3:] = rng.normal(size=(4, 3))
    other = gat.layer(conn, Xc, W2, m["a_src"][0], m["a_dst"][0], None, 2, last=False)
    assert np.allclose(full[:, :3], other[:, :3], atol=1e-14)
    assert not np.allclose(full[:, 3:], other[:, 3:])


def test_unreachable_edges_are_null_players():
    """Two layers on the 3-hop graph of a path-like instance: an edge whose two ends are both farther than
    one hop from the target never enters a needed attention row, so its exact Shapley value is 0 (unlike
    the GCN, whose degree normalisation couples every edge)."""
    rng = np.random.default_rng(5)
    # path 0-1-2-3 plus a chord 1-3
    src = np.array([0, 1, 2, 1])
    dst = np.array([1, 2, 3, 3])
    row_ptr, col = graphs.csr_from_undirected_edges(4, src, dst)
    cg = compgraph.extract(row_ptr, col, 0, 3, True)
    X = rng.normal(size=(4, 3))
    m = _model(rng, 3, (2, 1), (2, 3))
    f = gat.ValueFunction(cg, X, m)
    n = cg["num_players"]
    assert n == 4
    phi = shapley.exact_shapley(shapley.all_values(f, n), n)
    gid = cg["node_gid"]
    for j in range(n):
        ends = {int(gid[cg["lsrc"][j]]), int(gid[cg["ldst"][j]])}
        if ends == {2, 3}:
            assert phi[j] == 0.0
        else:
            assert abs(phi[j]) > 1e-6
    assert abs(phi.sum() - (f(np.ones(n, bool)) - f(np.zeros(n, bool)))) < 1e-13
