"""Value function of the game for the paper's second model family: a graph
attention network (the paper's evaluation uses a two-layer GAT with 8 heads;
the layer is the one of Velickovic et al., ICLR 2018, which the paper cites).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Layer with H heads of width F on the sub-graph selected by a coalition S.  With
Z = X W (W: [d_in, H*F]) and z_i^h the h-th width-F slice of row i,
  e_ij^h     = LeakyReLU_slope( a_dst^h . z_i^h  +  a_src^h . z_j^h )      for j in N_S(i) + {i}
  alpha_ij^h = exp(e_ij^h) / sum_{j'} exp(e_ij'^h)                          (softmax over the same j)
  out_i^h    = sum_j alpha_ij^h z_j^h
where N_S(i) are the in-neighbours of i whose edge belongs to S; the self term is
always present and is not a player (same reading as for the GCN).  A hidden
layer concatenates its heads, adds the bias and applies ELU; the last layer
averages its heads, adds the bias and applies nothing.  `a_dst` multiplies the
receiving node, `a_src` the neighbour (the two halves of the attention vector).
The game's value is the softmax probability (or logit) of the class predicted on
the full computational graph, at the target.

Everything is written with explicit dense [V, V] attention matrices, one per head,
for every node and every layer.
"""
import numpy as np


def elu(x):
    return np.where(x > 0.0, x, np.expm1(np.minimum(x, 0.0)))


def connectivity(cg, active):
    """Boolean [V, V]: entry [i, j] says that j sends a message to i (self included)."""
    n = cg["num_nodes"]
    A = np.eye(n, dtype=bool)
    act = np.flatnonzero(np.asarray(active, dtype=bool))
    s, d = cg["lsrc"][act], cg["ldst"][act]
    A[d, s] = True
    if cg["undirected"]:
        A[s, d] = True
    return A


def layer(conn, X, W, a_src, a_dst, bias, heads, last, slope=0.2):
    V = X.shape[0]
    Z = X @ np.asarray(W, dtype=np.float64)
    F = Z.shape[1] // heads
    a_src = np.asarray(a_src, dtype=np.float64).reshape(heads, F)
    a_dst = np.asarray(a_dst, dtype=np.float64).reshape(heads, F)
    outs = []
    for h in range(heads):
        Zh = Z[:, h * F:(h + 1) * F]
        e = (Zh @ a_dst[h])[:, None] + (Zh @ a_src[h])[None, :]      # [receiver i, neighbour j]
        e = np.where(e > 0.0, e, slope * e)
        e = np.where(conn, e, -np.inf)
        e = e - e.max(axis=1, keepdims=True)
        p = np.exp(e)
        alpha = p / p.sum(axis=1, keepdims=True)
        outs.append(alpha @ Zh)
    if last:
        out = sum(outs) / float(heads)
    else:
        out = np.concatenate(outs, axis=1)
    if bias is not None:
        out = out + np.asarray(bias, dtype=np.float64)
    return out if last else elu(out)


def forward(conn, X, model):
    """Logits of every node.  model: dict(W=[...], a_src=[...], a_dst=[...], bias=[...]|None, heads=[...], slope)."""
    H = np.asarray(X, dtype=np.float64)
    L = len(model["W"])
    for l in range(L):
        b = None if model.get("bias") is None else model["bias"][l]
        H = layer(conn, H, model["W"][l], model["a_src"][l], model["a_dst"][l], b, model["heads"][l],
                  last=(l == L - 1), slope=model.get("slope", 0.2))
    return H


def softmax(z):
    e = np.exp(z - np.max(z))
    return e / e.sum()


class ValueFunction:
    """f(S) for the target of a computational graph under a GAT."""

    def __init__(self, cg, X_global, model, score="prob"):
        self.cg = cg
        self.X = np.asarray(X_global, dtype=np.float64)[cg["node_gid"]]
        self.model = model
        self.score = score
        full = self.logits(np.ones(cg["num_players"], dtype=bool))
        self.pred_class = int(np.argmax(full))          # ties -> lowest index

    def logits(self, active):
        return forward(connectivity(self.cg, active), self.X, self.model)[self.cg["target_local"]]

    def __call__(self, active):
        z = self.logits(active)
        if self.score == "logit":
            return float(z[self.pred_class])
        return float(softmax(z)[self.pred_class])

    def batch(self, bits):
        return np.array([self(row) for row in bits], dtype=np.float64)
