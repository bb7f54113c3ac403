"""Value function of the game: the GCN's output for the target node on the
sub-graph selected by a coalition of edges.

GCN layer (Kipf & Welling, cited by the paper): with A_S the adjacency of the
coalition's edges on the computational graph's nodes,
  A~ = A_S + I,  d_i = sum_j A~[i, j],  A^ = D^-1/2 A~ D^-1/2,
  H^l = ReLU(A^ H^(l-1) W_l + b_l)  (no ReLU on the last layer).
Degrees are recomputed for every coalition.  An undirected player switches
both directions of its edge; a directed player (src -> dst) sets A~[dst, src].
The game's value is the softmax probability (or the raw logit) that the last
layer assigns, at the target, to the class predicted on the full graph
(evaluation-metric section: "prediction score of the predicted class").
"""
import numpy as np
import scipy.sparse as sp


def adjacency_dense(cg, active):
    n = cg["num_nodes"]
    A = np.eye(n, dtype=np.float64)
    act = np.flatnonzero(active)
    s, d = cg["lsrc"][act], cg["ldst"][act]
    A[d, s] = 1.0
    if cg["undirected"]:
        A[s, d] = 1.0
    deg = A.sum(axis=1)
    dinv = 1.0 / np.sqrt(deg)
    return dinv[:, None] * A * dinv[None, :]


def adjacency_sparse(cg, active):
    n = cg["num_nodes"]
    act = np.flatnonzero(active)
    s, d = cg["lsrc"][act], cg["ldst"][act]
    loops = np.arange(n)
    if cg["undirected"]:
        rows = np.concatenate([d, s, loops])
        cols = np.concatenate([s, d, loops])
    else:
        rows = np.concatenate([d, loops])
        cols = np.concatenate([s, loops])
    A = sp.csr_matrix((np.ones(len(rows)), (rows, cols)), shape=(n, n))
    deg = np.asarray(A.sum(axis=1)).ravel()
    D = sp.diags(1.0 / np.sqrt(deg))
    return (D @ A @ D).tocsr()


def round_bf16(x):
    """Round to the nearest bfloat16 (ties to even), returned as float64."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def forward(Ahat, X, weights, biases=None, bf16=False):
    """Logits of every node. X float64[n, d0].

    bf16=True is a DIAGNOSTIC mode (parity of the reduced-precision configuration is
    judged against bf16=False): in layers 2..L the two operands of the dense
    transform, the aggregated activations A^ H and W_l, are rounded to bfloat16 and
    the products are accumulated exactly; layer 1 (whose product with W_1 does not
    depend on the coalition) is left unrounded."""
    H = np.asarray(X, dtype=np.float64)
    L = len(weights)
    for l, W in enumerate(weights):
        W = np.asarray(W, dtype=np.float64)
        if bf16 and l >= 1:
            H = round_bf16(Ahat @ H) @ round_bf16(W)
        else:
            H = (Ahat @ H) @ W
        if biases is not None and biases[l] is not None:
            H = H + np.asarray(biases[l], dtype=np.float64)
        if l < L - 1:
            H = np.maximum(H, 0.0)
    return H


def softmax(z):
    e = np.exp(z - np.max(z))
    return e / e.sum()


class ValueFunction:
    """f(S) for the target of a computational graph."""

    def __init__(self, cg, X_global, weights, biases=None, score="prob", dense=False, bf16=False):
        self.bf16 = bf16
        self.cg = cg
        self.X = np.asarray(X_global, dtype=np.float64)[cg["node_gid"]]
        self.weights = weights
        self.biases = biases
        self.score = score
        self.adj = adjacency_dense if dense else adjacency_sparse
        full = self.logits(np.ones(cg["num_players"], dtype=bool))
        self.pred_class = int(np.argmax(full))          # ties -> lowest index

    def logits(self, active):
        Ahat = self.adj(self.cg, np.asarray(active, dtype=bool))
        return forward(Ahat, self.X, self.weights, self.biases, self.bf16)[self.cg["target_local"]]

    def __call__(self, active):
        z = self.logits(active)
        if self.score == "logit":
            return float(z[self.pred_class])
        return float(softmax(z)[self.pred_class])

    def batch(self, bits):
        return np.array([self(row) for row in bits], dtype=np.float64)
