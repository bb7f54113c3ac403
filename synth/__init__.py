"""Seeded synthetic inputs (graphs, features, GCN weights, targets) shared by
the CPU oracle's tests and the HIP path's tests and benchmark.

Nothing in this package performs any step of the explanation method: it only
manufactures graphs, feature matrices and weight matrices, and picks target
nodes by plain graph statistics.
"""
from .graphs import (csr_from_undirected_edges, tiny_graph, barabasi_albert,
                     rmat, khop_ball, induced_undirected_edge_count, fanout_capped_subgraph)
from .workloads import (Workload, make_workload, glorot_uniform, WORKLOADS)
