"""CPU oracle for Kernel-SHAP edge attribution of a GCN prediction.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 restatement of
what the method computes, written from the paper's definitions.  It shares no
code with the HIP library and must never be imported by it: only the tests,
the smoke check and the benchmark's CPU-baseline leg may use it.

Pin status (what checks each part against something other than itself is
listed in tests/test_oracle_*.py):
  philox, allocation, weights, masks, GCN forward, exact Shapley,
  enumerated Kernel-SHAP, least-squares solvers (dense, KKT, CGLS): pinned.
  Sampled-mode phi (a randomised estimate): pinned only statistically
  (error against exact Shapley shrinks with the sample count).
  Fidelity of explanations on the paper's datasets: parity unpinned (the
  datasets and trained weights are not available offline).
"""
