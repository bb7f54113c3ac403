"""The plain-C restatement of the oracle agrees with the (pinned) numpy oracle on small inputs."""
import os

import numpy as np
import pytest

from oracle import cfast, compgraph, gcn, philox, sampling, solve
from synth import make_workload


def test_c_philox_known_answers():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        assert list(cfast.philox(v[:4], v[4:6])) == v[6:]
    rng = np.random.default_rng(1)
    for _ in range(50):
        c = rng.integers(0, 1 << 32, size=4)
        k = rng.integers(0, 1 << 32, size=2)
        assert cfast.philox(c, k) == philox.philox4x32_10(c, k)


@pytest.mark.parametrize("n,ns", [(12, 4096), (2, 4), (30, 25000), (65, 1001), (1000, 20000), (4001, 600)])
def test_c_plan_and_masks_equal_numpy(n, ns):
    plan = sampling.allocation(n, ns)
    k, en, b, wtab = cfast.plan(n, ns)
    assert k == plan["k"] and en == plan["enumerate"]
    assert np.array_equal(wtab.view(np.uint32), plan["wtab"].view(np.uint32))
    if not en:
        assert np.array_equal(b, plan["b"])
    pr = None if k <= 8000 else (0, 1500)
    Z, w, sz = sampling.sample(n, ns, 77 + n, 5, pair_range=pr)
    Zc, wc, szc = cfast.sample(n, ns, 77 + n, 5, pair_range=pr)
    assert np.array_equal(Z, Zc) and np.array_equal(sz, szc)
    assert np.array_equal(w.view(np.uint32), wc.view(np.uint32))


@pytest.mark.parametrize("key,directed,score,bf16,with_bias", [
    ("c1", False, "prob", False, False), ("c1", True, "logit", False, True),
    ("c2_small", False, "prob", False, False), ("c2_small", False, "prob", True, True),
    ("c3_small", False, "logit", False, False),
])
def test_c_gcn_values_equal_numpy(key, directed, score, bf16, with_bias):
    w = make_workload(key)
    rng = np.random.default_rng(3)
    cg = compgraph.extract(w.row_ptr, w.col, w.targets[0], w.num_layers, undirected=not directed)
    biases = [0.1 * rng.standard_normal(d) for d in w.dims[1:]] if with_bias else None
    f = gcn.ValueFunction(cg, w.features, w.weights, biases, score, bf16=bf16)
    n = cg["num_players"]
    bits = rng.random((24, n)) < rng.random((24, 1))
    bits[0] = False
    bits[1] = True
    ref = f.batch(bits)
    y, pc, _ = cfast.gcn_values(cg, w.features, w.weights, sampling.pack_rows(bits), biases, score, bf16=bf16)
    assert pc == f.pred_class
    assert np.abs(y - ref).max() < 1e-12


def test_c_cgls_and_residual_equal_numpy():
    rng = np.random.default_rng(5)
    for n, ns in [(40, 2000), (300, 200)]:
        Z, w, sz = sampling.sample(n, ns, 9, 1)
        bits = sampling.unpack_rows(Z, n)
        y = 0.3 + bits @ rng.standard_normal(n) + 0.2 * np.sin(bits @ rng.standard_normal(n))
        for tol in (1e-6, 1e-11):
            ref, it, rel = solve.solve_cgls(bits, w, y, tol=tol)
            phi, itc, relc = cfast.cgls(n, Z, w, y, tol=tol)
            assert relc <= tol and abs(itc - it) <= 1
            # the two sum in different orders; near a loose threshold they may stop one iteration apart,
            # so the iterates are compared tightly only when both are converged far below it
            bound = 1e-9 if tol < 1e-9 else 1e-4
            assert np.abs(phi - ref).max() < bound * max(1.0, np.abs(ref).max())
            # the explicitly recomputed residual equals the recursively updated one up to round-off
            assert cfast.normal_residual(n, Z, w, y, phi) == pytest.approx(relc, rel=1e-3, abs=1e-9)
        # the C version is reproducible from run to run
        again = cfast.cgls(n, Z, w, y, tol=1e-6)[0]
        assert np.array_equal(again, cfast.cgls(n, Z, w, y, tol=1e-6)[0])
        assert cfast.normal_residual(n, Z, w, y, np.full(n, (y[1] - y[0]) / n)) == pytest.approx(1.0)
