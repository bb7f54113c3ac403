"""Top-k masks (bit-exact) and fidelity scores of the HIP path vs the oracle."""
import numpy as np
import pytest

from oracle import compgraph, fidelity, gcn, sampling
from synth import make_workload
from tests.gpu_common import make_context, say, to_u64

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("key,score", [("c1", 0), ("c2_small", 1), ("c2", 0), ("c3_small", 0)])
def test_fidelity_matches_oracle(key, score):
    w = make_workload(key)
    say(f"fidelity {key} score={score}")
    ctx = make_context(w)
    target = w.targets[0]
    phi, es, ed, rep, rc = ctx.explain(target, min(w.n_samples, 4096), w.seed, allow_not_converged=True)
    n = rep.num_players
    # plant ties and a signed zero so the tie rule is exercised
    phi = phi.clone()
    if n > 8:
        phi[5] = phi[2]
        phi[7] = -0.0
        phi[3] = 0.0
    cg = ctx.extract(target)
    ks = [0, 1, 2, 5, 10, 20, 30, 50, n // 2, n, n + 7]
    plus, minus, masks = ctx.fidelity(cg, phi, ks, score, want_masks=True)
    cgo = compgraph.extract(w.row_ptr, w.col, target, w.num_layers)
    f = gcn.ValueFunction(cgo, w.features, w.weights, score="logit" if score else "prob")
    ph = phi.cpu().numpy()
    ref_masks = sampling.pack_rows(fidelity.top_k_masks(ph, ks))
    assert np.array_equal(to_u64(masks), ref_masks)
    rp, rm = fidelity.fidelity(f, ph, ks)
    scale = max(1.0, abs(f(np.ones(n, bool))))
    assert np.abs(np.array(plus) - rp).max() <= 2e-5 * scale
    assert np.abs(np.array(minus) - rm).max() <= 2e-5 * scale
    ctx.cgraph_free(cg)
    ctx.close()
