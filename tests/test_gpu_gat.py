"""GAT model family on the GPU (masked attention inference and the explanation built on it) vs the
oracle's GAT value function (oracle/gat.py), same seeded inputs, through the C ABI."""
import numpy as np
import pytest

from oracle import compgraph, explain as oexplain, gat as ogat, sampling, solve
from synth import make_workload
from synth.workloads import _gat_model
from tests.gpu_common import say, to_u64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _context(w, model, biases=None):
    from paper_2506_22668_amd import Context
    ctx = Context("cuda:0")
    ctx.set_graph(w.row_ptr, w.col)
    ctx.set_features(w.features)
    ctx.set_gat(model["W"], model["a_src"], model["a_dst"], model["heads"], biases=biases,
                negative_slope=model["slope"])
    return ctx


def _random_rows(n, rows, rng):
    bits = np.zeros((rows, n), dtype=bool)
    bits[1] = True
    for i in range(2, rows):
        bits[i] = rng.random(n) < rng.random() ** 2
    bits[rows - 1] = ~bits[rows - 2]
    return bits


def _eval_case(w, model, hops, directed, score, rows, rng, biases=None, tol=2e-5):
    from paper_2506_22668_amd import Options
    ctx = _context(w, model, biases)
    target = w.targets[0]
    cg = ctx.extract(target, Options(hops=hops, directed=int(directed)))
    cgo = compgraph.extract(w.row_ptr, w.col, target, hops, undirected=not directed)
    n = cgo["num_players"]
    m = dict(model, bias=biases)
    f = ogat.ValueFunction(cgo, w.features, m, "logit" if score else "prob")
    bits = _random_rows(n, rows, rng)
    Z = torch.from_numpy(sampling.pack_rows(bits).view(np.int64)).cuda()
    y, pc = ctx.eval(cg, Z, score)
    ref = f.batch(bits)
    assert pc == f.pred_class
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref).max()
    scale = max(1.0, np.abs(ref).max())
    say(f"  n={n} V={cgo['num_nodes']} rows={rows} err={err:.2e}")
    assert err <= tol * scale, f"max |y - oracle| = {err}"
    ctx.cgraph_free(cg)
    ctx.close()


@pytest.mark.parametrize("key,hops,directed,score,with_bias", [
    ("gat_small", 2, False, 0, False), ("gat_small", 2, False, 1, True), ("gat_small", 3, False, 0, False),
    ("gat_small", 1, False, 0, True), ("gat_small", 2, True, 0, False),
])
def test_masked_gat_inference_matches_oracle(key, hops, directed, score, with_bias):
    w = make_workload(key)
    say(f"gat eval {key} hops={hops} directed={directed} score={score} bias={with_bias}")
    rng = np.random.default_rng(7)
    biases = None
    if with_bias:
        outs = [w.gat["heads"][0] * w.gat["widths"][0], w.gat["widths"][1]]
        biases = [0.1 * rng.standard_normal(o).astype(np.float32) for o in outs]
    # 96 rows: every layer in the one-workgroup-per-coalition kernel; 333 rows (five blocks of 64 and a ragged
    # tail): layer 1 of all coalitions on the matrix cores first
    _eval_case(w, w.gat, hops, directed, score, 96, rng, biases)
    _eval_case(w, w.gat, hops, directed, score, 333, rng, biases)


@pytest.mark.parametrize("heads,widths", [
    ((1,), (5,)),                 # one layer: heads averaged straight into the logits
    ((3,), (4,)),
    ((8, 4, 2), (8, 5, 6)),       # three layers
    ((8, 1), (40, 7)),            # transform width 320: more than one pass of feature columns
    ((5, 3), (13, 4)),            # widths that are not multiples of the wave size
])
def test_masked_gat_shapes(heads, widths):
    w = make_workload("gat_small")
    rng = np.random.default_rng(11)
    model = _gat_model(rng, w.dims[0], heads, widths)
    say(f"gat eval shapes heads={heads} widths={widths}")
    _eval_case(w, model, len(heads), False, 0, 40, rng)
    _eval_case(w, model, len(heads), False, 0, 270, rng)


def test_masked_gat_wide_attention_range_falls_back_to_the_running_maximum():
    """Attention vectors scaled up until the logits of one row span more than exp() can hold in fp32 relative
    to the row maximum: the matrix-core path for layer 1 must step aside (its weights would underflow) and the
    per-coalition kernel with the running maximum gives the answer."""
    w = make_workload("gat_small")
    rng = np.random.default_rng(13)
    model = _gat_model(rng, w.dims[0], (4, 2), (8, 6))
    model["a_src"] = [a * 60.0 for a in model["a_src"]]
    model["a_dst"] = [a * 60.0 for a in model["a_dst"]]
    cgo = compgraph.extract(w.row_ptr, w.col, w.targets[0], 2)
    Xc = w.features[cgo["node_gid"]].astype(np.float64)
    Zf = Xc @ model["W"][0].astype(np.float64)
    s = (Zf.reshape(len(Zf), 4, 8) * model["a_src"][0][None]).sum(-1)
    assert s.max() - s.min() > 200.0          # the premise of the test
    say("gat eval wide attention range")
    _eval_case(w, model, 2, False, 0, 300, rng, tol=1e-4)


def test_masked_gat_long_rows_shared_by_the_workgroup():
    """The R-MAT target sits next to a hub: the hub's row (hundreds of entries) is split over the waves and
    the partial soft-max states are merged; rows are compared one by one with the oracle."""
    from paper_2506_22668_amd import Options
    w = make_workload("gat_rmat")
    say(f"gat eval {w.name} (hub row)")
    ctx = _context(w, w.gat)
    target = w.targets[0]
    cg = ctx.extract(target, Options(hops=2))
    cgo = compgraph.extract(w.row_ptr, w.col, target, 2)
    n = cgo["num_players"]
    # the longest needed row must be a shared one
    deg = np.bincount(np.concatenate([cgo["ldst"], cgo["lsrc"]]), minlength=cgo["num_nodes"])
    assert deg[: w.info["balls"][1]].max() > 128
    rng = np.random.default_rng(3)
    bits = _random_rows(n, 24, rng)
    Z = torch.from_numpy(sampling.pack_rows(bits).view(np.int64)).cuda()
    y, pc = ctx.eval(cg, Z)
    f = ogat.ValueFunction(cgo, w.features, w.gat)
    ref = f.batch(bits)
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref).max()
    say(f"  n={n} V={cgo['num_nodes']} err={err:.2e}")
    assert pc == f.pred_class and err <= 2e-5
    # the same rows inside a batch large enough for the matrix-core path of layer 1 (its hub row spans dozens
    # of 16-entry steps): the first 24 against the oracle, the rest against the per-coalition kernel
    more = _random_rows(n, 320, rng)
    more[:24] = bits
    Zm = torch.from_numpy(sampling.pack_rows(more).view(np.int64)).cuda()
    ym = ctx.eval(cg, Zm)[0].cpu().numpy().astype(np.float64)
    assert np.abs(ym[:24] - ref).max() <= 2e-5
    parts = np.concatenate([ctx.eval(cg, Zm[i:i + 80].contiguous())[0].cpu().numpy() for i in range(0, 320, 80)])
    say(f"  matrix-core layer 1 vs per-coalition kernel: {np.abs(ym - parts).max():.2e}")
    assert np.abs(ym - parts).max() <= 5e-6
    ctx.cgraph_free(cg)
    ctx.close()


def test_gat_explanation_small_end_to_end():
    from paper_2506_22668_amd import Options
    w = make_workload("gat_small")
    ctx = _context(w, w.gat)
    target = w.targets[0]
    say(f"gat explain {w.name} target={target}")
    phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, Options(solver=1))
    ref = oexplain.explain(w.row_ptr, w.col, w.features, None, target, w.n_samples, w.seed, gat=w.gat)
    assert rep.num_players == ref["n"] and rep.num_rows == ref["k"] and rep.pred_class == ref["pred_class"]
    assert np.array_equal(es.cpu().numpy(), ref["cg"]["edge_src"])
    got = phi.cpu().numpy().astype(np.float64)
    scale = np.abs(ref["phi"]).max()
    err = np.abs(got - ref["phi"]).max()
    say(f"  n={ref['n']} k={ref['k']} max|phi|={scale:.3e} err={err:.3e}")
    assert err <= 1e-4 * scale
    assert abs(got.sum() - (rep.f_full - rep.f_empty)) <= 1e-5
    # edges that enter no needed attention row (both ends two hops away) carry no signal: the regression
    # leaves them at the level of the sampling noise, far below the edges at the target
    gid = ref["cg"]["node_gid"]
    hop = ref["cg"]["hop"]
    far = (hop[ref["cg"]["lsrc"]] >= 2) & (hop[ref["cg"]["ldst"]] >= 2)
    assert far.any() and (~far).any()
    assert np.abs(ref["phi"][far]).max() < 0.2 * np.abs(ref["phi"][~far]).max()
    # CGLS on the same rows agrees with the direct solve
    phi2, _, _, rep2, _ = ctx.explain(target, w.n_samples, w.seed, Options(solver=2, tol=1e-9))
    assert np.abs(phi2.cpu().numpy() - got).max() <= 1e-4 * scale
    ctx.close()


def test_gat_explanation_full_size_sampled_rows():
    """BA graph with 10^4 nodes, ~1000 players, 20,000 coalitions, 8 heads: masks bit-exact on all rows, y on a
    stratified 2 % of the rows against the oracle, phi against the oracle's fp64 solve on the GPU's y (the
    oracle's dense attention takes ~25 ms per coalition, so all 20,000 rows are out of reach of a test)."""
    from paper_2506_22668_amd import Options
    w = make_workload("gat_c2")
    ctx = _context(w, w.gat)
    target = w.targets[0]
    say(f"gat full size {w.name} target={target}")
    cg = ctx.extract(target, Options(hops=2))
    cgo = compgraph.extract(w.row_ptr, w.col, target, 2)
    n = cgo["num_players"]
    assert ctx.cgraph_info(cg).num_players == n
    Z, wt, sz = ctx.sample(n, w.n_samples, w.seed, target)
    Zo, wo, szo = sampling.sample(n, w.n_samples, w.seed, target & 0xFFFFFFFF)
    assert np.array_equal(to_u64(Z), Zo) and np.array_equal(wt.cpu().numpy(), wo)
    y, pc = ctx.eval(cg, Z)
    yh = y.cpu().numpy().astype(np.float64)
    f = ogat.ValueFunction(cgo, w.features, w.gat)
    assert pc == f.pred_class
    k = len(wo)
    pick = np.unique(np.concatenate([[0, 1, 2, 3, k - 2, k - 1], np.linspace(0, k - 1, 400).astype(np.int64)]))
    bits = sampling.unpack_rows(Zo[pick], n)
    ref = f.batch(bits)
    err = np.abs(yh[pick] - ref).max()
    say(f"  n={n} k={k} rows checked={len(pick)} err(y)={err:.2e}")
    assert err <= 2e-5
    phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, Options(solver=1))
    got = phi.cpu().numpy().astype(np.float64)
    want = solve.solve_lstsq(sampling.unpack_rows(Zo, n), wo, yh)
    scale = np.abs(want).max()
    say(f"  max|phi|={scale:.3e} err(phi)={np.abs(got - want).max():.3e} ms: eval={rep.ms_eval:.3f} total={rep.ms_total:.3f}")
    assert np.abs(got - want).max() <= 1e-4 * scale
    ctx.cgraph_free(cg)
    ctx.close()


def test_switching_model_family_on_one_context():
    """ds_set_gcn after ds_set_gat (and back) on the same context: a graph extracted for one model is refused
    for the other instead of being evaluated with the wrong first transform."""
    from paper_2506_22668_amd import DistShapError, Options
    w = make_workload("gat_small")
    say("model switch gat -> gcn -> gat")
    ctx = _context(w, w.gat)
    target = w.targets[0]
    phi_a = ctx.explain(target, 2000, 5, Options(solver=1))[0].cpu().numpy()
    cg = ctx.extract(target, Options(hops=2))
    ctx.set_gcn([np.ones((w.dims[0], 5), dtype=np.float32), np.ones((5, 3), dtype=np.float32)])
    n = ctx.cgraph_info(cg).num_players
    Z = torch.zeros((2, (n + 63) // 64), dtype=torch.int64, device="cuda")
    with pytest.raises(DistShapError):
        ctx.eval(cg, Z)
    ctx.cgraph_free(cg)
    ctx.set_gat(w.gat["W"], w.gat["a_src"], w.gat["a_dst"], w.gat["heads"])
    phi_b = ctx.explain(target, 2000, 5, Options(solver=1))[0].cpu().numpy()
    assert np.array_equal(phi_a, phi_b)
    ctx.close()


def test_gat_batch_equals_single_explanations_and_fidelity_matches_oracle():
    """The other entry points with a GAT set: ds_explain_batch (worker contexts take the attention model along) gives
    exactly the single-call results, and ds_fidelity evaluates the GAT on the top-k sub-graphs like the oracle."""
    from oracle import fidelity
    from paper_2506_22668_amd import Options
    w = make_workload("gat_small")
    ctx = _context(w, w.gat)
    rng = np.random.default_rng(2)
    deg = np.diff(w.row_ptr)
    targets = [w.targets[0]] + [int(t) for t in rng.choice(np.flatnonzero(deg >= 3), size=5, replace=False)]
    say(f"gat batch targets={targets}")
    singles = [ctx.explain(t, 2000, w.seed, Options(solver=1))[0] for t in targets]
    total = sum(len(x) for x in singles)
    phi, M, off, es, ed, reps, rc = ctx.explain_batch(targets, 2000, w.seed, Options(solver=1), capacity=total)
    assert rc == 0 and M == [len(x) for x in singles]
    for i, x in enumerate(singles):
        assert torch.equal(phi[off[i]:off[i + 1]], x)
    target = targets[0]
    cg = ctx.extract(target, Options(hops=2))
    cgo = compgraph.extract(w.row_ptr, w.col, target, 2)
    n = cgo["num_players"]
    ks = [0, 1, 3, 10, n // 2, n]
    plus, minus, masks = ctx.fidelity(cg, singles[0], ks, 0, want_masks=True)
    f = ogat.ValueFunction(cgo, w.features, w.gat)
    ph = singles[0].cpu().numpy()
    assert np.array_equal(to_u64(masks), sampling.pack_rows(fidelity.top_k_masks(ph, ks)))
    rp, rm = fidelity.fidelity(f, ph, ks)
    assert np.abs(np.array(plus) - rp).max() <= 2e-5 and np.abs(np.array(minus) - rm).max() <= 2e-5
    ctx.cgraph_free(cg)
    ctx.close()
