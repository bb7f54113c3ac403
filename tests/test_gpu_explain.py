"""End-to-end parity: ds_explain on the GPU vs the oracle's explanation, same seeded inputs."""
import numpy as np
import pytest

from oracle import explain as oexplain
from synth import csr_from_undirected_edges, make_workload
from tests.gpu_common import make_context, say

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SOLVERS = {"gram_chol": 1, "cgls": 2}


def _explain_case(key, tol, solver=None, oracle_solver="lstsq", targets=None, eval_path=0):
    from paper_2506_22668_amd import Options, Tuning
    w = make_workload(key)
    dtype = 1 if w.transform_dtype == "bf16" else 0
    ctx = make_context(w, transform_dtype=dtype)
    if eval_path:
        ctx.set_tuning(Tuning(eval_path=eval_path))
    opts = Options(solver=SOLVERS[solver or w.solver], tol=w.tol)
    for target in (targets or w.targets):
        say(f"explain {key} target={target}")
        phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, opts)
        # an iterative solve is compared at the same stopping rule on both sides: the
        # truncation error of CGLS at tol is part of the method, not of the arithmetic
        # the gate is always the plain fp64 oracle, also for the reduced-precision configuration
        ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed,
                               solver=oracle_solver, tol=w.tol)
        assert rep.num_players == ref["n"] and rep.num_rows == ref["k"]
        assert rep.pred_class == ref["pred_class"]
        assert np.array_equal(es.cpu().numpy(), ref["cg"]["edge_src"])
        assert np.array_equal(ed.cpu().numpy(), ref["cg"]["edge_dst"])
        got = phi.cpu().numpy().astype(np.float64)
        scale = np.abs(ref["phi"]).max()
        err = np.abs(got - ref["phi"]).max()
        say(f"  n={ref['n']} k={ref['k']} max|phi|={scale:.3e} err={err:.3e} iters={rep.cgls_iterations} "
            f"ms: ext={rep.ms_extract:.2f} smp={rep.ms_sample:.2f} eval={rep.ms_eval:.2f} solve={rep.ms_solve:.2f}")
        assert err <= tol * scale
        if dtype == 1:
            # diagnostic beside the gate: against the oracle's bfloat16-emulating mode (per-coalition transforms
            # round both operands) only accumulation order is left
            diag = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed,
                                    solver=oracle_solver, tol=w.tol, bf16=True)
            derr = np.abs(got - diag["phi"]).max()
            say(f"  diagnostic: err vs the bf16-emulating oracle mode = {derr:.3e} ({derr / scale:.1e} of max|phi|)")
            assert derr <= 1e-3 * scale
        if oracle_solver == "cgls":
            # the residual creeps over the threshold slowly near the end, so round-off can move the
            # stopping iteration by a few steps; phi above is what has to agree
            assert abs(rep.cgls_iterations - ref["iterations"]) <= 2 + ref["iterations"] // 50
        # efficiency: sum(phi) = f(full) - f(empty)
        assert abs(got.sum() - (rep.f_full - rep.f_empty)) <= 1e-5
        assert abs(rep.f_full - ref["y"][1]) <= 1e-5 * (1 if dtype == 0 else 1e3)
    ctx.close()


def test_tiny_exact_config_equals_exact_shapley():
    from oracle import gcn, shapley
    _explain_case("c1", 1e-4)
    _explain_case("c1", 1e-4, solver="cgls")
    # and the oracle it is compared with equals brute-force Shapley on this config
    w = make_workload("c1")
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, 0, w.n_samples, w.seed)
    f = gcn.ValueFunction(ref["cg"], w.features, w.weights, dense=True)
    exact = shapley.exact_shapley(shapley.all_values(f, 12), 12)
    assert np.abs(ref["phi"] - exact).max() < 1e-8


def test_small_ba_config_gram_cholesky():
    _explain_case("c2_small", 1e-4)


def test_small_rmat_config_cgls():
    _explain_case("c3_small", 1e-4, oracle_solver="cgls")


def test_small_underdetermined_config_cgls_minimum_norm():
    _explain_case("c4_small", 1e-4, oracle_solver="cgls")


def test_small_hub_target_with_fan_out_cap():
    # a hub target: nearly every player is an entry of a row the first layer produces (the gather-heavy shape)
    _explain_case("c4b_small", 1e-4, oracle_solver="cgls")


def test_long_row_kernels_inside_an_explanation_with_and_without_player_lists():
    """The mask-streaming kernel forced on a reduced config (6,000 players: the one-pass sampler runs). By default the
    sampler then also writes the players of every sparse small member as a list, and the streaming kernel reads the
    lists instead of those bit rows; with the lists switched off it reads bits only. Both count the same integers:
    phi must be identical, and equal to the oracle's."""
    from paper_2506_22668_amd import Options, Tuning
    w = make_workload("c4_small")
    ctx = make_context(w)
    target = w.targets[0]
    opts = Options(solver=SOLVERS["cgls"], tol=w.tol)
    got = {}
    for lists in (0, -1):
        ctx.set_tuning(Tuning(eval_path=3, pair_lists=lists))
        say(f"explain c4_small target={target} eval_path=3 pair_lists={lists}")
        phi, _, _, rep, _ = ctx.explain(target, w.n_samples, w.seed, opts)
        assert rep.ms_k_stream > 0.0      # the streaming kernel did run
        got[lists] = phi.cpu().numpy()
    ctx.set_tuning(None)
    assert np.array_equal(got[0], got[-1])
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed, solver="cgls", tol=w.tol)
    err, scale = np.abs(got[0].astype(np.float64) - ref["phi"]).max(), np.abs(ref["phi"]).max()
    say(f"  n={ref['n']} k={ref['k']} max|phi|={scale:.3e} err={err:.3e}")
    assert err <= 1e-4 * scale
    ctx.close()


def test_layer_by_layer_block_kernels_inside_explanations():
    """The inference that goes layer by layer over blocks of 64 coalitions (transposed mask matrix), forced on reduced
    configs it would not be chosen for: fp32 with CGLS, and the bfloat16 transforms of the batched config (one target)."""
    _explain_case("c3_small", 1e-4, oracle_solver="cgls", eval_path=4)
    _explain_case("c5_small", 1e-2, targets=make_workload("c5_small").targets[:1], eval_path=4)


def test_underdetermined_config_direct_solver_reports_and_auto_falls_back():
    """Fewer rows than players: the direct solver inside ds_explain must report the singular system (its pivot
    flag only reaches the host with the final read-back), and solver AUTO must then give the minimum-norm
    solution of CGLS."""
    from paper_2506_22668_amd import DistShapError, DS_ESINGULAR, DS_SOLVER_CGLS, Options
    w = make_workload("c4_small")
    ctx = make_context(w)
    target = w.targets[0]
    say(f"explain c4_small target={target} with the direct solver and with AUTO")
    with pytest.raises(DistShapError) as e:
        ctx.explain(target, w.n_samples, w.seed, Options(solver=1))
    assert e.value.code == DS_ESINGULAR
    phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, Options(solver=0, tol=w.tol))
    assert rep.solver_used == DS_SOLVER_CGLS and rep.cgls_iterations > 0
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed, solver="cgls", tol=w.tol)
    scale = np.abs(ref["phi"]).max()
    assert np.abs(phi.cpu().numpy() - ref["phi"]).max() <= 1e-4 * scale
    ctx.close()


def test_uniform_weighting_option_matches_the_oracle():
    """ds_options.weighting = UNIFORM (every sampled row weighs 1): same masks, phi against the oracle run with
    the same option, both solvers; and it is a different estimate from the default one."""
    from paper_2506_22668_amd import Options
    w = make_workload("c2_small")
    ctx = make_context(w)
    target = w.targets[0]
    say(f"explain c2_small target={target} weighting=uniform")
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed, weighting="uniform")
    base = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed)
    scale = np.abs(ref["phi"]).max()
    for solver in (1, 2):
        phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, Options(solver=solver, tol=1e-10, weighting=1))
        got = phi.cpu().numpy().astype(np.float64)
        say(f"  solver={solver} err={np.abs(got - ref['phi']).max():.2e} (default estimate differs by {np.abs(ref['phi'] - base['phi']).max():.2e})")
        assert np.abs(got - ref["phi"]).max() <= 1e-4 * scale
    assert np.abs(ref["phi"] - base["phi"]).max() > 1e-4 * scale
    with pytest.raises(Exception):
        ctx.explain(target, w.n_samples, w.seed, Options(weighting=7))
    ctx.close()


def test_saturated_size_classes_option_matches_the_oracle():
    """ds_options.saturate end to end (the size-1 class of a 200-player game is enumerated): phi against the
    oracle run with the same option; it is a different estimate from the default one."""
    from paper_2506_22668_amd import Options
    w = make_workload("c2_small")
    ctx = make_context(w)
    target = w.targets[0]
    say(f"explain c2_small target={target} saturate=1")
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed, saturate=True)
    base = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, target, w.n_samples, w.seed)
    scale = np.abs(ref["phi"]).max()
    for solver in (1, 2):
        phi, es, ed, rep, rc = ctx.explain(target, w.n_samples, w.seed, Options(solver=solver, tol=1e-10, saturate=1))
        got = phi.cpu().numpy().astype(np.float64)
        say(f"  solver={solver} err={np.abs(got - ref['phi']).max():.2e} (default estimate differs by {np.abs(ref['phi'] - base['phi']).max():.2e})")
        assert np.abs(got - ref["phi"]).max() <= 1e-4 * scale
    assert np.abs(ref["phi"] - base["phi"]).max() > 1e-4 * scale
    ctx.close()


def test_small_batched_bf16_config():
    # bf16 per-coalition transforms against the plain fp64 oracle, at the tolerance stated for this configuration
    _explain_case("c5_small", 1e-2)


def test_full_ba_config_20000_coalitions():
    _explain_case("c2", 1e-4)


def test_explain_batch_equals_single_explanations():
    from paper_2506_22668_amd import Options, DS_ECAPACITY
    w = make_workload("c5_small")
    say("explain_batch c5_small")
    ctx = make_context(w, transform_dtype=1)
    singles = [ctx.explain(t, w.n_samples, w.seed)[0] for t in w.targets]
    total = sum(len(s) for s in singles)
    phi, M, off, es, ed, reps, rc = ctx.explain_batch(w.targets, w.n_samples, w.seed, capacity=total)
    assert rc == 0 and off[-1] == total and M == [len(s) for s in singles]
    for i, s in enumerate(singles):
        assert torch.equal(phi[off[i]:off[i + 1]], s)
    phi, M, off, es, ed, reps, rc = ctx.explain_batch(w.targets, w.n_samples, w.seed, capacity=len(singles[0]))
    assert rc == DS_ECAPACITY and off[-1] == total
    ctx.close()


def test_explain_batch_matches_the_oracle():
    """The batch entry point against the oracle itself (not against single HIP calls): fp32 transforms at 1e-4 of
    max|phi|, and the reduced-precision configuration at its 1e-2, every target of the batch."""
    w = make_workload("c5_small")
    for dtype, tol in ((0, 1e-4), (1, 1e-2)):
        say(f"explain_batch c5_small vs oracle, transform dtype {dtype}")
        ctx = make_context(w, transform_dtype=dtype)
        refs = [oexplain.explain(w.row_ptr, w.col, w.features, w.weights, t, w.n_samples, w.seed) for t in w.targets]
        total = sum(r["n"] for r in refs)
        phi, M, off, es, ed, reps, rc = ctx.explain_batch(w.targets, w.n_samples, w.seed, capacity=total)
        assert rc == 0 and M == [r["n"] for r in refs]
        for i, r in enumerate(refs):
            got = phi[off[i]:off[i + 1]].cpu().numpy().astype(np.float64)
            scale = np.abs(r["phi"]).max()
            err = np.abs(got - r["phi"]).max()
            say(f"  target {w.targets[i]}: n={r['n']} err={err:.3e} ({err / scale:.1e} of max|phi|)")
            assert err <= tol * scale
            assert np.array_equal(es[off[i]:off[i + 1]].cpu().numpy(), r["cg"]["edge_src"])
            assert np.array_equal(ed[off[i]:off[i + 1]].cpu().numpy(), r["cg"]["edge_dst"])
            assert reps[i].pred_class == r["pred_class"]
            assert abs(got.sum() - (reps[i].f_full - reps[i].f_empty)) <= 1e-5
        ctx.close()


def test_explain_batch_more_targets_than_workers_and_a_bad_target():
    """Targets outnumber the worker contexts (each worker takes several, sizes are published out of order and
    every result still lands at its offset); a target outside the graph anywhere in the batch is an error of the
    call, reported after the workers have drained (none of them may be left waiting for its size)."""
    from paper_2506_22668_amd import DistShapError, DS_EINVAL
    w = make_workload("c2_small")
    say("explain_batch 21 targets, then one bad target")
    ctx = make_context(w)
    rng = np.random.default_rng(5)
    targets = [int(t) for t in rng.choice(w.num_nodes, size=21, replace=False)]
    ns = 600
    singles = [ctx.explain(t, ns, w.seed)[0] for t in targets]
    total = sum(len(x) for x in singles)
    phi, M, off, es, ed, reps, rc = ctx.explain_batch(targets, ns, w.seed, capacity=total)
    assert rc == 0 and M == [len(x) for x in singles] and off[-1] == total
    for i, x in enumerate(singles):
        assert torch.equal(phi[off[i]:off[i + 1]], x)
    bad = targets[:5] + [w.num_nodes + 7] + targets[5:9]
    with pytest.raises(DistShapError) as e:
        ctx.explain_batch(bad, ns, w.seed, capacity=total)
    assert e.value.code == DS_EINVAL
    # the context is still usable
    again = ctx.explain(targets[0], ns, w.seed)[0]
    assert torch.equal(again, singles[0])
    ctx.close()


def test_degenerate_graphs_and_error_paths():
    from paper_2506_22668_amd import DistShapError, Options, DS_ECAPACITY, DS_EINVAL
    from synth.workloads import Workload
    say("explain degenerate")
    rp, ci = csr_from_undirected_edges(6, [0, 1, 4], [1, 2, 5])
    rng = np.random.default_rng(0)
    W = [rng.standard_normal((4, 3)).astype(np.float32), rng.standard_normal((3, 2)).astype(np.float32)]
    w = Workload("deg", 6, rp, ci, rng.standard_normal((6, 4), dtype=np.float32), (4, 3, 2), W, [3], 16, 1, "gram_chol")
    ctx = make_context(w)
    phi, es, ed, rep, rc = ctx.explain(3, 16, 1)                 # isolated: no players
    assert len(phi) == 0 and rep.num_players == 0
    phi, es, ed, rep, rc = ctx.explain(4, 16, 1)                 # one player: phi = delta
    ref = oexplain.explain(rp, ci, w.features, W, 4, 16, 1)
    assert ref["n"] == 1 and abs(float(phi[0]) - ref["phi"][0]) <= 1e-6
    phi, es, ed, rep, rc = ctx.explain(0, 16, 1)                 # two players: enumerated
    ref = oexplain.explain(rp, ci, w.features, W, 0, 16, 1)
    assert ref["n"] == 2 and np.abs(phi.cpu().numpy() - ref["phi"]).max() <= 1e-6
    w2 = make_workload("c2_small")
    ctx2 = make_context(w2)
    with pytest.raises(DistShapError) as e:
        ctx2.explain(w2.targets[0], 3, 1)
    assert e.value.code == DS_EINVAL
    with pytest.raises(DistShapError) as e:
        ctx2.explain(w2.targets[0], 100, 1, capacity=5)
    assert e.value.code == DS_ECAPACITY
    ctx.close()
    ctx2.close()


def test_directed_players_and_wider_extraction():
    """Directed players (one CSR entry each) and a computational graph wider than the receptive
    field: edges joining two nodes beyond L hops are exact null players."""
    from paper_2506_22668_amd import Options
    from oracle import compgraph
    say("explain directed / hops > L")
    w = make_workload("c1")
    ctx = make_context(w)
    # directed, 1-hop graph of the target: 8 players, enumerated
    phi, es, ed, rep, rc = ctx.explain(0, 1 << 8, 3, Options(hops=1, directed=1))
    ref = oexplain.explain(w.row_ptr, w.col, w.features, w.weights, 0, 1 << 8, 3, hops=1, undirected=False)
    assert rep.num_players == 8 and rep.enumerated == 1
    assert np.array_equal(es.cpu().numpy(), ref["cg"]["edge_src"]) and np.array_equal(ed.cpu().numpy(), ref["cg"]["edge_dst"])
    assert np.abs(phi.cpu().numpy() - ref["phi"]).max() <= 1e-4 * np.abs(ref["phi"]).max()
    ctx.close()
    # 2-layer model on a graph extracted to 3 hops: edge (3,4) joins two nodes at distance 3
    rp, ci = csr_from_undirected_edges(5, [0, 1, 2, 2, 3], [1, 2, 3, 4, 4])
    from synth.workloads import Workload
    rng = np.random.default_rng(2)
    W = [rng.standard_normal((6, 5)).astype(np.float32), rng.standard_normal((5, 3)).astype(np.float32)]
    wl = Workload("null", 5, rp, ci, rng.standard_normal((5, 6), dtype=np.float32), (6, 5, 3), W, [0], 32, 1, "gram_chol")
    ctx = make_context(wl)
    phi, es, ed, rep, rc = ctx.explain(0, 32, 1, Options(hops=3))
    ref = oexplain.explain(rp, ci, wl.features, W, 0, 32, 1, hops=3)
    pairs = list(zip(es.cpu().numpy().tolist(), ed.cpu().numpy().tolist()))
    got = phi.cpu().numpy()
    assert abs(got[pairs.index((3, 4))]) <= 1e-6
    assert abs(got[pairs.index((2, 3))]) > 1e-4
    assert np.abs(got - ref["phi"]).max() <= 1e-4 * np.abs(ref["phi"]).max() + 1e-7
    ctx.close()
