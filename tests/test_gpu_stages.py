"""Stage-by-stage parity of the HIP path (called through the C ABI) with the CPU oracle."""
import numpy as np
import pytest

from oracle import compgraph, gcn, sampling, solve
from synth import csr_from_undirected_edges, make_workload
from tests.gpu_common import make_context, say, to_u64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ctx_tiny():
    w = make_workload("c1")
    ctx = make_context(w)
    yield ctx, w
    ctx.close()


# ---------------------------------------------------------------- sampler: bit-exact
@pytest.mark.parametrize("n,ns,seed,tag", [
    (12, 4096, 1, 0),            # enumeration
    (2, 4, 1, 0), (3, 100, 7, 1), (24, 5000, 3, 9),
    (30, 2000, 5, 3), (64, 1000, 11, 4), (65, 1000, 12, 5), (130, 3001, 2 ** 40 + 17, 2 ** 31 + 5),
    (255, 777, 1, 1), (256, 778, 1, 1), (257, 4, 1, 1),
    (1000, 20000, 22668002, 7965), (5000, 3000, 9, 10), (40000, 600, 13, 77),
    (4096, 500, 21, 3), (4099, 700, 23, 4), (6241, 9000, 25, 5),   # the one-pass kernel (4,096 players and more)
])
def test_sampler_bit_exact(ctx_tiny, n, ns, seed, tag):
    ctx, _ = ctx_tiny
    say(f"sampler n={n} n_samples={ns} seed={seed} tag={tag}")
    Z, w, sz = ctx.sample(n, ns, seed, tag)
    Zo, wo, szo = sampling.sample(n, ns, seed, tag)
    assert np.array_equal(to_u64(Z), Zo)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), wo.view(np.uint32))
    assert np.array_equal(sz.cpu().numpy(), szo)


@pytest.mark.parametrize("window", [-1, 3])
def test_sampler_four_pass_route_gives_the_same_masks(ctx_tiny, window):
    from paper_2506_22668_amd import Tuning
    ctx, _ = ctx_tiny
    say(f"sampler forced fallback window={window}")
    ctx.set_tuning(Tuning(sampler_window=window))
    try:
        for n, ns in [(300, 2000), (5000, 600)]:
            Z, w, sz = ctx.sample(n, ns, 31, 8)
            Zo, wo, szo = sampling.sample(n, ns, 31, 8)
            assert np.array_equal(to_u64(Z), Zo)
            assert np.array_equal(sz.cpu().numpy(), szo)
    finally:
        ctx.set_tuning(None)


@pytest.mark.parametrize("n,ns", [(30, 25000), (200, 3000), (12, 1000), (9, 510), (1010, 20000), (333, 70000)])
def test_sampler_with_saturated_size_classes_bit_exact(ctx_tiny, n, ns):
    """ds_options.saturate: size classes allotted at least C(n, s) pairs are enumerated (subsets in lexicographic
    order, kernel weights); masks, weights and sizes against the oracle run with the same option."""
    from paper_2506_22668_amd import Options, DistShapError
    ctx, _ = ctx_tiny
    say(f"sampler saturate n={n} n_samples={ns}")
    Z, w, sz = ctx.sample(n, ns, 11, 5, Options(saturate=1))
    Zo, wo, szo = sampling.sample(n, ns, 11, 5, saturate=True)
    assert sampling.allocation(n, ns, saturate=True)["enum_upto"] >= 1
    assert np.array_equal(to_u64(Z), Zo)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), wo.view(np.uint32))
    assert np.array_equal(sz.cpu().numpy(), szo)
    with pytest.raises(DistShapError):
        ctx.sample(n, ns, 11, 5, Options(saturate=1, weighting=1))


def test_sampler_pair_ranges_equal_the_full_run(ctx_tiny):
    ctx, _ = ctx_tiny
    n, ns, seed, tag = 333, 5000, 99, 3
    say("sampler ranges")
    Z, w, sz = ctx.sample(n, ns, seed, tag)
    for r0, r1 in [(0, 1), (0, 100), (100, 1777), (1777, 2500), (5, 5)]:
        Zp, wp, szp = ctx.sample_range(n, ns, seed, tag, r0, r1)
        assert torch.equal(Zp, Z[2 * r0:2 * r1])
        assert torch.equal(wp, w[2 * r0:2 * r1])
        assert torch.equal(szp, sz[2 * r0:2 * r1])


def test_sampler_rejects_bad_arguments(ctx_tiny):
    from paper_2506_22668_amd import DistShapError, DS_EINVAL
    ctx, _ = ctx_tiny
    say("sampler errors")
    with pytest.raises(DistShapError) as e:
        ctx.sample(100, 3, 1, 1)
    assert e.value.code == DS_EINVAL
    with pytest.raises(DistShapError) as e:
        ctx.sample(1, 10, 1, 1)
    assert e.value.code == DS_EINVAL
    with pytest.raises(DistShapError) as e:
        ctx.sample_range(100, 50, 1, 1, 3, 26)
    assert e.value.code == DS_EINVAL


# ---------------------------------------------------------------- extraction: exact
def _check_extraction(ctx, w, target, hops, directed):
    from paper_2506_22668_amd import Options
    cgo = compgraph.extract(w.row_ptr, w.col, target, hops, undirected=not directed)
    cg = ctx.extract(target, Options(hops=hops, directed=int(directed)))
    info = ctx.cgraph_info(cg)
    assert info.num_players == cgo["num_players"]
    assert info.num_nodes == cgo["num_nodes"]
    assert list(info.ball[:hops + 1]) == cgo["ball"]
    gid, hop = ctx.cgraph_nodes(cg)
    assert np.array_equal(gid.cpu().numpy(), cgo["node_gid"])
    assert np.array_equal(hop.cpu().numpy(), cgo["hop"])
    es, ed = ctx.cgraph_edges(cg)
    assert np.array_equal(es.cpu().numpy(), cgo["edge_src"])
    assert np.array_equal(ed.cpu().numpy(), cgo["edge_dst"])
    return cg, cgo


@pytest.mark.parametrize("key,hops,directed", [
    ("c1", 2, False), ("c1", 1, False), ("c1", 3, False), ("c1", 2, True),
    ("c2_small", 3, False), ("c2_small", 2, True), ("c2_small", 4, False),
    ("c3_small", 3, False), ("c4_small", 3, False), ("c4_small", 1, True),
])
def test_extraction_matches_oracle(key, hops, directed):
    w = make_workload(key)
    say(f"extract {key} hops={hops} directed={directed}")
    ctx = make_context(w)
    for target in w.targets[:2]:
        cg, _ = _check_extraction(ctx, w, target, hops, directed)
        ctx.cgraph_free(cg)
    ctx.close()


def test_extraction_isolated_and_pendant_targets():
    # node 3 is isolated (no players); node 2 hangs off node 1 (one player at 1 hop)
    rp, ci = csr_from_undirected_edges(5, [0, 1], [1, 2])
    from synth.workloads import Workload
    rng = np.random.default_rng(0)
    w = Workload("iso", 5, rp, ci, rng.standard_normal((5, 4), dtype=np.float32), (4, 3, 2),
                 [rng.standard_normal((4, 3)).astype(np.float32), rng.standard_normal((3, 2)).astype(np.float32)],
                 [3], 16, 1, "gram_chol")
    say("extract isolated")
    ctx = make_context(w)
    cg, cgo = _check_extraction(ctx, w, 3, 2, False)
    assert cgo["num_players"] == 0
    ctx.cgraph_free(cg)
    cg, cgo = _check_extraction(ctx, w, 2, 1, False)
    assert cgo["num_players"] == 1
    ctx.cgraph_free(cg)
    ctx.close()


def test_malformed_graphs_are_rejected():
    from paper_2506_22668_amd import Context, DistShapError, DS_EINVAL, Options
    say("graph validation")
    ctx = Context("cuda:0")
    bad = [
        (np.array([0, 2, 1, 3]), np.array([1, 2, 0])),          # row_ptr not monotone
        (np.array([0, 2, 3, 3]), np.array([2, 1, 0])),          # row not ascending
        (np.array([0, 2, 3, 3]), np.array([1, 1, 0])),          # duplicate
        (np.array([0, 1, 2, 3]), np.array([1, 7, 0])),          # id out of range
        (np.array([1, 1, 2, 3]), np.array([1, 2, 0])),          # row_ptr[0] != 0
    ]
    for rp, ci in bad:
        with pytest.raises(DistShapError) as e:
            ctx.set_graph(rp, ci)
        assert e.value.code == DS_EINVAL
    # asymmetric CSR: fine for directed players, an error for undirected ones
    ctx.set_graph(np.array([0, 1, 1]), np.array([1]))
    ctx.set_features(np.zeros((2, 3), dtype=np.float32))
    ctx.set_gcn([np.zeros((3, 2), dtype=np.float32)])
    with pytest.raises(DistShapError) as e:
        ctx.extract(0, Options(hops=1))
    assert e.value.code == DS_EINVAL
    cg = ctx.extract(0, Options(hops=1, directed=1))
    assert ctx.cgraph_info(cg).num_players == 1
    ctx.cgraph_free(cg)
    with pytest.raises(DistShapError):
        ctx.extract(5, Options(hops=1))
    ctx.close()


# ---------------------------------------------------------------- shared first transform (MFMA)
@pytest.mark.parametrize("key,dtype,tol", [("c1", 0, 2e-6), ("c2_small", 0, 2e-6), ("c3_small", 0, 2e-6),
                                           ("c2", 0, 5e-6), ("c5_small", 1, 2e-2)])
def test_first_transform_matches_matmul(key, dtype, tol):
    w = make_workload(key)
    say(f"first transform {key} dtype={dtype}")
    ctx = make_context(w, transform_dtype=dtype)
    cg = ctx.extract(w.targets[0])
    gid, _ = ctx.cgraph_nodes(cg)
    P = ctx.cgraph_first_transform(cg).cpu().numpy().astype(np.float64)
    ref = w.features[gid.cpu().numpy()].astype(np.float64) @ w.weights[0].astype(np.float64)
    scale = np.abs(ref).max()
    assert np.abs(P - ref).max() <= tol * scale
    ctx.cgraph_free(cg)
    ctx.close()


# ---------------------------------------------------------------- masked inference
def _eval_case(w, hops, directed, score, biases, rows, rng, tol=1e-5, layers=None):
    from paper_2506_22668_amd import Options
    weights = w.weights if layers is None else w.weights[:layers]
    if layers is not None:
        w = type(w)(**{**w.__dict__, "weights": weights, "dims": w.dims[:layers + 1]})
    ctx = make_context(w, biases=biases)
    target = w.targets[0]
    cg = ctx.extract(target, Options(hops=hops, directed=int(directed)))
    cgo = compgraph.extract(w.row_ptr, w.col, target, hops, undirected=not directed)
    n = cgo["num_players"]
    f = gcn.ValueFunction(cgo, w.features, weights, biases, "logit" if score else "prob")
    bits = np.zeros((rows, n), dtype=bool)
    bits[1] = True
    for i in range(2, rows):
        bits[i] = rng.random(n) < rng.random() ** 2
    bits[rows - 1] = ~bits[rows - 2]
    Z = torch.from_numpy(sampling.pack_rows(bits).view(np.int64)).cuda()
    ref = f.batch(bits)
    scale = max(1.0, np.abs(ref).max())
    # every inference kernel on the same rows: the size-based choice, then each kernel forced (one workgroup per
    # coalition; one coalition per lane with the masks on chip; the mask-streaming kernel + layers on its output;
    # layer by layer over blocks of 64 coalitions from the transposed mask matrix)
    from paper_2506_22668_amd import Tuning
    for path in (0, 1, 2, 3, 4):
        ctx.set_tuning(Tuning(eval_path=path))
        y, pc = ctx.eval(cg, Z, score)
        assert pc == f.pred_class
        err = np.abs(y.cpu().numpy().astype(np.float64) - ref).max()
        assert err <= tol * scale, f"path {path}: max |y - oracle| = {err}"
    # rows as complementary pairs (only the even rows are read): masks 2r+1 = complement of 2r
    if rows % 2 == 0 and n > 0:
        pbits = bits.copy()
        pbits[1::2] = ~pbits[0::2]
        Zp = torch.from_numpy(sampling.pack_rows(pbits).view(np.int64)).cuda()
        refp = f.batch(pbits)
        for path in (0, 3, 4):
            ctx.set_tuning(Tuning(eval_path=path))
            y, pc = ctx.eval(cg, Zp, score, pairs=True)
            err = np.abs(y.cpu().numpy().astype(np.float64) - refp).max()
            assert err <= tol * max(1.0, np.abs(refp).max()), f"pairs, path {path}: max |y - oracle| = {err}"
    ctx.cgraph_free(cg)
    ctx.close()


@pytest.mark.parametrize("key,hops,directed,score,with_bias,layers", [
    ("c1", 2, False, 0, False, None), ("c1", 2, False, 1, True, None), ("c1", 3, False, 0, False, None),
    ("c1", 1, False, 0, False, None), ("c1", 2, True, 0, True, None), ("c1", 2, False, 0, False, 1),
    ("c2_small", 3, False, 0, False, None), ("c2_small", 3, False, 1, True, None),
    ("c2_small", 4, False, 0, False, None), ("c2_small", 2, False, 0, False, 2),
    ("c2_small", 3, True, 0, False, None),
    ("c3_small", 3, False, 0, False, None), ("c4_small", 3, False, 1, False, None),
])
def test_masked_inference_matches_oracle(key, hops, directed, score, with_bias, layers):
    w = make_workload(key)
    say(f"eval {key} hops={hops} directed={directed} score={score} bias={with_bias} layers={layers}")
    rng = np.random.default_rng(5)
    biases = None
    if with_bias:
        L = layers or w.num_layers
        biases = [0.1 * rng.standard_normal(w.dims[l + 1]).astype(np.float32) for l in range(L)]
    # 96 rows go through the one-workgroup-per-coalition kernel; 320 rows through the
    # one-coalition-per-lane kernel when the graph has at most 2048 players
    _eval_case(w, hops, directed, score, biases, 96, rng, layers=layers)
    _eval_case(w, hops, directed, score, biases, 320, rng, layers=layers)


def test_masked_inference_all_enumerated_rows_tiny(ctx_tiny):
    ctx, w = ctx_tiny
    say("eval c1 all 4096 rows")
    cg = ctx.extract(0)
    Z, wt, sz = ctx.sample(12, 4096, w.seed, 0)
    y, pc = ctx.eval(cg, Z)
    cgo = compgraph.extract(w.row_ptr, w.col, 0, 2)
    f = gcn.ValueFunction(cgo, w.features, w.weights)
    ref = f.batch(sampling.unpack_rows(to_u64(Z), 12))
    assert np.abs(y.cpu().numpy() - ref).max() <= 1e-5
    ctx.cgraph_free(cg)


# ---------------------------------------------------------------- solvers
def _solve_inputs(n, ns, seed):
    rng = np.random.default_rng(seed)
    Z, w, sz = sampling.sample(n, ns, seed, 3)
    bits = sampling.unpack_rows(Z, n)
    a = rng.standard_normal(n) / np.sqrt(n)
    y = (0.2 + bits @ a + 0.1 * np.tanh(bits @ rng.standard_normal(n))).astype(np.float32)
    return Z, w, bits, y


# sizes around the factorisation's block edges too: one block exactly (64), a block and one column (65), whole blocks
# only (128, 192: the last fused step is followed by a full last block), a last block of one column (129)
@pytest.mark.parametrize("n,ns", [(12, 4096), (40, 2000), (63, 3000), (64, 3000), (65, 3000), (128, 4000), (129, 4000),
                                  (192, 4000), (200, 3000), (333, 6000), (1000, 20000)])
def test_gram_cholesky_matches_oracle_least_squares(ctx_tiny, n, ns):
    from paper_2506_22668_amd import Options, DS_SOLVER_GRAM_CHOL
    ctx, _ = ctx_tiny
    say(f"gram+chol n={n} n_samples={ns}")
    Z, w, bits, y = _solve_inputs(n, ns, 100 + n)
    ref = solve.solve_lstsq(bits, w, y)
    phi, rep, rc = ctx.solve(n, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(),
                             torch.from_numpy(y).cuda(), Options(solver=DS_SOLVER_GRAM_CHOL))
    assert rep.solver_used == DS_SOLVER_GRAM_CHOL
    got = phi.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max()
    assert abs(got.sum() - (float(y[1]) - float(y[0]))) <= 1e-5 * max(1.0, abs(float(y[1]) - float(y[0])))


@pytest.mark.parametrize("n,ns,paired", [(12, 4096, 1), (40, 2000, 0), (40, 2000, 1), (333, 6000, 1),
                                         (1000, 20000, 1), (1000, 20000, 0), (3000, 1000, 1), (3000, 1000, 0),
                                         # >= 4096 players and paired: index lists + the matrix-core product of the dense rows
                                         (4100, 3000, 1), (6000, 14000, 1), (4097, 130, 1), (5000, 2000, 0),
                                         # exactly one 8192-column chunk / one column more; more than 8192 sparse
                                         # rows (several row blocks of tile entries)
                                         (8192, 3000, 1), (8193, 9000, 1), (5000, 40000, 1)])
def test_cgls_matches_oracle(ctx_tiny, n, ns, paired):
    from paper_2506_22668_amd import Options, DS_SOLVER_CGLS
    ctx, _ = ctx_tiny
    say(f"cgls n={n} n_samples={ns} paired={paired}")
    Z, w, bits, y = _solve_inputs(n, ns, 200 + n)
    ref, it_ref, _ = solve.solve_cgls(bits, w, y, tol=1e-12)
    phi, rep, rc = ctx.solve(n, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(),
                             torch.from_numpy(y).cuda(), Options(solver=DS_SOLVER_CGLS, tol=1e-9, paired=paired))
    got = phi.cpu().numpy().astype(np.float64)
    assert rep.cgls_rel_residual <= 1e-9
    assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max()
    if n <= 1000:   # well-determined: also the dense least-squares answer
        assert np.abs(got - solve.solve_lstsq(bits, w, y)).max() <= 1e-4 * np.abs(ref).max()


@pytest.mark.parametrize("dense_div", [32, 1024, 65536])
def test_cgls_dense_row_threshold_leaves_the_solution_alone(ctx_tiny, dense_div):
    """Which pair rows are multiplied as bitmaps on the matrix cores and which as index lists is a tuning choice:
    nearly all dense (65536), the built-in split, nearly all sparse (32). 6,200 players: rows of 97 words, so the last
    1024-column chunk is short and the transposed copy has an odd number of words per row."""
    from paper_2506_22668_amd import Options, DS_SOLVER_CGLS
    from paper_2506_22668_amd.binding import Tuning
    ctx, _ = ctx_tiny
    n, ns = 6200, 8250
    say(f"cgls dense_div={dense_div}")
    Z, w, bits, y = _solve_inputs(n, ns, 77)
    ref, _, _ = solve.solve_cgls(bits, w, y, tol=1e-12)
    args = (n, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(y).cuda(),
            Options(solver=DS_SOLVER_CGLS, tol=1e-9, paired=1))
    base, rep0, _ = ctx.solve(*args)
    try:
        ctx.set_tuning(Tuning(cgls_dense_div=dense_div))
        phi, rep, _ = ctx.solve(*args)
    finally:
        ctx.set_tuning(None)
    assert rep.cgls_rel_residual <= 1e-9
    got = phi.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max()
    assert np.abs(got - base.cpu().numpy()).max() <= 1e-6 * np.abs(ref).max()
    assert abs(rep.cgls_iterations - rep0.cgls_iterations) <= 2


def test_cgls_one_iteration_under_enumeration(ctx_tiny):
    from paper_2506_22668_amd import Options, DS_SOLVER_CGLS
    ctx, _ = ctx_tiny
    say("cgls enumeration one step")
    Z, w, bits, y = _solve_inputs(10, 1 << 10, 5)
    phi, rep, rc = ctx.solve(10, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(),
                             torch.from_numpy(y).cuda(), Options(solver=DS_SOLVER_CGLS, tol=1e-6, paired=1))
    assert rep.cgls_iterations == 1


def test_cgls_reports_non_convergence(ctx_tiny):
    from paper_2506_22668_amd import Options, DS_SOLVER_CGLS, DS_ENOTCONV
    ctx, _ = ctx_tiny
    say("cgls max_iter")
    Z, w, bits, y = _solve_inputs(200, 3000, 6)
    phi, rep, rc = ctx.solve(200, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(),
                             torch.from_numpy(y).cuda(), Options(solver=DS_SOLVER_CGLS, tol=1e-14, max_iter=2, paired=1),
                             allow_not_converged=True)
    assert rc == DS_ENOTCONV and rep.cgls_iterations == 2
    ref2 = solve.solve_cgls(bits, w, y, tol=1e-30, max_iter=2)[0]
    assert np.abs(phi.cpu().numpy() - ref2).max() <= 1e-4 * np.abs(ref2).max()


def test_gram_cholesky_mid_size_crosses_every_factorisation_regime(ctx_tiny):
    """2,700 players: the factorisation starts with super-panels of 256 columns (one wide trailing update each),
    continues with single blocks and ends with the steps whose update factorises the next diagonal block; the
    back substitution takes one launch per block."""
    from paper_2506_22668_amd import Options, DS_SOLVER_GRAM_CHOL
    ctx, _ = ctx_tiny
    n, ns = 2700, 9000
    say(f"gram+chol n={n} n_samples={ns}")
    Z, w, bits, y = _solve_inputs(n, ns, 77)
    ref = solve.solve_lstsq(bits, w, y)
    phi, rep, rc = ctx.solve(n, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(),
                             torch.from_numpy(y).cuda(), Options(solver=DS_SOLVER_GRAM_CHOL, paired=1))
    got = phi.cpu().numpy().astype(np.float64)
    err = np.abs(got - ref).max()
    say(f"  err={err:.2e} max|phi|={np.abs(ref).max():.2e}")
    assert err <= 1e-4 * np.abs(ref).max()


def test_rank_deficient_gram_is_reported_and_auto_falls_back(ctx_tiny):
    from paper_2506_22668_amd import Options, DistShapError, DS_SOLVER_GRAM_CHOL, DS_SOLVER_CGLS, DS_ESINGULAR
    ctx, _ = ctx_tiny
    say("singular gram")
    Z, w, bits, y = _solve_inputs(300, 40, 8)      # 38 weighted rows for 300 players
    args = (300, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(y).cuda())
    with pytest.raises(DistShapError) as e:
        ctx.solve(*args, Options(solver=DS_SOLVER_GRAM_CHOL))
    assert e.value.code == DS_ESINGULAR
    phi, rep, rc = ctx.solve(*args, Options(tol=1e-10, paired=1))
    assert rep.solver_used == DS_SOLVER_CGLS
    ref = solve.solve_lstsq(bits, w, y)
    assert np.abs(phi.cpu().numpy() - ref).max() <= 1e-4 * np.abs(ref).max()


@pytest.mark.parametrize("n,ns", [(150, 1000), (400, 3000)])
def test_gram_with_one_lost_direction_is_reported_and_auto_falls_back(ctx_tiny, n, ns):
    """Nullity one: two players that appear together in every sampled row (column n-1 is made a copy of column
    n-2). Exact arithmetic gives one zero pivot; in fp64 it comes out as round-off of either sign, which only a
    relative test catches. The direct solver must report the singular system, AUTO must return the minimum-norm
    solution (the oracle's projected least-squares solution)."""
    from paper_2506_22668_amd import Options, DistShapError, DS_SOLVER_GRAM_CHOL, DS_SOLVER_CGLS, DS_ESINGULAR
    ctx, _ = ctx_tiny
    say(f"gram nullity 1 n={n}")
    Z, w, bits, y = _solve_inputs(n, ns, 300 + n)
    bits = bits.copy()
    bits[2:, n - 1] = bits[2:, n - 2]
    Z = sampling.pack_rows(bits)
    args = (n, torch.from_numpy(Z.view(np.int64)).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(y).cuda())
    with pytest.raises(DistShapError) as e:
        ctx.solve(*args, Options(solver=DS_SOLVER_GRAM_CHOL))
    assert e.value.code == DS_ESINGULAR
    phi, rep, rc = ctx.solve(*args, Options(tol=1e-11))
    assert rep.solver_used == DS_SOLVER_CGLS
    ref = solve.solve_lstsq(bits, w, y)
    got = phi.cpu().numpy().astype(np.float64)
    assert abs(ref[n - 1] - ref[n - 2]) <= 1e-9            # minimum norm splits the pair's share evenly
    assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max()
