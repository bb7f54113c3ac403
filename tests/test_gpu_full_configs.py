"""Configs 3, 4 and 5 at their full sizes, in the launch configuration bench.py uses.

The numpy oracle cannot finish these, so the plain-C restatement (oracle/oracle.c, itself tested
against the numpy oracle) is used, and only on what it can compute in seconds:
  * masks / weights / sizes: bit-exact on a stratified sample of pairs taken from the full mask
    matrix the GPU wrote, plus popcount and complement invariants on every row;
  * y: sampled rows, element by element;
  * phi: efficiency, and the normal-equation residual |P Z^T W (t - Z psi)| / |P Z^T W t| recomputed
    by the oracle from the GPU's phi (what CGLS must have driven below tol) for the CGLS configs;
    for the Gram+Cholesky config the oracle's converged CGLS solution on the same y (the
    least-squares solution is unique there). phi checks use the GPU's y (validated on samples),
    because the oracle needs hours for all rows.
"""
import numpy as np
import pytest

from oracle import cfast, compgraph
from synth import make_workload
from tests.gpu_common import make_context, say, to_u64

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _popcount_rows(Z):
    """popcount of every row of a torch int64 [k, W] tensor (on the device, in slabs)."""
    out = torch.empty(Z.shape[0], dtype=torch.int64, device=Z.device)
    m1, m2, m4 = 0x5555555555555555, 0x3333333333333333, 0x0F0F0F0F0F0F0F0F
    step = max(1, (1 << 26) // max(Z.shape[1], 1))
    for a in range(0, Z.shape[0], step):
        x = Z[a:a + step].clone()
        x = x - ((x >> 1) & m1)
        x = (x & m2) + ((x >> 2) & m2)
        x = (x + (x >> 4)) & m4
        x = (x * 0x0101010101010101) >> 56
        out[a:a + step] = (x & 0xFF).sum(dim=1)
    return out


def _stage_check(key, pair_stride, y_rows, check_residual=True):
    from paper_2506_22668_amd import Options, DS_SOLVER_CGLS, DS_SOLVER_GRAM_CHOL
    w = make_workload(key)
    bf16 = w.transform_dtype == "bf16"
    ctx = make_context(w, transform_dtype=1 if bf16 else 0)
    target = w.targets[0]
    say(f"{key}: extract target={target}")
    cg = ctx.extract(target)
    info = ctx.cgraph_info(cg)
    cgo = compgraph.extract(w.row_ptr, w.col, target, w.num_layers)
    n = cgo["num_players"]
    assert info.num_players == n and info.num_nodes == cgo["num_nodes"]
    es, ed = ctx.cgraph_edges(cg)
    assert np.array_equal(es.cpu().numpy(), cgo["edge_src"]) and np.array_equal(ed.cpu().numpy(), cgo["edge_dst"])

    say(f"{key}: sample n={n} k={w.n_samples}")
    Z, wt, sz = ctx.sample(n, w.n_samples, w.seed, target)
    k = Z.shape[0]
    K1 = k // 2
    # invariants on every row
    pc = _popcount_rows(Z)
    assert torch.equal(pc, sz.to(torch.int64))
    assert torch.equal(pc[0::2] + pc[1::2], torch.full((K1,), n, dtype=torch.int64, device=pc.device))
    tail = (1 << (n % 64)) - 1 if n % 64 else -1
    full = torch.full((Z.shape[1],), -1, dtype=torch.int64, device=Z.device)
    full[-1] = tail
    step = max(1, (1 << 25) // Z.shape[1])
    for a in range(0, K1, step):
        assert torch.equal(Z[2 * a:2 * (a + step):2] ^ Z[2 * a + 1:2 * (a + step):2],
                           full.expand(min(step, K1 - a), -1))
    assert torch.all(sz[2::2][1:] >= sz[2::2][:-1])          # pairs ascending by size
    # bit-exact against the oracle on a stratified sample of pairs
    pairs = np.unique(np.concatenate([np.arange(0, K1, pair_stride), [1, K1 - 1]]))
    say(f"{key}: oracle masks for {len(pairs)} pairs")
    rows = np.stack([2 * pairs, 2 * pairs + 1], axis=1).ravel()
    Zg = to_u64(Z[torch.from_numpy(rows).cuda()])
    wg, szg = wt.cpu().numpy()[rows], sz.cpu().numpy()[rows]
    for i, r in enumerate(pairs):
        Zo, wo, szo = cfast.sample(n, w.n_samples, w.seed, target, pair_range=(int(r), int(r) + 1))
        assert np.array_equal(Zo, Zg[2 * i:2 * i + 2]), f"pair {r}"
        assert np.array_equal(wo.view(np.uint32), wg[2 * i:2 * i + 2].view(np.uint32))
        assert np.array_equal(szo, szg[2 * i:2 * i + 2])

    say(f"{key}: eval all rows, oracle on {y_rows} of them")
    y, pcl = ctx.eval(cg, Z)
    sel = np.unique(np.concatenate([[0, 1, 2, 3, k - 2, k - 1],
                                    np.random.default_rng(1).integers(0, k, size=y_rows)]))
    yo, pco, _ = cfast.gcn_values(cgo, w.features, w.weights, to_u64(Z[torch.from_numpy(sel).cuda()]), bf16=bf16)
    assert pcl == pco
    err = np.abs(y.cpu().numpy()[sel].astype(np.float64) - yo).max()
    say(f"{key}: max |y - oracle| on sampled rows = {err:.3e}")
    assert err <= (1e-5 if not bf16 else 2e-5)

    say(f"{key}: solve")
    opts = Options(solver=DS_SOLVER_CGLS if w.solver == "cgls" else DS_SOLVER_GRAM_CHOL, tol=w.tol,
                   max_iter=w.max_iter, paired=1)
    phi, rep, rc = ctx.solve(n, Z, wt, y, opts)
    got = phi.cpu().numpy().astype(np.float64)
    yh = y.cpu().numpy().astype(np.float64)
    assert abs(got.sum() - (yh[1] - yh[0])) <= 1e-5
    say(f"{key}: solver={rep.solver_used} iterations={rep.cgls_iterations} rel={rep.cgls_rel_residual:.3e} "
        f"max|phi|={np.abs(got).max():.3e}")
    Zh = to_u64(Z)
    if w.solver == "cgls":
        assert rep.cgls_rel_residual <= w.tol
        if check_residual:
            res = cfast.normal_residual(n, Zh, wt.cpu().numpy(), yh, got)
            say(f"{key}: oracle-side residual of the GPU solution = {res:.3e}")
            # phi is rounded to fp32 on output: allow that rounding on top of tol
            assert res <= 2.0 * w.tol
    else:
        # 1e-11 is safely above where fp64 round-off stalls the recurrence on this size
        ref, it, rel = cfast.cgls(n, Zh, wt.cpu().numpy(), yh, tol=1e-11, max_iter=2000)
        assert rel <= 1e-11
        err = np.abs(got - ref).max()
        say(f"{key}: max |phi - oracle| = {err:.3e}")
        assert err <= 1e-4 * np.abs(ref).max()

    # the one-shot call gives the same answer as the stages
    say(f"{key}: one-shot explain")
    phi2, _, _, rep2, _ = ctx.explain(target, w.n_samples, w.seed,
                                      Options(solver=opts.solver, tol=w.tol, max_iter=w.max_iter), capacity=n,
                                      want_edges=False)
    assert torch.equal(phi2, phi)
    say(f"{key}: ms extract={rep2.ms_extract:.2f} sample={rep2.ms_sample:.2f} eval={rep2.ms_eval:.2f} "
        f"solve={rep2.ms_solve:.2f}")
    ctx.cgraph_free(cg)
    ctx.close()


def test_config3_rmat18_100k_players_cgls():
    _stage_check("c3", pair_stride=400, y_rows=48)


def test_config5_batched_bf16_gram_cholesky_first_target():
    _stage_check("c5", pair_stride=100, y_rows=48)


def test_config4_rmat20_1m_players_underdetermined_cgls():
    _stage_check("c4", pair_stride=5000, y_rows=16)
