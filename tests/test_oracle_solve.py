"""Pins for the oracle's least-squares solvers."""
import numpy as np
import pytest

from oracle import sampling, solve


def _game(n, ns, seed, linear=False):
    rng = np.random.default_rng(seed)
    Z, w, sz = sampling.sample(n, ns, seed, 1)
    bits = sampling.unpack_rows(Z, n)
    a = rng.standard_normal(n)
    y = 0.25 + bits @ a
    if not linear:
        y = y + 0.3 * np.sin(bits @ rng.standard_normal(n))
    return bits, w, y, a


def test_linear_game_is_recovered_exactly():
    bits, w, y, a = _game(15, 600, 1, linear=True)
    for phi in (solve.solve_lstsq(bits, w, y), solve.solve_kkt(bits, w, y),
                solve.solve_cgls(bits, w, y)[0]):
        assert np.allclose(phi, a, atol=1e-9)


def test_three_solvers_agree_and_satisfy_efficiency():
    bits, w, y, _ = _game(20, 3000, 2)
    p1 = solve.solve_lstsq(bits, w, y)
    p2 = solve.solve_kkt(bits, w, y)
    p3, it, rel = solve.solve_cgls(bits, w, y)
    assert np.allclose(p1, p2, atol=1e-10)
    assert np.allclose(p1, p3, atol=1e-8)
    assert rel <= 1e-10 and it <= 20
    for p in (p1, p2, p3):
        assert p.sum() == pytest.approx(y[1] - y[0], abs=1e-12)


def test_constrained_minimiser_by_brute_force_perturbation():
    # the solution must beat any feasible perturbation of itself
    bits, w, y, _ = _game(8, 400, 3)
    phi = solve.solve_lstsq(bits, w, y)

    def loss(p):
        r = y[2:] - y[0] - bits[2:] @ p
        return float((w[2:] * r * r).sum())

    rng = np.random.default_rng(0)
    base = loss(phi)
    for _ in range(50):
        d = rng.standard_normal(8)
        d -= d.mean()                      # stay on sum(phi) = delta
        assert loss(phi + 1e-3 * d) >= base


def test_underdetermined_gives_minimum_norm_deviation():
    # fewer rows than players: among all minimisers the one closest to delta/n
    n, ns = 40, 24
    bits, w, y, _ = _game(n, ns, 4)
    phi_l = solve.solve_lstsq(bits, w, y)
    phi_c, it, rel = solve.solve_cgls(bits, w, y, tol=1e-13)
    assert np.allclose(phi_l, phi_c, atol=1e-9)
    delta = y[1] - y[0]
    sq = np.sqrt(w[2:].astype(np.float64))
    A = sq[:, None] * (bits[2:] - bits[2:].mean(axis=1, keepdims=True))
    t = y[2:] - y[0] - delta / n * bits[2:].sum(axis=1)
    psi = np.linalg.pinv(A) @ (sq * t)
    assert np.allclose(phi_l, psi + delta / n, atol=1e-9)
    # minimum norm: no component in the null space of the matrix
    U, sv, Vt = np.linalg.svd(A)
    rank = int((sv > 1e-10 * sv[0]).sum())
    assert rank < n - 1
    assert np.abs(Vt[rank:] @ (phi_l - delta / n)).max() < 1e-9


def test_cgls_takes_one_iteration_under_enumeration():
    # with kernel weights over all coalitions the projected Gram is a multiple
    # of the projector, so the first step lands on the solution
    n = 9
    Z, w, sz = sampling.sample(n, 1 << n, 0, 0)
    bits = sampling.unpack_rows(Z, n)
    rng = np.random.default_rng(6)
    y = rng.standard_normal(1 << n)
    phi, it, rel = solve.solve_cgls(bits, w, y, tol=1e-6)
    assert it == 1 and rel < 1e-6
    assert np.allclose(phi, solve.solve_lstsq(bits, w, y), atol=1e-7)
