"""Kernel-SHAP regression: phi = argmin sum_i w_i (y_i - phi_0 - z_i . phi)^2
(the paper's weighted-regression equation with a linear surrogate), with the
two infinite-weight coalitions imposed as hard constraints: phi_0 = f(empty)
and sum(phi) = f(full) - f(empty) (the efficiency decomposition).

Rows 0 and 1 of the mask matrix are the empty and full coalitions; rows >= 2
are the weighted samples.  With delta = y_1 - y_0, psi = phi - delta/n (so psi
sums to zero), t_i = y_i - y_0 - (delta/n)|S_i| and P = I - 11^T/n, the problem
is  min || sqrt(w) (Z P psi - t) ||, and when it is rank-deficient the
minimum-norm psi is taken.
"""
import numpy as np


def _setup(Zbits, w, y):
    Zs = np.asarray(Zbits[2:], dtype=np.float64)
    ws = np.asarray(w[2:], dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = Zs.shape[1]
    f0, delta = y[0], y[1] - y[0]
    t = y[2:] - f0 - (delta / n) * Zs.sum(axis=1)
    return Zs, ws, t, n, f0, delta


def solve_lstsq(Zbits, w, y):
    """Library least squares on sqrt(w) Z P (minimum-norm solution)."""
    Zs, ws, t, n, f0, delta = _setup(Zbits, w, y)
    if n == 0:
        return np.zeros(0)
    sq = np.sqrt(ws)
    A = sq[:, None] * (Zs - Zs.mean(axis=1, keepdims=True))     # Z P
    psi = np.linalg.lstsq(A, sq * t, rcond=None)[0] if len(t) else np.zeros(n)
    return psi + delta / n


def solve_kkt(Zbits, w, y):
    """Normal equations with the efficiency constraint by a Lagrange
    multiplier: phi = phi_u - a (1.phi_u - delta)/(1.a), a = G^-1 1."""
    Zs = np.asarray(Zbits[2:], dtype=np.float64)
    ws = np.asarray(w[2:], dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = Zs.shape[1]
    f0, delta = y[0], y[1] - y[0]
    G = Zs.T @ (ws[:, None] * Zs)
    c = Zs.T @ (ws * (y[2:] - f0))
    phi_u = np.linalg.solve(G, c)
    a = np.linalg.solve(G, np.ones(n))
    return phi_u - a * (phi_u.sum() - delta) / a.sum()


def solve_cgls(Zbits, w, y, tol=1e-10, max_iter=None):
    """Conjugate gradients for least squares (the paper's CGLS algorithm in its
    standard Hestenes-Stiefel form, with the step ratio
    beta = |s_i|^2/|s_(i-1)|^2) on the matrix sqrt(w) Z P, started from zero.
    Returns (phi, iterations, final |s|/|s_0|)."""
    Zs, ws, t, n, f0, delta = _setup(Zbits, w, y)
    sq = np.sqrt(ws)
    if max_iter is None:
        max_iter = min(max(n, 1), 10000)

    def fwd(u):
        return sq * (Zs @ u)

    def adj(r):
        s = Zs.T @ (sq * r)
        return s - s.mean()

    x = np.zeros(n)
    r = sq * t
    s = adj(r)
    u = s.copy()
    gamma0 = gamma = float(s @ s)
    it, rel = 0, 1.0 if gamma0 > 0 else 0.0
    if gamma0 == 0.0:
        return x + delta / n, 0, 0.0
    while it < max_iter:
        v = fwd(u)
        dlt = float(v @ v)
        if dlt == 0.0:
            break
        theta = gamma / dlt
        x = x + theta * u
        r = r - theta * v
        s = adj(r)
        gnew = float(s @ s)
        it += 1
        rel = np.sqrt(gnew) / np.sqrt(gamma0)
        if rel <= tol:
            break
        u = s + (gnew / gamma) * u
        gamma = gnew
    return x + delta / n, it, rel
