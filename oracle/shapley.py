"""Exact Shapley values by the definition (the paper's first equation):
  phi_i = sum over S subset of N \\ {i} of |S|! (n-|S|-1)! / n! * [f(S + i) - f(S)].
"""
from math import factorial
import numpy as np


def all_values(f, n):
    """f evaluated on every coalition, indexed by bit pattern (player j = bit j)."""
    vals = np.empty(1 << n, dtype=np.float64)
    for m in range(1 << n):
        vals[m] = f(np.array([(m >> j) & 1 for j in range(n)], dtype=bool))
    return vals


def exact_shapley(vals, n):
    coef = [factorial(s) * factorial(n - s - 1) / factorial(n) for s in range(n)]
    phi = np.zeros(n, dtype=np.float64)
    for i in range(n):
        bit = 1 << i
        for m in range(1 << n):
            if m & bit:
                continue
            s = bin(m).count("1")
            phi[i] += coef[s] * (vals[m | bit] - vals[m])
    return phi
