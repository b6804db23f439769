"""Dense NumPy/SciPy brute force on explicit n x m matrices (tiny inputs only).

Test infrastructure.  It exists to cross-check ``fs_oracle.c``: same
definitions (Section 2.1, Eq. 1-5 of the paper), but written with whole-matrix
library calls (``scipy.special.logsumexp``, matrix products) instead of loops.
"""
from __future__ import annotations

import numpy as np
from scipy.special import logsumexp


def cost(x, y):
    """C_ij = |x_i - y_j|^2 by explicit differences."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    diff = x[:, None, :] - y[None, :, :]
    return np.einsum("ijk,ijk->ij", diff, diff)


def update_f(C, b, eps, g):
    """Eq. 2."""
    return -eps * logsumexp((g[None, :] - C) / eps + np.log(b)[None, :], axis=1)


def update_g(C, a, eps, f):
    """Eq. 3."""
    return -eps * logsumexp((f[:, None] - C) / eps + np.log(a)[:, None], axis=0)


def solve(x, y, a, b, eps_list, iters):
    """Alternating schedule; eps_list gives the eps of each stage."""
    C = cost(x, y)
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    f = np.zeros(C.shape[0])
    g = np.zeros(C.shape[1])
    for eps in eps_list:
        for _ in range(iters):
            f = update_f(C, b, eps, g)
            g = update_g(C, a, eps, f)
    return f, g


def solve_symmetric(x, y, a, b, eps, iters):
    """Eq. 4-5."""
    C = cost(x, y)
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    f = np.zeros(C.shape[0])
    g = np.zeros(C.shape[1])
    for _ in range(iters):
        fn = update_f(C, b, eps, g)
        gn = update_g(C, a, eps, f)
        f, g = 0.5 * (f + fn), 0.5 * (g + gn)
    return f, g


def plan(x, y, a, b, eps, f, g):
    """P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps)."""
    C = cost(x, y)
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return a[:, None] * b[None, :] * np.exp((f[:, None] + g[None, :] - C) / eps)


def primal(x, y, a, b, eps, P):
    """Eq. 1 objective for a given plan (generalised KL with the -P + ab terms)."""
    C = cost(x, y)
    ab = np.outer(a, b)
    with np.errstate(divide="ignore", invalid="ignore"):
        ent = np.where(P > 0, P * np.log(P / ab), 0.0)
    return float((C * P).sum() + eps * (ent - P + ab).sum())
