"""Dense float64 Hessian-vector product of the entropic OT value with respect to the source
cloud (test infrastructure; small n, m only: it forms the n x m plan and (n+m) x (n+m) systems).

Follows Section 3.3 / App. E of the paper (Thm. 5 and its proof), with whole-matrix NumPy calls:
    G = T A = (1/eps) R^T w + E A,     w = H^+ (R A),     H = [[diag(r), P], [P^T, diag(c)]]
where P is the plan induced by the potentials (text after Eq. 3) and r = P 1, c = P^T 1 are its
own marginals (the appendix on implementation uses the induced marginals throughout, so that
the formulas stay consistent for potentials that are not converged; at convergence r = a, c = b).
  explicit term   E A = B1 - (4/eps)(B2 - B3 - B4 + B5)          (App. E.1)
  right-hand side R A = (r1, r2)                                   (App. E.2, step 1)
  Schur system    (diag(c) - P^T diag(r)^-1 P + tau I) w2 = r2 - P^T (r1 / r)    (step 2)
  back to G       R^T w                                            (step 3)
tau = 0 takes the Moore-Penrose solution of the full system instead of the Schur complement.
Pinned in tests/test_oracle_pins.py: hvp by central differences of the gradient of Cor. 4 at
converged potentials (which shares none of these formulas); hadamard_transport by the entry-by-entry
double loop and by the special direction A_i = e_k, which turns it into an ordinary plan
application computed by the C oracle.
"""
from __future__ import annotations

import numpy as np


def _plan(x, y, a, b, eps, f, g):
    diff = x[:, None, :] - y[None, :, :]
    C = np.einsum("ijk,ijk->ij", diff, diff)
    return a[:, None] * b[None, :] * np.exp((f[:, None] + g[None, :] - C) / eps)


def hvp(x, y, a, b, eps, f, g, A, tau=0.0):
    x, y, A = (np.asarray(v, dtype=np.float64) for v in (x, y, A))
    a, b, f, g = (np.asarray(v, dtype=np.float64) for v in (a, b, f, g))
    n, m = len(x), len(y)
    P = _plan(x, y, a, b, eps, f, g)
    r, c = P.sum(1), P.sum(0)
    PY = P @ y
    u = (x * A).sum(1)                 # <X, A> row-wise
    uP = (PY * A).sum(1)               # <PY, A>
    W = A @ y.T
    # explicit term
    B1 = 2.0 * r[:, None] * A
    B2 = (r * u)[:, None] * x
    B3 = u[:, None] * PY
    B4 = uP[:, None] * x
    B5 = (P * W) @ y
    EA = B1 - (4.0 / eps) * (B2 - B3 - B4 + B5)
    # implicit term
    r1 = 2.0 * (r * u - uP)
    r2 = 2.0 * (P.T @ u - ((P.T @ A) * y).sum(1))
    if tau == 0.0:
        H = np.block([[np.diag(r), P], [P.T, np.diag(c)]])
        w = np.linalg.pinv(H, rcond=1e-13) @ np.concatenate([r1, r2])
        w1, w2 = w[:n], w[n:]
    else:
        S = np.diag(c) - P.T @ (P / r[:, None]) + tau * np.eye(m)
        w2 = np.linalg.solve(S, r2 - P.T @ (r1 / r))
        w1 = (r1 - P @ w2) / r
    Rtw = 2.0 * ((r * w1)[:, None] * x - w1[:, None] * PY + (P @ w2)[:, None] * x - P @ (w2[:, None] * y))
    return Rtw / eps + EA


def hadamard_transport(x, y, a, b, eps, f, g, A, V=None):
    """(P o (A Y^T)) V, n x p: the output of Alg. 5 with B = Y (Thm. 5 uses it with V = Y, the
    default), dense: every plan entry P_ij is multiplied by the weight <A_i, y_j> before the
    product with V."""
    x, y, A = (np.asarray(v, dtype=np.float64) for v in (x, y, A))
    V = y if V is None else np.asarray(V, dtype=np.float64)
    P = _plan(x, y, *(np.asarray(v, dtype=np.float64) for v in (a, b)), eps,
              np.asarray(f, dtype=np.float64), np.asarray(g, dtype=np.float64))
    return (P * (A @ y.T)) @ V
