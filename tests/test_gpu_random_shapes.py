"""GPU parity on a seeded sweep of random shapes: sizes that are not multiples of any tile, every
dimension from 1 to 100, both schedules and compute modes, plan applications with odd widths --
against the float64 oracle at the bars of the other GPU tests.  A second batch stays on the fp64 matrix-core
path with contractions up to d = 260 and plan applications up to 200 columns."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu
BF = binding.FS_COMPUTE_BF16_MFMA


def _cases():
    rng = np.random.default_rng(20260203)
    out = []
    for k in range(36):
        n = int(rng.integers(1, 2600))
        m = int(rng.integers(1, 2600))
        d = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 16, 17, 19, 24, 31, 32, 33, 48, 64, 65, 100]))
        bf = bool(d >= 16 and rng.random() < 0.4)
        eps = float(rng.choice([0.05, 0.2, 1.0, 3.0]))
        iters = int(rng.integers(1, 6))
        p = int(rng.choice([1, 2, 3, 4, 5, 9, 63, 64, 65]))
        out.append(pytest.param(k, n, m, d, bf, eps, iters, p, id="case%02d_n%d_m%d_d%d_%s" % (k, n, m, d, "bf16" if bf else "fp32")))
    # the fp64 matrix-core path once more, with longer contractions and wide plan applications
    rng = np.random.default_rng(20260204)
    for k in range(100, 124):
        n = int(rng.integers(1, 2600))
        m = int(rng.integers(1, 2600))
        d = int(rng.choice([17, 20, 33, 40, 64, 65, 72, 100, 130, 200, 260]))
        eps = float(rng.choice([0.2, 1.0, 3.0]))
        iters = int(rng.integers(1, 5))
        p = int(rng.choice([1, 16, 17, 64, 65, 100, 128, 129, 200]))
        out.append(pytest.param(k, n, m, d, False, eps, iters, p, id="case%03d_n%d_m%d_d%d_p%d_fp32" % (k, n, m, d, p)))
    return out


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("k,n,m,d,bf,eps,iters,p", _cases())
def test_random_shape(ctx, oracle, k, n, m, d, bf, eps, iters, p):
    rng = np.random.default_rng(1000 + k)
    scale = 1.0 / np.sqrt(d)
    x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    y = (rng.standard_normal((m, d)) * scale + 0.2 * scale).astype(np.float32)
    a = rng.random(n) + 0.05
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.05
    b = (b / b.sum()).astype(np.float32)
    eps = float(np.float32(eps))
    symmetric = (k % 3 == 0)
    say("random shape %d: n=%d m=%d d=%d %s eps=%g iters=%d p=%d %s" % (k, n, m, d, "bf16" if bf else "fp32", eps, iters, p,
                                                                      "symmetric" if symmetric else "alternating"))
    prob = make_problem(x, y, a, b, compute=BF) if bf else make_problem(x, y, a, b)
    xs, ys = (workloads.to_bf16_round(x), workloads.to_bf16_round(y)) if bf else (x, y)
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    if symmetric:
        ctx.fs_solve_symmetric(prob, eps, iters, f, g)
        fo, go = oracle.solve_symmetric(xs, ys, a, b, eps, iters)
    else:
        ctx.fs_solve(prob, eps, eps, 1, iters, f, g)
        fo, go = oracle.solve(xs, ys, a, b, eps, eps, 1, iters)
    tol = 2e-4 if bf else 1e-4     # bf16 mode against the oracle on the rounded points
    ef, eg = max_err_over_eps(host(f), fo, eps), max_err_over_eps(host(g), go, eps)
    V = rng.standard_normal((m, p)).astype(np.float32)
    out, mass = ctx.fs_apply_plan(prob, eps, f, g, dev(V), want_mass=True)
    want, r = oracle.apply_plan(xs, ys, a, b, eps, host(f).astype(np.float32), host(g).astype(np.float32), V, return_mass=True)
    ea = np.linalg.norm(host(out) - want) / max(np.linalg.norm(want), 1e-300)
    em = np.abs(host(mass) / r - 1).max()
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    ero, eco = oracle.marginal_err(xs, ys, a, b, eps, host(f).astype(np.float32), host(g).astype(np.float32))
    say("  max|df|/eps=%.2e max|dg|/eps=%.2e apply rel=%.2e mass rel=%.2e marginal err diff=%.1e/%.1e" % (ef, eg, ea, em, abs(er - ero), abs(ec - eco)))
    assert ef <= tol and eg <= tol
    assert ea <= (6e-3 if bf else 2e-4) and em <= (6e-3 if bf else 2e-4)
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5
