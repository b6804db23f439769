"""GPU parity of the bf16 matrix-core path against the float64 oracle.

Two oracles are used: A = the oracle on the inputs as given (the contract: 2e-2*eps), and
B = the same float64 oracle on the inputs rounded to bfloat16 first, against which the kernel
should agree to fp32 accuracy -- this separates "bf16 rounding" from "kernel bug"."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu
TOL_A = 2e-2
TOL_B = 2e-4
BF = binding.FS_COMPUTE_BF16_MFMA


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def _rand_problem(rng, n, m, d):
    x = (rng.standard_normal((n, d)) / np.sqrt(d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) / np.sqrt(d) + 0.3 / np.sqrt(d)).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.1
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


@pytest.mark.parametrize("n,m,d", [(1, 1, 16), (100, 90, 16), (300, 500, 64), (257, 129, 100),
                                   (1000, 777, 784), (50, 2000, 1024), (513, 300, 48)])
def test_single_half_steps(ctx, oracle, n, m, d):
    rng = np.random.default_rng(2 * n + 3 * m + 5 * d)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.5))      # |x| ~ 1: bf16 rounding moves C/eps by ~5e-3 at this eps
    g = (0.3 * rng.standard_normal(m)).astype(np.float32)
    f = (0.3 * rng.standard_normal(n)).astype(np.float32)
    say("bf16 path update_f/update_g n=%d m=%d d=%d" % (n, m, d))
    prob = make_problem(x, y, a, b, compute=BF)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    g_gpu = host(ctx.fs_update_g(prob, eps, dev(f)))
    xb, yb = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    eB = max(max_err_over_eps(f_gpu, oracle.update_f(xb, yb, b, eps, g), eps),
             max_err_over_eps(g_gpu, oracle.update_g(xb, yb, a, eps, f), eps))
    eA = max(max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps),
             max_err_over_eps(g_gpu, oracle.update_g(x, y, a, eps, f), eps))
    say("  vs oracle on bf16-rounded inputs %.3e, vs oracle on given inputs %.3e" % (eB, eA))
    assert eB <= TOL_B and eA <= TOL_A


def test_bf16_mode_refuses_small_d(ctx):
    rng = np.random.default_rng(0)
    x, y, a, b = _rand_problem(rng, 10, 10, 8)
    prob = make_problem(x, y, a, b, compute=BF)
    with pytest.raises(binding.FlashSinkError) as ei:
        ctx.fs_update_f(prob, 0.1, dev(np.zeros(10, dtype=np.float32)))
    assert ei.value.status == 5


def test_mnist_shape_trajectory_scaled_down(ctx, oracle):
    """Beta(0.5, 2) coordinates, d = 784, eps = 0.05 * mean squared distance, 100 iterations,
    at n = m = 2048 (the oracle needs ~40 s)."""
    w = workloads.make("mnist_shape", n=2048, m=2048)
    say("solve mnist_shape n=m=2048 d=784 eps=%.4f iters=%d" % (w.eps_end, w.iters))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    say("mnist_shape 2048: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL_A and eg <= TOL_A
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    xb, yb = workloads.to_bf16_round(w.x), workloads.to_bf16_round(w.y)
    ero, eco = oracle.marginal_err(xb, yb, w.a, w.b, eps, host(f), host(g))
    say("mnist_shape 2048: err_row gpu=%.6e oracleB=%.6e err_col gpu=%.3e oracleB=%.3e" % (er, ero, ec, eco))
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5


def test_embedding_trajectory_scaled_down(ctx, oracle):
    """Unit-norm rows, bf16 storage, Dirichlet weights, eps = 0.05, 200 iterations at
    n = 2000, m = 800, d = 1024."""
    w = workloads.make("embedding", n=2000, m=800)
    say("solve embedding n=%d m=%d d=%d iters=%d" % (w.n, w.m, w.d, w.iters))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    say("embedding: max|df|/eps=%.3e max|dg|/eps=%.3e (bf16 storage: oracle A == oracle B)" % (ef, eg))
    assert ef <= TOL_A and eg <= TOL_A
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    ero, eco = oracle.marginal_err(w.x, w.y, w.a, w.b, eps, host(f), host(g))
    say("embedding: err_row gpu=%.6e oracle=%.6e err_col gpu=%.3e oracle=%.3e" % (er, ero, ec, eco))
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5


@pytest.mark.parametrize("name,iters", [("mnist_shape", 100), ("embedding", 200)])
def test_full_size_sampled(ctx, oracle, name, iters):
    """Full-size runs in the bench's launch configuration; the last half-steps are re-derived by
    the oracle on 64 sampled rows/columns."""
    w = workloads.make(name, iters=iters)
    say("solve %s FULL n=%d m=%d d=%d iters=%d" % (name, w.n, w.m, w.d, w.iters))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    assert torch.isfinite(f).all() and torch.isfinite(g).all()
    eps = float(np.float32(w.eps_end))
    rng = np.random.default_rng(99)
    rows = np.sort(rng.choice(w.n, size=64, replace=False))
    cols = np.sort(rng.choice(w.m, size=64, replace=False))
    f_next = ctx.fs_update_f(prob, eps, g)
    g_next = ctx.fs_update_g(prob, eps, f_next)
    gh, fnh = host(g), host(f_next)
    ef = max_err_over_eps(fnh[rows], oracle.update_f(w.x, w.y, w.b, eps, gh, rows=rows), eps)
    eg = max_err_over_eps(host(g_next)[cols], oracle.update_g(w.x, w.y, w.a, eps, fnh, cols=cols), eps)
    say("%s full: sampled max|df|/eps=%.3e max|dg|/eps=%.3e" % (name, ef, eg))
    assert ef <= TOL_A and eg <= TOL_A
    # marginals of the plan the solve ended on: the column marginal is exact after a g-update (holds at any size), and
    # on the sampled rows / columns the marginals Prop. 3 gives from the GPU's half-steps equal the oracle's plan sums
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    say("%s full: err_row=%.4e err_col=%.4e" % (name, er, ec))
    assert ec <= 1e-4 and 0.0 <= er < 2.0
    xb, yb = workloads.to_bf16_round(w.x), workloads.to_bf16_round(w.y)
    fh = host(f)
    r_or = oracle.apply_plan(xb, yb, w.a, w.b, eps, fh, gh, np.ones((w.m, 1)), rows=rows)[:, 0]
    c_or = oracle.apply_plan_T(xb, yb, w.a, w.b, eps, fh, gh, np.ones((w.n, 1)), cols=cols)[:, 0]
    r_gpu = w.a[rows].astype(np.float64) * np.exp((fh[rows] - fnh[rows]) / eps)
    c_gpu = w.b[cols].astype(np.float64) * np.exp((gh[cols] - host(ctx.fs_update_g(prob, eps, f))[cols]) / eps)
    dr = np.abs(r_gpu / r_or - 1).max()
    dc = np.abs(c_gpu / c_or - 1).max()
    say("%s full: sampled marginals against the oracle on the rounded points: rows %.3e cols %.3e (relative)" % (name, dr, dc))
    # one half-step agrees with the oracle on the rounded points to TOL_B in units of eps; r = a exp(df/eps)
    assert dr <= 2 * TOL_B and dc <= 2 * TOL_B
    # the sampled part of the L1 errors, term by term
    assert abs(np.abs(r_gpu - w.a[rows]).sum() - np.abs(r_or - w.a[rows]).sum()) <= 1e-5
    assert abs(np.abs(c_gpu - w.b[cols]).sum() - np.abs(c_or - w.b[cols]).sum()) <= 1e-5


TOL_APPLY_A = 2e-2    # relative Frobenius error against the oracle on the inputs as given
TOL_APPLY_B = 6e-3    # ... on the bf16-rounded points (what is left: bf16 plan entries and values)
# Element by element: an entry of P V is a sum of terms P_ij V_jc of either sign, and every term carries the bf16
# roundings of its plan entry and of its value (8 significant bits: unit roundoff 2^-8 each, 2^-7 = 7.8e-3 together in
# the worst case, which a plan close to an assignment reaches: one term per row), so the error of an entry is bounded
# relative to (P |V|)_ic, which the oracle gives as a second application; on top comes the error of the exponent
# (TOL_B).  Against the inputs as given the rounding of the points moves every exponent by up to the 2e-2 the contract
# allows.
TOL_APPLY_EL_A = 2e-2 + 8e-3
TOL_APPLY_EL_B = 8.5e-3


@pytest.mark.parametrize("n,m,d,p", [(1, 1, 16, 1), (130, 70, 20, 1), (200, 333, 64, 5), (257, 600, 40, 70),
                                     (64, 64, 96, 64), (300, 1100, 784, 64), (1500, 129, 128, 33)])
def test_apply_shapes_bf16_mode(ctx, oracle, n, m, d, p):
    """Plan application (Alg. 2 / Alg. 4) in bf16 mode: both directions, with the plan's mass,
    ragged sizes, several streamed tiles and more than one pass of 64 value columns."""
    rng = np.random.default_rng(13 * n + m + d + p)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.5))
    xb, yb = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    fo, go = oracle.solve(xb, yb, a, b, eps, eps, 1, 3)
    f32 = (fo + 0.05 * rng.standard_normal(n)).astype(np.float32)
    g32 = go.astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    U = rng.standard_normal((n, p)).astype(np.float32)
    say("bf16 path apply n=%d m=%d d=%d p=%d" % (n, m, d, p))
    prob = make_problem(x, y, a, b, compute=BF)
    out, mass = ctx.fs_apply_plan(prob, eps, dev(f32), dev(g32), dev(V), want_mass=True)
    outT, massT = ctx.fs_apply_plan_T(prob, eps, dev(f32), dev(g32), dev(U), want_mass=True)
    torch.cuda.synchronize()
    for tag, xs, ys, tol, tol_el in (("given", x, y, TOL_APPLY_A, TOL_APPLY_EL_A),
                                     ("bf16-rounded", xb, yb, TOL_APPLY_B, TOL_APPLY_EL_B)):
        want, r = oracle.apply_plan(xs, ys, a, b, eps, f32, g32, V, return_mass=True)
        wantT, c = oracle.apply_plan_T(xs, ys, a, b, eps, f32, g32, U, return_mass=True)
        e1 = np.linalg.norm(host(out) - want) / np.linalg.norm(want)
        e2 = np.linalg.norm(host(outT) - wantT) / np.linalg.norm(wantT)
        em = max(np.abs(host(mass) / r - 1).max(), np.abs(host(massT) / c - 1).max())
        scale = oracle.apply_plan(xs, ys, a, b, eps, f32, g32, np.abs(V))
        scaleT = oracle.apply_plan_T(xs, ys, a, b, eps, f32, g32, np.abs(U))
        el = max((np.abs(host(out) - want) / scale).max(), (np.abs(host(outT) - wantT) / scaleT).max())
        say("  vs oracle on %s inputs: PV %.3e  PtU %.3e  mass %.3e  element-wise / (P|V|) %.3e" % (tag, e1, e2, em, el))
        assert e1 <= tol and e2 <= tol and em <= tol
        assert el <= tol_el


def test_apply_bf16_mode_large_score_spread(ctx, oracle):
    """Small eps: the plan is close to an assignment and the running max moves by hundreds between
    tiles, so the accumulators are rescaled many times."""
    rng = np.random.default_rng(77)
    n, m, d, p = 700, 900, 64, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) + 1.0).astype(np.float32)
    a = np.full(n, 1.0 / n, dtype=np.float32)
    b = np.full(m, 1.0 / m, dtype=np.float32)
    eps = float(np.float32(0.5))
    xb, yb = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    fo, go = oracle.solve(xb, yb, a, b, eps, eps, 1, 20)
    f32, g32 = fo.astype(np.float32), go.astype(np.float32)
    say("bf16 path apply, score spread: n=%d m=%d d=%d eps=%g" % (n, m, d, eps))
    prob = make_problem(x, y, a, b, compute=BF)
    PY, r = ctx.fs_apply_plan(prob, eps, dev(f32), dev(g32), dev(y), want_mass=True)
    want, r_o = oracle.apply_plan(xb, yb, a, b, eps, f32, g32, y, return_mass=True)
    e1 = np.linalg.norm(host(PY) - want) / np.linalg.norm(want)
    em = np.abs(host(r) / r_o - 1).max()
    el = (np.abs(host(PY) - want) / oracle.apply_plan(xb, yb, a, b, eps, f32, g32, np.abs(y))).max()
    say("  PY %.3e  mass %.3e  element-wise / (P|y|) %.3e" % (e1, em, el))
    assert e1 <= TOL_APPLY_B and em <= TOL_APPLY_B
    assert el <= TOL_APPLY_EL_B
