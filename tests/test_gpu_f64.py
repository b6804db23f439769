"""GPU parity of the fp32-accuracy path for d > 16 (score contraction on the fp64 matrix
cores) against the float64 oracle.  Tolerances as for the low-d path: 1e-4*eps on the
potentials, 1e-5 on marginal errors, 2e-4 relative on plan applications."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu
TOL = 1e-4


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def _rand_problem(rng, n, m, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) * 0.8 + 0.5).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.1
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


@pytest.mark.parametrize("n,m,d", [(1, 1, 17), (70, 65, 32), (300, 500, 64), (129, 1000, 33),
                                   (1000, 777, 100), (64, 2100, 200)])
def test_single_half_steps(ctx, oracle, n, m, d):
    rng = np.random.default_rng(n + 3 * m + 7 * d)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.5))
    g = rng.standard_normal(m).astype(np.float32)
    f = rng.standard_normal(n).astype(np.float32)
    say("f64 path update_f/update_g n=%d m=%d d=%d" % (n, m, d))
    prob = make_problem(x, y, a, b)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    g_gpu = host(ctx.fs_update_g(prob, eps, dev(f)))
    assert max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps) <= TOL
    assert max_err_over_eps(g_gpu, oracle.update_g(x, y, a, eps, f), eps) <= TOL


def test_bf16_storage_in_fp32_mode(ctx, oracle):
    rng = np.random.default_rng(3)
    x, y, a, b = _rand_problem(rng, 200, 150, 48)
    x, y = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    eps = float(np.float32(0.5))
    g = rng.standard_normal(150).astype(np.float32)
    say("f64 path with bf16 storage")
    prob = make_problem(x, y, a, b, bf16_storage=True)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    assert max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps) <= TOL


def test_transport_grad_trajectory_scaled_down(ctx, oracle):
    """n = m = 2048, d = 64, eps = 0.1, 100 iterations (scores reach ~2e3)."""
    w = workloads.make("transport_grad", n=2048, m=2048)
    say("solve transport_grad n=m=2048 d=64 iters=%d" % w.iters)
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    floor = float(np.max(np.abs(fo.astype(np.float32).astype(np.float64) - fo)) / eps)
    say("grad 2048: max|df|/eps=%.3e max|dg|/eps=%.3e (float32 output rounding alone: %.3e)" % (ef, eg, floor))
    assert ef <= TOL and eg <= TOL
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    ero, eco = oracle.marginal_err(w.x, w.y, w.a, w.b, eps, host(f), host(g))
    say("grad 2048: err_row gpu=%.6e oracle=%.6e err_col gpu=%.3e oracle=%.3e" % (er, ero, ec, eco))
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5
    # plan applications with the GPU's own potentials: P Y, P^T U, and the gradient of Cor. 4
    fh, gh = host(f), host(g)
    PY, r = ctx.fs_apply_plan(prob, eps, f, g, prob.y, want_mass=True)
    PtU, c = ctx.fs_apply_plan_T(prob, eps, f, g, dev(w.U), want_mass=True)
    want, r_o = oracle.apply_plan(w.x, w.y, w.a, w.b, eps, fh, gh, w.y, return_mass=True)
    wantT, c_o = oracle.apply_plan_T(w.x, w.y, w.a, w.b, eps, fh, gh, w.U, return_mass=True)
    for got, ref, nm in ((host(PY), want, "PY"), (host(PtU), wantT, "PtU")):
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        mx = np.abs(got - ref).max() / np.abs(ref).max()
        say("grad 2048: %s rel_fro=%.3e max/absmax=%.3e" % (nm, rel, mx))
        assert rel <= 2e-4 and mx <= 1e-3
    np.testing.assert_allclose(host(r), r_o, rtol=2e-4)
    np.testing.assert_allclose(host(c), c_o, rtol=2e-4)
    a64 = w.a.astype(np.float64)[:, None]
    grad_gpu = 2.0 * (a64 * w.x - host(PY))
    grad_ref = 2.0 * (a64 * w.x - want)
    assert np.linalg.norm(grad_gpu - grad_ref) <= 2e-4 * np.linalg.norm(grad_ref)
    T_gpu = host(PY) / a64                      # barycentric projection (x - T is the other form)
    assert np.linalg.norm(T_gpu - want / a64) <= 2e-4 * np.linalg.norm(want / a64)
    # the gradient with respect to the other cloud: 2 (diag(b) y - P^T x), by the transposed application
    PtX = ctx.fs_apply_plan_T(prob, eps, f, g, prob.x)
    wantX = oracle.apply_plan_T(w.x, w.y, w.a, w.b, eps, fh, gh, w.x)
    b64 = w.b.astype(np.float64)[:, None]
    gy_gpu, gy_ref = 2.0 * (b64 * w.y - host(PtX)), 2.0 * (b64 * w.y - wantX)
    say("grad 2048: gradient wrt y rel=%.3e" % (np.linalg.norm(gy_gpu - gy_ref) / np.linalg.norm(gy_ref)))
    assert np.linalg.norm(gy_gpu - gy_ref) <= 2e-4 * np.linalg.norm(gy_ref)


@pytest.mark.parametrize("n,m,d,p", [(130, 70, 20, 1), (200, 333, 64, 5), (257, 190, 40, 70), (64, 64, 96, 64),
                                     # more than 64 columns: passes of 128, then the rest (wide or plain)
                                     (150, 333, 100, 200), (90, 260, 33, 129), (1100, 700, 64, 128)])
def test_apply_shapes(ctx, oracle, n, m, d, p):
    rng = np.random.default_rng(11 * n + m + d + p)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(2.0))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 3)
    f32 = (fo + 0.05 * rng.standard_normal(n)).astype(np.float32)
    g32 = go.astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    U = rng.standard_normal((n, p)).astype(np.float32)
    say("f64 path apply n=%d m=%d d=%d p=%d" % (n, m, d, p))
    prob = make_problem(x, y, a, b)
    out, mass = ctx.fs_apply_plan(prob, eps, dev(f32), dev(g32), dev(V), want_mass=True)
    outT, massT = ctx.fs_apply_plan_T(prob, eps, dev(f32), dev(g32), dev(U), want_mass=True)
    want, r = oracle.apply_plan(x, y, a, b, eps, f32, g32, V, return_mass=True)
    wantT, c = oracle.apply_plan_T(x, y, a, b, eps, f32, g32, U, return_mass=True)
    for got, ref in ((host(out), want), (host(outT), wantT)):
        assert np.linalg.norm(got - ref) <= 2e-4 * np.linalg.norm(ref)
        assert np.abs(got - ref).max() <= 1e-3 * np.abs(ref).max()
    np.testing.assert_allclose(host(mass), r, rtol=2e-4)
    np.testing.assert_allclose(host(massT), c, rtol=2e-4)


def test_full_size_transport_grad_sampled(ctx, oracle):
    """n = m = 16384, d = 64, p = 64: full solve on the GPU, then one more half-step each way and
    both plan applications are checked by the oracle on 128 sampled rows."""
    w = workloads.make("transport_grad")
    say("solve transport_grad FULL n=m=%d d=%d" % (w.n, w.d))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    assert torch.isfinite(f).all() and torch.isfinite(g).all()
    eps = float(np.float32(w.eps_end))
    rng = np.random.default_rng(555)
    rows = np.sort(rng.choice(w.n, size=128, replace=False))
    f_next = ctx.fs_update_f(prob, eps, g)
    g_next = ctx.fs_update_g(prob, eps, f_next)
    gh, fnh = host(g), host(f_next)
    ef = max_err_over_eps(fnh[rows], oracle.update_f(w.x, w.y, w.b, eps, gh, rows=rows), eps)
    eg = max_err_over_eps(host(g_next)[rows], oracle.update_g(w.x, w.y, w.a, eps, fnh, cols=rows), eps)
    say("grad full: sampled max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL and eg <= TOL
    fh = host(f)
    PY = host(ctx.fs_apply_plan(prob, eps, f, g, prob.y))
    PtU = host(ctx.fs_apply_plan_T(prob, eps, f, g, dev(w.U)))
    want = oracle.apply_plan(w.x, w.y, w.a, w.b, eps, fh, gh, w.y, rows=rows)
    wantT = oracle.apply_plan_T(w.x, w.y, w.a, w.b, eps, fh, gh, w.U, cols=rows)
    for got, ref, nm in ((PY[rows], want, "PY"), (PtU[rows], wantT, "PtU")):
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        say("grad full: %s sampled rel_fro=%.3e" % (nm, rel))
        assert rel <= 2e-4
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    say("grad full: err_row=%.4e err_col=%.4e" % (er, ec))
    assert ec <= 1e-4 and 0.0 <= er < 2.0
