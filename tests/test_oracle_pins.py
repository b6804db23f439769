"""Pins for the float64 CPU oracle (CPU only).

The oracle is the reference every GPU result is compared with, so it is pinned
here to things other than itself: dense whole-matrix brute force on tiny inputs,
exact special cases, invariants the mathematics fixes, and the closed form of
entropic OT between Gaussians.  Citations are to the paper's sections/equations.
"""
import numpy as np
import pytest
from scipy.linalg import sqrtm

from oracle import dense_ref


def _e(eps):
    """solve() takes eps as a float32 value (like the GPU ABI); use the same value everywhere."""
    return float(np.float32(eps))


def _problem(rng, n, m, d, uniform=False):
    x = rng.standard_normal((n, d))
    y = rng.standard_normal((m, d)) * 0.7 + 0.3
    if uniform:
        a = np.full(n, 1.0 / n)
        b = np.full(m, 1.0 / m)
    else:
        a = rng.random(n) + 0.1
        a /= a.sum()
        b = rng.random(m) + 0.1
        b /= b.sum()
    return x, y, a, b


# ----------------------------------------------------------------------------------------
# P1: brute force on tiny inputs (Eq. 2-3 on an explicit cost matrix, scipy logsumexp)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,m", [(1, 1), (2, 3), (3, 2), (17, 5), (64, 33)])
@pytest.mark.parametrize("d", [1, 3, 7])
@pytest.mark.parametrize("eps", [0.01, 0.1, 1.0, 10.0])
def test_solve_matches_dense_bruteforce(oracle, n, m, d, eps):
    rng = np.random.default_rng(100 * n + 10 * m + d)
    x, y, a, b = _problem(rng, n, m, d)
    eps = _e(eps)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 7)
    f2, g2 = dense_ref.solve(x, y, a, b, [eps], 7)
    scale = max(1.0, np.abs(f2).max(), np.abs(g2).max())
    assert np.abs(f - f2).max() <= 1e-12 * scale
    assert np.abs(g - g2).max() <= 1e-12 * scale


def test_single_half_steps_match_dense(oracle):
    rng = np.random.default_rng(7)
    x, y, a, b = _problem(rng, 19, 23, 4)
    C = dense_ref.cost(x, y)
    g = rng.standard_normal(23)
    f = rng.standard_normal(19)
    np.testing.assert_allclose(oracle.update_f(x, y, b, 0.3, g), dense_ref.update_f(C, b, 0.3, g),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.update_g(x, y, a, 0.3, f), dense_ref.update_g(C, a, 0.3, f),
                               rtol=0, atol=1e-12)
    rows = np.array([3, 0, 18, 3])
    np.testing.assert_array_equal(oracle.update_f(x, y, b, 0.3, g, rows=rows),
                                  oracle.update_f(x, y, b, 0.3, g)[rows])
    cols = np.array([22, 1])
    np.testing.assert_array_equal(oracle.update_g(x, y, a, 0.3, f, cols=cols),
                                  oracle.update_g(x, y, a, 0.3, f)[cols])


def test_annealed_schedule_matches_dense(oracle):
    """Geometric eps schedule, both endpoints included, potentials carried across stages."""
    rng = np.random.default_rng(11)
    x, y, a, b = _problem(rng, 12, 9, 3)
    S = 5
    eps_list = [oracle.stage_eps(1.0, 0.05, S, s) for s in range(S)]
    assert eps_list[0] == 1.0 and eps_list[-1] == float(np.float32(0.05))
    ratios = np.array(eps_list[1:]) / np.array(eps_list[:-1])
    np.testing.assert_allclose(ratios, (0.05 / 1.0) ** (1.0 / (S - 1)), rtol=1e-6)
    for e in eps_list:
        assert e == float(np.float32(e))          # each stage eps is a float32 value
    f, g = oracle.solve(x, y, a, b, 1.0, 0.05, S, 3)
    f2, g2 = dense_ref.solve(x, y, a, b, eps_list, 3)
    np.testing.assert_allclose(f, f2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g, g2, rtol=0, atol=1e-12)
    assert oracle.stage_eps(0.3, 0.7, 1, 0) == float(np.float32(0.7))


def test_symmetric_schedule_matches_dense(oracle):
    rng = np.random.default_rng(12)
    x, y, a, b = _problem(rng, 10, 14, 2)
    f, g = oracle.solve_symmetric(x, y, a, b, 0.4, 9)      # this entry does not round eps
    f2, g2 = dense_ref.solve_symmetric(x, y, a, b, 0.4, 9)
    np.testing.assert_allclose(f, f2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(g, g2, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------------------
# P2: Prop. 1 -- the shifted biased-dot-product form equals Eq. 2-3
# ----------------------------------------------------------------------------------------
def test_prop1_shifted_form_equals_unshifted(oracle):
    from scipy.special import logsumexp
    rng = np.random.default_rng(21)
    x, y, a, b = _problem(rng, 31, 27, 5)
    eps = _e(0.37)
    g = rng.standard_normal(27)
    alpha = oracle.row_norms(x)
    beta = oracle.row_norms(y)
    np.testing.assert_allclose(alpha, (x * x).sum(1), rtol=1e-15)
    # S_X(ghat) = (Q K^T + 1 (ghat + delta)) / eps with Q = sqrt2 X, K = sqrt2 Y
    Q, K = np.sqrt(2.0) * x, np.sqrt(2.0) * y
    ghat = g - beta
    delta = eps * np.log(b)
    fhat = -eps * logsumexp((Q @ K.T + (ghat + delta)[None, :]) / eps, axis=1)
    f = oracle.update_f(x, y, b, eps, g)
    np.testing.assert_allclose(fhat + alpha, f, rtol=0, atol=1e-11)
    fcur = rng.standard_normal(31)
    gamma = eps * np.log(a)
    ghat_new = -eps * logsumexp((K @ Q.T + (fcur - alpha + gamma)[None, :]) / eps, axis=1)
    np.testing.assert_allclose(ghat_new + beta, oracle.update_g(x, y, a, eps, fcur), rtol=0,
                               atol=1e-11)


# ----------------------------------------------------------------------------------------
# P3: marginals
# ----------------------------------------------------------------------------------------
def test_marginals_after_half_steps(oracle):
    rng = np.random.default_rng(31)
    x, y, a, b = _problem(rng, 40, 25, 3)
    eps = _e(0.2)
    errs = []
    for iters in (1, 2, 5, 20, 100, 400):
        f, g = oracle.solve(x, y, a, b, eps, eps, 1, iters)
        r, c = oracle.marginals(x, y, a, b, eps, f, g)
        # the solve ends on a g-update, so the column marginal is exact
        assert np.abs(c - b).max() <= 1e-14
        assert abs(r.sum() - 1.0) <= 1e-12 and abs(c.sum() - 1.0) <= 1e-12
        er, ec = oracle.marginal_err(x, y, a, b, eps, f, g)
        assert er == pytest.approx(np.abs(r - a).sum(), abs=1e-15)
        assert ec == pytest.approx(np.abs(c - b).sum(), abs=1e-15)
        errs.append(er)
    assert all(e2 <= e1 * (1 + 1e-12) for e1, e2 in zip(errs, errs[1:]))
    assert errs[-1] < 1e-10
    # right after an f-update the ROW marginal is exact instead
    f2 = oracle.update_f(x, y, b, eps, g)
    r2, _ = oracle.marginals(x, y, a, b, eps, f2, g)
    assert np.abs(r2 - a).max() <= 1e-14


def test_marginals_match_dense_plan(oracle):
    rng = np.random.default_rng(32)
    x, y, a, b = _problem(rng, 13, 21, 4)
    f = rng.standard_normal(13) * 0.3
    g = rng.standard_normal(21) * 0.3
    P = dense_ref.plan(x, y, a, b, 0.5, f, g)
    r, c = oracle.marginals(x, y, a, b, 0.5, f, g)
    np.testing.assert_allclose(r, P.sum(1), rtol=1e-13)
    np.testing.assert_allclose(c, P.sum(0), rtol=1e-13)


def test_prop3_induced_marginals(oracle):
    """r = a*exp((f - f+)/eps), c = b*exp((g - g+)/eps) for ANY potentials (Prop. 3)."""
    rng = np.random.default_rng(33)
    x, y, a, b = _problem(rng, 18, 15, 3)
    eps = _e(0.25)
    f = rng.standard_normal(18)
    g = rng.standard_normal(15)
    r, c = oracle.marginals(x, y, a, b, eps, f, g)
    fplus = oracle.update_f(x, y, b, eps, g)
    gplus = oracle.update_g(x, y, a, eps, f)
    np.testing.assert_allclose(r, a * np.exp((f - fplus) / eps), rtol=1e-12)
    np.testing.assert_allclose(c, b * np.exp((g - gplus) / eps), rtol=1e-12)


# ----------------------------------------------------------------------------------------
# P4: symmetry x = y, a = b
# ----------------------------------------------------------------------------------------
def test_symmetry_when_clouds_coincide(oracle):
    rng = np.random.default_rng(41)
    x, _, a, _ = _problem(rng, 30, 30, 3)
    eps = _e(0.5)
    for iters in (1, 3, 10):
        f, g = oracle.solve_symmetric(x, x, a, a, eps, iters)
        assert np.abs(f - g).max() <= 1e-13
    f, g = oracle.solve(x, x, a, a, eps, eps, 1, 600)
    diff = f - g
    assert diff.std() <= 1e-10                     # equal up to the gauge constant
    fs, gs = oracle.solve_symmetric(x, x, a, a, eps, 600)
    np.testing.assert_allclose(0.5 * (f + g), fs, rtol=0, atol=1e-9)


# ----------------------------------------------------------------------------------------
# P5: primal-dual
# ----------------------------------------------------------------------------------------
def test_primal_dual_gap_identity_and_convergence(oracle):
    rng = np.random.default_rng(51)
    x, y, a, b = _problem(rng, 22, 17, 3)
    eps = _e(0.3)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 4)
    pr, du = oracle.objectives(x, y, a, b, eps, f, g)
    P = dense_ref.plan(x, y, a, b, eps, f, g)
    assert pr == pytest.approx(dense_ref.primal(x, y, a, b, eps, P), rel=1e-12)
    r, c = P.sum(1), P.sum(0)
    # log(P/ab) = (f+g-C)/eps  =>  primal - dual = <r-a, f> + <c-b, g>
    assert pr - du == pytest.approx(np.dot(r - a, f) + np.dot(c - b, g), abs=1e-12)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 2000)
    pr, du = oracle.objectives(x, y, a, b, eps, f, g)
    assert pr == pytest.approx(du, abs=1e-10)
    assert du == pytest.approx(np.dot(a, f) + np.dot(b, g), abs=1e-10)
    # weak duality: any feasible coupling costs at least the optimal dual value
    indep = np.outer(a, b)
    assert dense_ref.primal(x, y, a, b, eps, indep) >= du - 1e-12


# ----------------------------------------------------------------------------------------
# P6: closed form of entropic OT between Gaussians (cost |x-y|^2, eps*KL(P | a(x)b)):
#   sigma^2 = eps/2, D = (4 A^{1/2} B A^{1/2} + sigma^4 I)^{1/2},
#   OT = |mu_a-mu_b|^2 + tr A + tr B - tr D + d sigma^2 (1 - log(2 sigma^2))
#        + sigma^2 log det(D + sigma^2 I)
# (Janati, Muzellec, Peyre, Cuturi 2020, Theorem 1.)  The discrete measures are
# quadrature rules for the Gaussians, which converge spectrally fast.
# ----------------------------------------------------------------------------------------
def _gaussian_eot(mu_a, A, mu_b, B, eps):
    A = np.atleast_2d(A).astype(float)
    B = np.atleast_2d(B).astype(float)
    d = A.shape[0]
    s2 = eps / 2.0
    Ah = np.real(sqrtm(A))
    D = np.real(sqrtm(4.0 * Ah @ B @ Ah + s2 * s2 * np.eye(d)))
    dm = np.atleast_1d(mu_a) - np.atleast_1d(mu_b)
    return (dm @ dm + np.trace(A) + np.trace(B) - np.trace(D) + d * s2 * (1 - np.log(2 * s2))
            + s2 * np.log(np.linalg.det(D + s2 * np.eye(d))))


@pytest.mark.parametrize("eps,iters", [(0.1, 3000), (0.5, 800), (2.0, 300)])
def test_gaussian_closed_form_1d(oracle, eps, iters):
    eps = _e(eps)
    xs = np.linspace(-8.0, 8.0, 600)
    ys = np.linspace(-3.0, 5.0, 500)
    a = np.exp(-0.5 * xs ** 2)
    a /= a.sum()
    b = np.exp(-0.5 * ((ys - 1.0) / 0.5) ** 2)
    b /= b.sum()
    x, y = xs[:, None], ys[:, None]
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, iters)
    er, ec = oracle.marginal_err(x, y, a, b, eps, f, g)
    assert er < 1e-12
    exact = _gaussian_eot(0.0, 1.0, 1.0, 0.25, eps)
    pr, du = oracle.objectives(x, y, a, b, eps, f, g)
    assert du == pytest.approx(exact, abs=1e-10)
    assert pr == pytest.approx(exact, abs=1e-10)
    assert np.dot(a, f) + np.dot(b, g) == pytest.approx(exact, abs=1e-10)


def test_gaussian_closed_form_2d_correlated(oracle):
    """d = 2 with non-commuting covariances: pins the multi-coordinate cost."""
    k = 41
    t = np.linspace(-6.0, 6.0, k)
    gx, gy = np.meshgrid(t, t, indexing="ij")
    z = np.stack([gx.ravel(), gy.ravel()], axis=1)           # standard-normal quadrature nodes
    wz = np.exp(-0.5 * (z ** 2).sum(1))
    wz /= wz.sum()
    A = np.array([[1.0, 0.6], [0.6, 0.8]])
    B = np.array([[0.5, -0.2], [-0.2, 1.2]])
    mu_a = np.array([0.2, -0.1])
    mu_b = np.array([-0.5, 0.4])
    La, Lb = np.linalg.cholesky(A), np.linalg.cholesky(B)
    x = z @ La.T + mu_a
    y = z @ Lb.T + mu_b
    eps = _e(1.0)
    f, g = oracle.solve(x, y, wz, wz, eps, eps, 1, 200)
    er, _ = oracle.marginal_err(x, y, wz, wz, eps, f, g)
    assert er < 1e-10
    exact = _gaussian_eot(mu_a, A, mu_b, B, eps)
    _, du = oracle.objectives(x, y, wz, wz, eps, f, g)
    assert du == pytest.approx(exact, abs=1e-7)


# ----------------------------------------------------------------------------------------
# P7: invariances
# ----------------------------------------------------------------------------------------
def test_invariances(oracle):
    rng = np.random.default_rng(71)
    x, y, a, b = _problem(rng, 16, 11, 3)
    eps = _e(0.3)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 6)
    # translation
    t = np.array([0.7, -1.3, 2.0])
    f2, g2 = oracle.solve(x + t, y + t, a, b, eps, eps, 1, 6)
    np.testing.assert_allclose(f2, f, rtol=0, atol=1e-11)
    np.testing.assert_allclose(g2, g, rtol=0, atol=1e-11)
    # permutation of the points permutes the potentials
    pi, pj = rng.permutation(16), rng.permutation(11)
    f3, g3 = oracle.solve(x[pi], y[pj], a[pi], b[pj], eps, eps, 1, 6)
    np.testing.assert_allclose(f3, f[pi], rtol=0, atol=1e-12)
    np.testing.assert_allclose(g3, g[pj], rtol=0, atol=1e-12)
    # scaling (x, y, eps) -> (s x, s y, s^2 eps) scales the potentials by s^2
    s = 2.0                                    # power of two: s*s*eps stays a float32 value
    f4, g4 = oracle.solve(s * x, s * y, a, b, s * s * eps, s * s * eps, 1, 6)
    np.testing.assert_allclose(f4, s * s * f, rtol=0, atol=1e-11)
    np.testing.assert_allclose(g4, s * s * g, rtol=0, atol=1e-11)
    # splitting a target point into two copies with half the weight each
    y5 = np.vstack([y, y[:1]])
    b5 = np.concatenate([b, b[:1] * 0.5])
    b5[0] *= 0.5
    f5, g5 = oracle.solve(x, y5, a, b5, eps, eps, 1, 6)
    np.testing.assert_allclose(f5, f, rtol=0, atol=1e-12)
    assert g5[0] == pytest.approx(g5[-1], abs=1e-13)
    np.testing.assert_allclose(g5[:-1], g, rtol=0, atol=1e-12)
    # gauge: (f + c, g - c) induces the same plan
    r1, c1 = oracle.marginals(x, y, a, b, eps, f, g)
    r2, c2 = oracle.marginals(x, y, a, b, eps, f + 0.9, g - 0.9)
    np.testing.assert_allclose(r2, r1, rtol=1e-12)
    np.testing.assert_allclose(c2, c1, rtol=1e-12)


# ----------------------------------------------------------------------------------------
# P8: exact special cases
# ----------------------------------------------------------------------------------------
def test_single_target_point(oracle):
    """m = 1, b = (1), g = 0: f_i = C_i1 exactly, then g_1 = -eps*log(sum a) = 0."""
    rng = np.random.default_rng(81)
    x = rng.standard_normal((9, 4))
    y = rng.standard_normal((1, 4))
    a = rng.random(9)
    a /= a.sum()
    f, g = oracle.solve(x, y, a, np.ones(1), 0.25, 0.25, 1, 1)
    np.testing.assert_allclose(f, ((x - y) ** 2).sum(1), rtol=1e-14)
    assert abs(g[0]) <= 1e-14


def test_two_by_two_by_hand(oracle):
    """n = m = 2 on the line, one f-update written out by hand."""
    x = np.array([[0.0], [1.0]])
    y = np.array([[0.0], [2.0]])
    a = np.array([0.25, 0.75])
    b = np.array([0.4, 0.6])
    eps = _e(0.5)
    g = np.array([0.1, -0.2])
    f = oracle.update_f(x, y, b, eps, g)
    f0 = -eps * np.log(0.4 * np.exp((0.1 - 0.0) / eps) + 0.6 * np.exp((-0.2 - 4.0) / eps))
    f1 = -eps * np.log(0.4 * np.exp((0.1 - 1.0) / eps) + 0.6 * np.exp((-0.2 - 1.0) / eps))
    np.testing.assert_allclose(f, [f0, f1], rtol=1e-14)
    gg = oracle.update_g(x, y, a, eps, f)
    g0 = -eps * np.log(0.25 * np.exp((f0 - 0.0) / eps) + 0.75 * np.exp((f1 - 1.0) / eps))
    g1 = -eps * np.log(0.25 * np.exp((f0 - 4.0) / eps) + 0.75 * np.exp((f1 - 1.0) / eps))
    np.testing.assert_allclose(gg, [g0, g1], rtol=1e-14)


def test_large_scores_do_not_overflow(oracle):
    """C/eps in the thousands (plan close to a hard assignment) stays finite."""
    rng = np.random.default_rng(82)
    x = rng.standard_normal((20, 64))
    y = rng.standard_normal((20, 64)) + 1.0
    a = np.full(20, 0.05)
    f, g = oracle.solve(x, y, a, a, _e(0.05), _e(0.05), 1, 5)
    assert np.isfinite(f).all() and np.isfinite(g).all()
    f2, g2 = dense_ref.solve(x, y, a, a, [_e(0.05)], 5)
    np.testing.assert_allclose(f, f2, rtol=1e-13)


def test_zero_weight_drops_out(oracle):
    rng = np.random.default_rng(83)
    x, y, a, b = _problem(rng, 8, 6, 2)
    b0 = np.concatenate([b, [0.0]])
    y0 = np.vstack([y, [[5.0, 5.0]]])
    g0 = np.concatenate([np.zeros(6), [3.0]])
    with np.errstate(divide="ignore"):
        f0 = oracle.update_f(x, y0, b0, 0.3, g0)
    np.testing.assert_allclose(f0, oracle.update_f(x, y, b, 0.3, np.zeros(6)), rtol=1e-14)


# ----------------------------------------------------------------------------------------
# P9: plan application
# ----------------------------------------------------------------------------------------
def test_apply_plan_matches_dense(oracle):
    rng = np.random.default_rng(91)
    x, y, a, b = _problem(rng, 14, 19, 3)
    eps = _e(0.4)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 3)
    f = f + 0.05 * rng.standard_normal(14)           # not a fixed point: Prop. 3 holds anyway
    V = rng.standard_normal((19, 5))
    U = rng.standard_normal((14, 4))
    P = dense_ref.plan(x, y, a, b, eps, f, g)
    out, mass = oracle.apply_plan(x, y, a, b, eps, f, g, V, return_mass=True)
    np.testing.assert_allclose(out, P @ V, rtol=0, atol=1e-13)
    np.testing.assert_allclose(mass, P.sum(1), rtol=1e-13)
    outT, massT = oracle.apply_plan_T(x, y, a, b, eps, f, g, U, return_mass=True)
    np.testing.assert_allclose(outT, P.T @ U, rtol=0, atol=1e-13)
    np.testing.assert_allclose(massT, P.sum(0), rtol=1e-13)
    # P 1 = r and P^T 1 = c
    r, c = oracle.marginals(x, y, a, b, eps, f, g)
    np.testing.assert_allclose(oracle.apply_plan(x, y, a, b, eps, f, g, np.ones((19, 1)))[:, 0], r,
                               rtol=1e-13)
    np.testing.assert_allclose(oracle.apply_plan_T(x, y, a, b, eps, f, g, np.ones((14, 1)))[:, 0],
                               c, rtol=1e-13)
    rows = np.array([5, 5, 0])
    np.testing.assert_array_equal(oracle.apply_plan(x, y, a, b, eps, f, g, V, rows=rows), out[rows])
    cols = np.array([18, 2])
    np.testing.assert_array_equal(oracle.apply_plan_T(x, y, a, b, eps, f, g, U, cols=cols),
                                  outT[cols])


def test_prop3_attention_form_and_streaming_epilogues(oracle):
    """P V = diag(r) Softmax(S_X) V (Prop. 3); Alg. 2's epilogue a*exp(fhat/eps + m)*O and the
    c*O/s epilogue of Alg. 4 give the same numbers as the direct sum."""
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(92)
    x, y, a, b = _problem(rng, 12, 16, 3)
    eps = _e(0.3)
    f = rng.standard_normal(12) * 0.2
    g = rng.standard_normal(16) * 0.2
    V = rng.standard_normal((16, 3))
    U = rng.standard_normal((12, 2))
    alpha, beta = oracle.row_norms(x), oracle.row_norms(y)
    fhat, ghat = f - alpha, g - beta
    SX = (2.0 * x @ y.T + (ghat + eps * np.log(b))[None, :]) / eps
    SY = (2.0 * y @ x.T + (fhat + eps * np.log(a))[None, :]) / eps
    r, c = oracle.marginals(x, y, a, b, eps, f, g)
    PV = oracle.apply_plan(x, y, a, b, eps, f, g, V)
    PtU = oracle.apply_plan_T(x, y, a, b, eps, f, g, U)
    np.testing.assert_allclose(PV, r[:, None] * (softmax(SX, axis=1) @ V), rtol=0, atol=1e-13)
    np.testing.assert_allclose(PtU, c[:, None] * (softmax(SY, axis=1) @ U), rtol=0, atol=1e-13)
    # Alg. 2 epilogue
    mX = SX.max(1)
    O = np.exp(SX - mX[:, None]) @ V
    np.testing.assert_allclose(PV, (a * np.exp(fhat / eps + mX))[:, None] * O, rtol=0, atol=1e-13)
    # Alg. 4 epilogue
    mY = SY.max(1)
    E = np.exp(SY - mY[:, None])
    s = E.sum(1)
    ghat_plus = -eps * (mY + np.log(s))
    cc = b * np.exp((ghat - ghat_plus) / eps)
    np.testing.assert_allclose(cc, c, rtol=1e-12)
    np.testing.assert_allclose(PtU, (cc / s)[:, None] * (E @ U), rtol=0, atol=1e-13)
    assert logsumexp(SX, axis=1) == pytest.approx(-(oracle.update_f(x, y, b, eps, g) - alpha) / eps)


def test_barycentric_projection_at_convergence(oracle):
    """Cor. 4: at the fixed point P Y / a = Softmax_row(S_X) Y and the gradient is
    2 diag(a)(X - T)."""
    from scipy.special import softmax
    rng = np.random.default_rng(93)
    x, y, a, b = _problem(rng, 10, 13, 2)
    eps = _e(0.5)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 1500)
    PY = oracle.apply_plan(x, y, a, b, eps, f, g, y)
    beta = oracle.row_norms(y)
    SX = (2.0 * x @ y.T + (g - beta + eps * np.log(b))[None, :]) / eps
    np.testing.assert_allclose(PY / a[:, None], softmax(SX, axis=1) @ y, rtol=0, atol=1e-10)
    # gradient of the converged dual value wrt x by central differences
    i, k, h = 3, 1, 1e-5
    vals = []
    for sgn in (+1, -1):
        xp = x.copy()
        xp[i, k] += sgn * h
        fp, gp = oracle.solve(xp, y, a, b, eps, eps, 1, 1500)
        vals.append(np.dot(a, fp) + np.dot(b, gp))
    fd = (vals[0] - vals[1]) / (2 * h)
    grad = 2.0 * (a[:, None] * x - PY)
    assert fd == pytest.approx(grad[i, k], abs=1e-7)


# ----------------------------------------------------------------------------------------
# Gradient of the OT value with respect to the points (Section 2.2, Cor. 4): by the envelope
# theorem the derivative of the converged value only sees the cost, so central differences of
# the VALUE (computed from a dense plan, no plan application involved) must reproduce
# 2 (diag(a) x - P y) and 2 (diag(b) y - P^T x) built from the oracle's plan applications.
# ----------------------------------------------------------------------------------------
def test_gradient_is_the_derivative_of_the_converged_value(oracle):
    rng = np.random.default_rng(77)
    n, m, d = 6, 7, 2
    x, y, a, b = _problem(rng, n, m, d)
    eps = _e(0.5)

    def value(xx, yy):
        f, g = oracle.solve(xx, yy, a, b, eps, eps, 1, 4000)
        C = ((xx[:, None, :] - yy[None, :, :]) ** 2).sum(-1)
        P = a[:, None] * b[None, :] * np.exp((f[:, None] + g[None, :] - C) / eps)
        assert abs(P.sum() - 1.0) < 1e-10 and np.abs(P.sum(1) - a).max() < 1e-10      # converged
        return (P * C).sum() + eps * (P * np.log(P / (a[:, None] * b[None, :]))).sum()   # Eq. 1

    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 4000)
    PY = oracle.apply_plan(x, y, a, b, eps, f, g, y)
    PtX = oracle.apply_plan_T(x, y, a, b, eps, f, g, x)
    gx = 2.0 * (a[:, None] * x - PY)
    gy = 2.0 * (b[:, None] * y - PtX)
    h = 1e-5
    for (i, k) in ((0, 0), (3, 1), (5, 0)):
        xp, xm = x.copy(), x.copy()
        xp[i, k] += h
        xm[i, k] -= h
        assert abs((value(xp, y) - value(xm, y)) / (2 * h) - gx[i, k]) < 2e-6
    for (j, k) in ((1, 1), (6, 0)):
        yp, ym = y.copy(), y.copy()
        yp[j, k] += h
        ym[j, k] -= h
        assert abs((value(x, yp) - value(x, ym)) / (2 * h) - gy[j, k]) < 2e-6


# ----------------------------------------------------------------------------------------
# P10: the online LSE recurrence of App. D.3 reproduces the two-pass LSE for any tiling
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("tile", [1, 3, 8, 50])
def test_online_lse_invariant_against_oracle(oracle, tile):
    rng = np.random.default_rng(101)
    x, y, a, b = _problem(rng, 6, 37, 3)
    eps = _e(0.15)
    g = rng.standard_normal(37)
    beta = oracle.row_norms(y)
    alpha = oracle.row_norms(x)
    S = (2.0 * x @ y.T + (g - beta + eps * np.log(b))[None, :]) / eps
    mrun = np.full(6, -np.inf)
    srun = np.zeros(6)
    for j0 in range(0, 37, tile):
        blk = S[:, j0:j0 + tile]
        mnew = np.maximum(mrun, blk.max(1))
        srun = np.exp(mrun - mnew) * srun + np.exp(blk - mnew[:, None]).sum(1)
        mrun = mnew
        seen = S[:, :j0 + tile]
        np.testing.assert_allclose(srun, np.exp(seen - mrun[:, None]).sum(1), rtol=1e-13)
    fhat = -eps * (mrun + np.log(srun))
    np.testing.assert_allclose(fhat + alpha, oracle.update_f(x, y, b, eps, g), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------------------
# statistical sanity: sampled Gaussians approach the closed form (loose)
# ----------------------------------------------------------------------------------------
def test_sampled_gaussians_near_closed_form(oracle):
    from paper_2602_03067_amd import workloads
    w = workloads.make("tiny")
    f, g = oracle.solve(w.x, w.y, w.a, w.b, 0.1, 0.1, 1, 50)
    val = float(np.dot(w.a.astype(np.float64), f) + np.dot(w.b.astype(np.float64), g))
    exact = _gaussian_eot(np.zeros(3), np.eye(3), 0.5 * np.ones(3), np.eye(3), 0.1)
    assert abs(val - exact) < 0.5                      # sampling error of 1024 points in 3-d


# ---- Hessian-vector product (Thm. 5): the dense oracle against differences of the gradient ----
def test_hvp_dense_matches_central_differences_of_the_gradient(oracle):
    """G = d/dh grad_X OT(X + h A) at h = 0, with grad_X OT = 2 (diag(a) X - P* Y) (Cor. 4) taken
    at CONVERGED potentials of the perturbed clouds: shares no formula with the decomposition."""
    from oracle import hvp_dense
    rng = np.random.default_rng(17)
    n, m, d = 9, 7, 2
    x = rng.standard_normal((n, d))
    y = rng.standard_normal((m, d)) * 0.8 + 0.3
    a = rng.random(n) + 0.5
    a /= a.sum()
    b = rng.random(m) + 0.5
    b /= b.sum()
    A = rng.standard_normal((n, d))
    eps = 0.7

    def grad(xx):
        f, g = oracle.solve(xx, y, a, b, eps, eps, 1, 4000)
        PY = oracle.apply_plan(xx, y, a, b, eps, f, g, y)
        return 2.0 * (a[:, None] * xx - PY)

    h = 1e-4
    G_fd = (grad(x + h * A) - grad(x - h * A)) / (2.0 * h)
    f, g = oracle.solve(x, y, a, b, eps, eps, 1, 4000)
    G = hvp_dense.hvp(x, y, a, b, eps, f, g, A)
    assert np.abs(G - G_fd).max() <= 2e-6 * np.abs(G_fd).max()
    # a small damping changes little, and the Schur route equals the pseudo-inverse route as tau -> 0
    G_tau = hvp_dense.hvp(x, y, a, b, eps, f, g, A, tau=1e-9)
    assert np.abs(G_tau - G).max() <= 1e-5 * np.abs(G).max()
    # linear in A
    A2 = rng.standard_normal((n, d))
    lhs = hvp_dense.hvp(x, y, a, b, eps, f, g, 2.0 * A - 3.0 * A2, tau=1e-6)
    rhs = 2.0 * hvp_dense.hvp(x, y, a, b, eps, f, g, A, tau=1e-6) - 3.0 * hvp_dense.hvp(x, y, a, b, eps, f, g, A2, tau=1e-6)
    assert np.abs(lhs - rhs).max() <= 1e-9 * np.abs(rhs).max()
    # the Hessian is symmetric: <B, T A> = <A, T B>
    TB = hvp_dense.hvp(x, y, a, b, eps, f, g, A2)
    assert abs((A2 * G).sum() - (A * TB).sum()) <= 1e-8 * abs((A2 * G).sum())


# ---- Hadamard-weighted transport (Alg. 5): the dense oracle against its entry-by-entry definition ----
def test_hadamard_transport_matches_the_double_loop_and_reduces_to_a_plan_application(oracle):
    """out_i = sum_j P_ij <A_i, y_j> V_j written as plain loops over a hand-built plan (Section 2.1's
    P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps)), for potentials that are NOT converged; and with every
    row of A equal to the unit vector e_k the weights are y_jk, so the result is the ordinary plan
    application P (diag(y_k) V), which the C oracle computes with none of this code."""
    import math

    from oracle import hvp_dense
    rng = np.random.default_rng(29)
    n, m, d, p = 6, 5, 3, 4
    x, y, a, b = _problem(rng, n, m, d)
    f = rng.standard_normal(n) * 0.3
    g = rng.standard_normal(m) * 0.3
    A = rng.standard_normal((n, d))
    V = rng.standard_normal((m, p))
    eps = 0.6
    want = np.zeros((n, p))
    for i in range(n):
        for j in range(m):
            c = sum((x[i, k] - y[j, k]) ** 2 for k in range(d))
            pij = a[i] * b[j] * math.exp((f[i] + g[j] - c) / eps)
            wij = sum(A[i, k] * y[j, k] for k in range(d))
            for q in range(p):
                want[i, q] += pij * wij * V[j, q]
    got = hvp_dense.hadamard_transport(x, y, a, b, eps, f, g, A, V)
    assert np.abs(got - want).max() <= 1e-13 * np.abs(want).max()
    # default value matrix: the clouds' own y (the form Thm. 5 uses)
    got_y = hvp_dense.hadamard_transport(x, y, a, b, eps, f, g, A)
    assert np.array_equal(got_y, hvp_dense.hadamard_transport(x, y, a, b, eps, f, g, A, y))
    # a transposed or swapped operand would fail here: weights <A_i, y_j> with A_i = e_k are y_jk
    for k in range(d):
        Ak = np.zeros((n, d))
        Ak[:, k] = 1.0
        ref = oracle.apply_plan(x, y, a, b, eps, f, g, y[:, k:k + 1] * V)
        assert np.abs(hvp_dense.hadamard_transport(x, y, a, b, eps, f, g, Ak, V) - ref).max() <= 1e-13 * np.abs(ref).max()
    # linear in A, and a row scaling of A scales the matching output row
    s = rng.random(n) + 0.5
    assert np.allclose(hvp_dense.hadamard_transport(x, y, a, b, eps, f, g, s[:, None] * A, V), s[:, None] * got,
                       rtol=1e-13, atol=0)
