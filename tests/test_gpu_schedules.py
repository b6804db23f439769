"""GPU parity of fs_solve_symmetric (Eq. 4-5, the averaged Jacobi schedule) and of fs_solve_tol (early
stopping on the row marginal error) against the float64
oracle, on the three arithmetic paths.  Tolerances as for fs_solve: |df|/eps <= 1e-4 in fp32-accuracy
mode, <= 2e-2 in bf16 mode against the oracle on the unrounded inputs (and 2e-4 against the oracle
on the bf16-rounded inputs, which separates rounding of the data from the kernels' arithmetic)."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return binding.Context(0)


def _problem(rng, n, m, d, scale):
    x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    y = (rng.standard_normal((m, d)) * scale * 0.8 + 0.2 * scale).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.1
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


@pytest.mark.parametrize("n,m,d,eps,iters", [(300, 421, 3, 0.25, 25), (1030, 700, 2, 0.05, 12),   # low-d passes
                                             (260, 300, 8, 0.5, 10),
                                             # very different split counts of the two passes that share a launch
                                             (2100, 150, 3, 0.2, 6), (77, 6000, 3, 0.3, 6),
                                             (500, 900, 3, 0.01, 8),   # float64-score half-steps
                                             (200, 333, 40, 2.0, 15), (130, 257, 64, 1.0, 8),      # fp64 MFMA pass
                                             # the paired fp64 pass with very different shapes of its two halves,
                                             # and on behalf of the low-d path (float64 scores at d = 8)
                                             (2100, 150, 64, 1.0, 5), (90, 5000, 40, 2.0, 5), (700, 400, 8, 0.03, 5)])
def test_symmetric_fp32_mode(ctx, oracle, n, m, d, eps, iters):
    rng = np.random.default_rng(1000 * n + m + d)
    x, y, a, b = _problem(rng, n, m, d, 1.0 if d <= 16 else 0.5)
    eps = float(np.float32(eps))
    f0 = (0.1 * rng.standard_normal(n)).astype(np.float32)
    g0 = (0.1 * rng.standard_normal(m)).astype(np.float32)
    say("solve_symmetric n=%d m=%d d=%d eps=%g iters=%d (non-zero start)" % (n, m, d, eps, iters))
    fo, go = oracle.solve_symmetric(x, y, a, b, eps, iters, f0=f0.astype(np.float64), g0=g0.astype(np.float64))
    prob = make_problem(x, y, a, b)
    f, g = dev(f0), dev(g0)
    ctx.fs_solve_symmetric(prob, eps, iters, f, g)
    ef, eg = max_err_over_eps(host(f), fo, eps), max_err_over_eps(host(g), go, eps)
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= 1e-4 and eg <= 1e-4


def test_symmetric_long_run_at_a_larger_size(ctx, oracle):
    """80 averaged iterations at a small eps on two clouds of different shape (uniform cube against a clustered
    mixture, n = m = 12288): the run where a systematic difference between the roundings of the f-pass and of the
    g-pass would add up along the iteration's neutral direction (f + t, g - t) if it were not measured and removed."""
    from paper_2602_03067_amd import workloads
    w = workloads.make("lowdim_anneal", n=12288, m=12288)
    eps = float(np.float32(0.02))
    iters = 80
    say("solve_symmetric on the annealed workload's clouds, n=m=%d eps=%g iters=%d" % (w.n, eps, iters))
    fo, go = oracle.solve_symmetric(w.x, w.y, w.a, w.b, eps, iters)
    prob = make_problem(w.x, w.y, w.a, w.b)
    f, g = dev(np.zeros(w.n, dtype=np.float32)), dev(np.zeros(w.m, dtype=np.float32))
    ctx.fs_solve_symmetric(prob, eps, iters, f, g)
    df, dg = (host(f) - fo) / eps, (host(g) - go) / eps
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e (mean shifts %.3e, %.3e)" % (np.abs(df).max(), np.abs(dg).max(), df.mean(), dg.mean()))
    assert np.abs(df).max() <= 1e-4 and np.abs(dg).max() <= 1e-4


def test_symmetric_equal_clouds_keep_f_equal_g(ctx, oracle):
    """x = y and a = b: under the symmetric schedule f = g at every iteration (the oracle is pinned
    to this); on the GPU the two passes are the same arithmetic on swapped roles."""
    rng = np.random.default_rng(5)
    n, d = 777, 3
    x, _, a, _ = _problem(rng, n, n, d, 1.0)
    eps = float(np.float32(0.2))
    say("solve_symmetric with x = y, a = b: f must equal g, n=%d" % n)
    prob = make_problem(x, x, a, a)
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(n, device="cuda:0")
    ctx.fs_solve_symmetric(prob, eps, 9, f, g)
    fo, go = oracle.solve_symmetric(x, x, a, a, eps, 9)
    assert float(np.max(np.abs(host(f) - host(g)))) / eps <= 2e-6
    assert max_err_over_eps(host(f), fo, eps) <= 1e-4


@pytest.mark.parametrize("n,m,d", [(300, 520, 96), (3000, 260, 64)])
def test_symmetric_bf16_mode(ctx, oracle, n, m, d):
    rng = np.random.default_rng(77 + n)
    x, y, a, b = _problem(rng, n, m, d, 0.3)
    eps = float(np.float32(1.5))
    iters = 10
    say("solve_symmetric bf16 mode n=%d m=%d d=%d eps=%g iters=%d" % (n, m, d, eps, iters))
    prob = make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA)
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    ctx.fs_solve_symmetric(prob, eps, iters, f, g)
    fa, ga = oracle.solve_symmetric(x, y, a, b, eps, iters)
    xb, yb = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    fb, gb = oracle.solve_symmetric(xb, yb, a, b, eps, iters)
    ea = max(max_err_over_eps(host(f), fa, eps), max_err_over_eps(host(g), ga, eps))
    eb = max(max_err_over_eps(host(f), fb, eps), max_err_over_eps(host(g), gb, eps))
    say("  vs oracle on bf16-rounded inputs %.3e, vs oracle on given inputs %.3e" % (eb, ea))
    assert ea <= 2e-2 and eb <= 2e-4


def test_symmetric_zero_iterations_leaves_potentials(ctx):
    rng = np.random.default_rng(3)
    x, y, a, b = _problem(rng, 50, 60, 3, 1.0)
    prob = make_problem(x, y, a, b)
    f0 = rng.standard_normal(50).astype(np.float32)
    g0 = rng.standard_normal(60).astype(np.float32)
    f, g = dev(f0), dev(g0)
    say("solve_symmetric with iters=0")
    ctx.fs_solve_symmetric(prob, 0.3, 0, f, g)
    assert np.array_equal(host(f), f0.astype(np.float64)) and np.array_equal(host(g), g0.astype(np.float64))


# ---- early stopping on the row marginal error (fs_solve_tol) ---------------------------------
@pytest.mark.parametrize("n,m,d,eps", [(400, 500, 3, 0.1), (300, 260, 40, 0.15)])
def test_solve_tol_stops_where_the_oracle_does(ctx, oracle, n, m, d, eps):
    rng = np.random.default_rng(31 * n + d)
    x, y, a, b = _problem(rng, n, m, d, 1.0 if d <= 16 else 0.4)
    eps = float(np.float32(eps))
    check_every, max_iters = 3, 30
    # the oracle's trajectory and its row errors at the check points
    fo, go = np.zeros(n), np.zeros(m)
    errs = {}
    for t in range(1, max_iters + 1):
        fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 1, f0=fo, g0=go)
        if t % check_every == 0:
            errs[t] = (oracle.marginal_err(x, y, a, b, eps, fo, go)[0], fo.copy(), go.copy())
    checks = sorted(errs)
    # a tolerance well between the errors at the third and fourth check, so that both sides stop at the fourth
    tol = float(np.sqrt(errs[checks[2]][0] * errs[checks[3]][0]))
    say("solve_tol n=%d m=%d d=%d eps=%g: oracle errors at checks %s, tol=%.3e"
        % (n, m, d, eps, ["%.2e" % errs[t][0] for t in checks[:5]], tol))
    prob = make_problem(x, y, a, b)
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    done, err = ctx.fs_solve_tol(prob, eps, max_iters, check_every, tol, f, g)
    want_err, want_f, want_g = errs[checks[3]]
    say("  stopped after %d iterations with error %.6e (oracle: %d, %.6e)" % (done, err, checks[3], want_err))
    assert done == checks[3]
    assert abs(err - want_err) <= 1e-5
    assert max_err_over_eps(host(f), want_f, eps) <= 1e-4 and max_err_over_eps(host(g), want_g, eps) <= 1e-4


def test_solve_tol_runs_to_max_iters(ctx, oracle):
    rng = np.random.default_rng(8)
    n, m, d = 200, 150, 3
    x, y, a, b = _problem(rng, n, m, d, 1.0)
    eps = float(np.float32(0.05))
    say("solve_tol with tol = 0: runs all 7 iterations")
    prob = make_problem(x, y, a, b)
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    done, err = ctx.fs_solve_tol(prob, eps, 7, 5, 0.0, f, g)
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 7)
    assert done == 7
    assert abs(err - oracle.marginal_err(x, y, a, b, eps, fo, go)[0]) <= 1e-5
    assert max_err_over_eps(host(f), fo, eps) <= 1e-4 and max_err_over_eps(host(g), go, eps) <= 1e-4


# ---- extreme aspect ratio: a few hundred rows against tens of thousands (split reduction) ------
@pytest.mark.parametrize("d,mode", [(3, "fp32"), (64, "fp32"), (64, "bf16")])
def test_few_rows_many_columns(ctx, oracle, d, mode):
    """n = 500, m = 50000: the f-update has two to eight row blocks, so nearly all parallelism comes
    from splitting the streamed side into hundreds of pieces that are merged afterwards; the
    g-update is the opposite shape."""
    rng = np.random.default_rng(500 + d)
    n, m = 500, 50000
    x, y, a, b = _problem(rng, n, m, d, 1.0 if d <= 16 else 0.35)
    eps = float(np.float32(0.3 if d <= 16 else 1.0))
    g0 = (0.2 * rng.standard_normal(m)).astype(np.float32)
    f0 = (0.2 * rng.standard_normal(n)).astype(np.float32)
    say("update_f / update_g n=%d m=%d d=%d %s mode" % (n, m, d, mode))
    if mode == "bf16":
        prob = make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA)
        xo, yo, tol = workloads.to_bf16_round(x), workloads.to_bf16_round(y), 2e-4
    else:
        prob = make_problem(x, y, a, b)
        xo, yo, tol = x, y, 1e-4
    f = host(ctx.fs_update_f(prob, eps, dev(g0)))
    g = host(ctx.fs_update_g(prob, eps, dev(f0)))
    ef = max_err_over_eps(f, oracle.update_f(xo, yo, b, eps, g0), eps)
    eg = max_err_over_eps(g, oracle.update_g(xo, yo, a, eps, f0), eps)
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= tol and eg <= tol
