"""GPU parity of the low-dimension (d <= 16) path against the float64 oracle.

Tolerances: |f_gpu - f_oracle| / eps <= 1e-4 and marginal errors equal to 1e-5 (the
fp32-path bar); plan applications 2e-4 relative (Frobenius) and 1e-3 of the largest entry.
"""
import os

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


def _rand_problem(rng, n, m, d, uniform=False):
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) * 0.7 + 0.3).astype(np.float32)
    if uniform:
        a = np.full(n, 1.0 / n, dtype=np.float32)
        b = np.full(m, 1.0 / m, dtype=np.float32)
    else:
        a = rng.random(n) + 0.1
        a = (a / a.sum()).astype(np.float32)
        b = rng.random(m) + 0.1
        b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


def test_row_norms(ctx, oracle):
    rng = np.random.default_rng(1)
    for rows, d in ((1, 1), (1000, 3), (777, 64), (50, 1024)):
        say("row_norms rows=%d d=%d" % (rows, d))
        pts = rng.standard_normal((rows, d)).astype(np.float32)
        got = host(ctx.fs_row_norms(dev(pts)))
        want = oracle.row_norms(pts)
        np.testing.assert_allclose(got, want, rtol=1e-6)
    say("row_norms bf16 storage, strided")
    pts = workloads.to_bf16_round(rng.standard_normal((300, 40)).astype(np.float32))
    t = dev(pts, torch.bfloat16)[:, :33]
    got = host(ctx.fs_row_norms(t))
    np.testing.assert_allclose(got, oracle.row_norms(pts[:, :33]), rtol=1e-6)


# d = 1..16 covers every record length of the matrix-core pass (1..9 contraction steps), sizes
# cover one lane, ragged tails of row blocks and streamed tiles, and several splits
@pytest.mark.parametrize("n,m,d", [(1, 1, 3), (5, 3, 1), (255, 257, 2), (1000, 777, 3),
                                   (1024, 1024, 3), (2049, 513, 5), (300, 4100, 8), (700, 900, 16),
                                   (129, 385, 4), (640, 130, 6), (333, 2000, 7), (513, 300, 10),
                                   (260, 1100, 12), (1500, 260, 14)])
def test_single_half_steps(ctx, oracle, n, m, d):
    rng = np.random.default_rng(n * 7 + m * 3 + d)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.3))
    g = rng.standard_normal(m).astype(np.float32)
    f = rng.standard_normal(n).astype(np.float32)
    say("update_f/update_g n=%d m=%d d=%d eps=%g" % (n, m, d, eps))
    prob = make_problem(x, y, a, b)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    g_gpu = host(ctx.fs_update_g(prob, eps, dev(f)))
    assert max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps) <= TOL
    assert max_err_over_eps(g_gpu, oracle.update_g(x, y, a, eps, f), eps) <= TOL


@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("score", ["auto", "f32"])
def test_running_max_is_lifted_many_times(ctx, oracle, direction, score):
    """Potentials that rise steeply along the streamed index: every chunk of streamed points
    exceeds the running max by more than 2^60, so the lazy stabiliser has to lift the max and
    rescale in nearly every chunk (and never, after the first one, when they fall).
    The biases reach 1900 in base 2: on its own the library takes float64 scores there
    (tolerance 1e-4); with fp32 scores forced, the matrix-core pass is held to what fp32 can
    give at that magnitude (ulp 1.2e-4 of the score)."""
    rng = np.random.default_rng(11)
    n, m, d = 700, 2300, 3
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.3))
    ramp = np.linspace(0.0, 400.0, m)[::direction]
    g = (ramp + rng.standard_normal(m)).astype(np.float32)
    say("update_f with a potential ramp of 400 (%s), scores %s, n=%d m=%d"
        % ("rising" if direction > 0 else "falling", score, n, m))
    prob = make_problem(x, y, a, b)
    try:
        ctx.fs_debug_set("lowd_score", {"auto": 0, "f32": 32, "f64": 64}[score])
        f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    finally:
        ctx.fs_debug_set("lowd_score", 0)
    err = max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps)
    say("  max|df|/eps = %.3e" % err)
    assert err <= (TOL if score == "auto" else 1e-3)


def test_biases_beyond_the_digit_range_of_the_float64_grade_records(ctx, oracle):
    """d <= 3, float64-grade scores on the matrix cores: the bias of a streamed point is carried as three 8-bit digits on
    a fixed grid q plus a residual.  The library takes those records only for biases it can foresee inside the digit
    range; potentials that outgrow the bound during a solve would still meet them.  Forced here with a potential of 300
    on a cloud of radius ~0.17 at eps = 0.05: the bias is 8656 base-2 units = 2^25 q, so its leading digit needs nine
    bits and cannot be stored exactly.  The pieces must still sum to the bias, i.e. the half-step stays at fp32-grade
    accuracy of the score (2^-24 x 8656 x ln 2 = 3.6e-4 of eps) instead of carrying a rounded digit (off by up to
    2^-9 x 8656 = 17 units).  Both runs are also held by the float format of the output: |f| ~ 300 has an ulp of
    3e-5, i.e. 3e-4 of eps, which is why the bar here is not 1e-4."""
    rng = np.random.default_rng(77)
    n, m, d = 500, 1400, 3
    x = (0.05 * rng.standard_normal((n, d))).astype(np.float32)
    y = (0.05 * rng.standard_normal((m, d)) + 0.02).astype(np.float32)
    a = np.full(n, 1.0 / n, np.float32)
    b = np.full(m, 1.0 / m, np.float32)
    eps = float(np.float32(0.05))
    g = (300.0 + 0.01 * rng.standard_normal(m)).astype(np.float32)
    want = oracle.update_f(x, y, b, eps, g)
    out_rounding = 0.5 * float(np.spacing(np.float32(300.0))) / eps
    prob = make_problem(x, y, a, b)
    say("update_f with biases of ~8656 base-2 units on a cloud of radius ~0.17 (digits of the records reach ~2048)")
    f_own = host(ctx.fs_update_f(prob, eps, dev(g)))
    e_own = max_err_over_eps(f_own, want, eps)
    try:
        ctx.fs_debug_set("lowd_score", 64)
        ctx.fs_debug_set("lowd_precise_any_bias", 1)
        f_forced = host(ctx.fs_update_f(prob, eps, dev(g)))
    finally:
        ctx.fs_debug_set("lowd_score", 0)
        ctx.fs_debug_set("lowd_precise_any_bias", 0)
    e_forced = max_err_over_eps(f_forced, want, eps)
    say("  library's own choice: %.3e; records forced beyond their range: %.3e (output rounding alone: %.1e)"
        % (e_own, e_forced, out_rounding))
    assert e_own <= out_rounding * 1.05 + TOL
    assert e_forced <= out_rounding + 1e-3


def test_uniform_weights_by_null_pointer(ctx, oracle):
    rng = np.random.default_rng(5)
    n, m = 600, 500
    x, y, _, _ = _rand_problem(rng, n, m, 3)
    eps = float(np.float32(0.2))
    g = rng.standard_normal(m).astype(np.float32)
    say("update_f with a=b=NULL (uniform)")
    prob = make_problem(x, y, None, None)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    want = oracle.update_f(x, y, np.full(m, 1.0 / m), eps, g)
    assert max_err_over_eps(f_gpu, want, eps) <= TOL


def test_tiny_config_full_trajectory(ctx, oracle):
    """n = m = 1024, d = 3, eps = 0.1, 50 iterations from f = g = 0."""
    w = workloads.make("tiny")
    say("solve tiny n=%d m=%d d=%d eps=%g iters=%d" % (w.n, w.m, w.d, w.eps_end, w.iters))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    ef = max_err_over_eps(host(f), fo, w.eps_end)
    eg = max_err_over_eps(host(g), go, w.eps_end)
    say("tiny: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL and eg <= TOL
    er, ec = ctx.fs_marginal_err(prob, w.eps_end, f, g)
    # the oracle evaluates the marginals of the SAME float potentials the GPU returned
    ero, eco = oracle.marginal_err(w.x, w.y, w.a, w.b, w.eps_end, host(f), host(g))
    say("tiny: err_row gpu=%.6e oracle=%.6e  err_col gpu=%.3e oracle=%.3e" % (er, ero, ec, eco))
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5
    # and the oracle's own trajectory has the same marginal error
    ero2, eco2 = oracle.marginal_err(w.x, w.y, w.a, w.b, w.eps_end, fo, go)
    assert abs(er - ero2) <= 1e-5 and abs(ec - eco2) <= 1e-5


def test_solve_resumes_from_given_potentials(ctx, oracle):
    rng = np.random.default_rng(9)
    x, y, a, b = _rand_problem(rng, 500, 640, 3)
    eps = float(np.float32(0.25))
    prob = make_problem(x, y, a, b)
    g0 = rng.standard_normal(640).astype(np.float32) * 0.1
    say("solve warm start 500x640 + zero-iteration call")
    f = torch.full((500,), 7.0, device="cuda:0")        # never read by the first half-step
    g = dev(g0)
    ctx.fs_solve(prob, eps, eps, 1, 3, f, g)
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 3, g0=g0)
    assert max_err_over_eps(host(f), fo, eps) <= TOL
    assert max_err_over_eps(host(g), go, eps) <= TOL
    f2, g2 = f.clone(), g.clone()
    ctx.fs_solve(prob, eps, eps, 1, 0, f2, g2)           # zero iterations: unchanged
    assert torch.equal(f2, f) and torch.equal(g2, g)


def test_annealed_trajectory_scaled_down(ctx, oracle):
    """The eps-annealed workload (1.0 -> 0.01, 20 stages x 10 iterations) at n = m = 2048."""
    w = workloads.make("lowdim_anneal", n=2048, m=2048)
    say("solve lowdim_anneal n=m=2048 stages=%d iters=%d" % (w.n_stages, w.iters))
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    say("anneal 2048: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL and eg <= TOL
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    ero, eco = oracle.marginal_err(w.x, w.y, w.a, w.b, eps, host(f), host(g))
    say("anneal 2048: err_row gpu=%.6e oracle=%.6e err_col gpu=%.3e oracle=%.3e" % (er, ero, ec, eco))
    assert abs(er - ero) <= 1e-5 and abs(ec - eco) <= 1e-5


def test_annealed_trajectory_8192(ctx, oracle):
    """Same annealed workload at n = m = 8192 (several row blocks, two rows per lane)."""
    w = workloads.make("lowdim_anneal", n=8192, m=8192)
    say("solve lowdim_anneal n=m=8192 (oracle takes ~40 s)")
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    say("anneal 8192: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL and eg <= TOL


def _staged_oracle_trajectory(oracle, w, tag):
    """The oracle's annealed trajectory, one stage per call (the same arithmetic as one call: g is carried over and
    f is never read), with a progress line per stage so that a long run is seen to be alive."""
    go = np.zeros(w.m)
    fo = np.zeros(w.n)
    for s in range(w.n_stages):
        eps_s = oracle.stage_eps(w.eps_start, w.eps_end, w.n_stages, s)
        fo, go = oracle.solve(w.x, w.y, w.a, w.b, eps_s, eps_s, 1, w.iters, g0=go)
        say("  %s: oracle stage %d/%d (eps=%.5f) done" % (tag, s + 1, w.n_stages, eps_s))
    return fo, go


def _trajectory_case(ctx, oracle, n):
    w = workloads.make("lowdim_anneal", n=n, m=n)
    say("solve lowdim_anneal n=m=%d, full oracle trajectory stage by stage" % n)
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    fo, go = _staged_oracle_trajectory(oracle, w, "anneal %d" % n)
    eps = float(np.float32(w.eps_end))
    ef = max_err_over_eps(host(f), fo, eps)
    eg = max_err_over_eps(host(g), go, eps)
    say("anneal %d: max|df|/eps=%.3e max|dg|/eps=%.3e" % (n, ef, eg))
    return ef, eg


def test_annealed_trajectory_16384(ctx, oracle):
    """The annealed workload at n = m = 16384 against the oracle's full trajectory: the third point of the trend of
    the trajectory error with the size (2048, 8192, 16384), which the bench size cannot have (its oracle trajectory
    would take hours)."""
    ef, eg = _trajectory_case(ctx, oracle, 16384)
    assert ef <= TOL and eg <= TOL


@pytest.mark.skipif(not os.environ.get("FS_SLOW_TESTS"), reason="about three minutes of oracle time: set FS_SLOW_TESTS=1")
def test_annealed_trajectory_32768(ctx, oracle):
    ef, eg = _trajectory_case(ctx, oracle, 32768)
    assert ef <= TOL and eg <= TOL


def test_full_size_lowdim_every_stage_sampled(ctx, oracle):
    """n = m = 262144, d = 3 in the launch configuration the bench times, checked ALONG the annealed run and not only
    at its end: the solve is run stage by stage (potentials handed over in float, as a caller would), and after every
    stage one more f-update and g-update at that stage's eps are re-derived by the oracle on 256 sampled rows and
    columns.  Every such half-step must hold the 1e-4 bar in units of its own eps.  Printed, not asserted: the sum over
    all 400 half-steps of these errors in absolute terms, divided by the final eps -- what the trajectory error could
    be at worst if every half-step erred by its sampled maximum in the same direction and nothing was damped (a
    half-step is non-expansive in the sup norm, so errors add at most).  That worst case is above the bar by
    construction: fp32 scores are off by ~2^-24 of their magnitude, i.e. by ~1e-7 in a potential whatever the eps,
    which is 1e-5 of the final eps per half-step.  What does add up in practice is only the part of these errors that
    is common to all rows (a shift along the iteration's neutral direction f + t, g - t), which fs_solve measures and
    takes out; what is left is seen in the full oracle trajectories at the sizes the oracle can afford: 1e-5 eps at
    every size from 2048 to 32768 (tests above)."""
    w = workloads.make("lowdim_anneal")
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    rng = np.random.default_rng(2024)
    rows = np.sort(rng.choice(w.n, size=256, replace=False))
    cols = np.sort(rng.choice(w.m, size=256, replace=False))
    worst = 0.0
    sum_abs = 0.0
    for s in range(w.n_stages):
        eps_s = oracle.stage_eps(w.eps_start, w.eps_end, w.n_stages, s)
        say("full size, stage %d/%d: eps=%.5f, %d iterations, then sampled half-steps" % (s + 1, w.n_stages, eps_s, w.iters))
        ctx.fs_solve(prob, eps_s, eps_s, 1, w.iters, f, g)
        f_next = ctx.fs_update_f(prob, eps_s, g)
        g_next = ctx.fs_update_g(prob, eps_s, f_next)
        torch.cuda.synchronize()
        gh, fnh = host(g), host(f_next)
        ef = max_err_over_eps(fnh[rows], oracle.update_f(w.x, w.y, w.b, eps_s, gh, rows=rows), eps_s)
        eg = max_err_over_eps(host(g_next)[cols], oracle.update_g(w.x, w.y, w.a, eps_s, fnh, cols=cols), eps_s)
        say("  sampled max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
        assert np.isfinite(fnh).all()
        assert ef <= TOL and eg <= TOL
        worst = max(worst, ef, eg)
        sum_abs += w.iters * (ef + eg) * eps_s
    eps_end = float(np.float32(w.eps_end))
    say("full size: worst sampled half-step error along the run %.3e (units of its eps); worst-case sum of all %d "
        "half-step errors %.3e of the final eps (not a bound the bar applies to, see the docstring)"
        % (worst, 2 * w.total_iters, sum_abs / eps_end))


# (p = 1 runs the kernel with the products on the vector ALU, as does p <= 4 at d = 16; everything else has them on the
# matrix cores: up to eight columns in one pass with the values in three bf16 pieces, more in passes of fifteen with two
# pieces: p = 9 and 12 are one pass, 16 and 17 two (the second with one and two columns), 31 three)
@pytest.mark.parametrize("n,m,d,p", [(300, 200, 3, 3), (1000, 1300, 3, 1), (513, 255, 2, 7), (260, 300, 8, 5), (700, 900, 3, 8),
                                     (450, 520, 1, 9), (390, 1100, 5, 17), (640, 300, 16, 16), (300, 640, 16, 3),
                                     (1200, 900, 12, 12), (333, 444, 4, 31), (250, 380, 3, 15)])
def test_apply_plan_and_transpose(ctx, oracle, n, m, d, p):
    rng = np.random.default_rng(n + m + d + p)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.3))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 4)
    f32 = (fo + 0.02 * rng.standard_normal(n)).astype(np.float32)   # not a fixed point
    g32 = go.astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    U = rng.standard_normal((n, p)).astype(np.float32)
    say("apply_plan / apply_plan_T n=%d m=%d d=%d p=%d" % (n, m, d, p))
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


@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("p", [1, 3])
@pytest.mark.parametrize("span", [18.0, 150.0])
def test_apply_with_a_running_max_that_is_lifted(ctx, oracle, direction, p, span):
    """Plan application with potentials that rise (fall) steeply along the streamed index: the lazy stabiliser of the
    application lifts the max along the way and rescales the output accumulators with it (vector-ALU products for
    p = 1, matrix-core products for p = 3).  A ramp of 18 spans 87 base-2 units at eps = 0.3: beyond the 2^60 window,
    still fp32 scores; a ramp of 150 spans 720, a dozen lifts, and the library takes its float64-grade records."""
    rng = np.random.default_rng(23 + p)
    n, m, d = 600, 2300, 3
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.3))
    ramp = np.linspace(0.0, span, m)[::direction]
    g32 = (ramp + 0.1 * rng.standard_normal(m)).astype(np.float32)
    f32 = oracle.update_f(x, y, b, eps, g32).astype(np.float32)
    V = (rng.standard_normal((m, p)) + 2.0).astype(np.float32)
    say("apply_plan under a potential ramp of %g (%s), n=%d m=%d p=%d" % (span, "rising" if direction > 0 else "falling", n, m, p))
    prob = make_problem(x, y, a, b)
    out, mass = ctx.fs_apply_plan(prob, eps, dev(f32), dev(g32), dev(V), want_mass=True)
    want, r = oracle.apply_plan(x, y, a, b, eps, f32, g32, V, return_mass=True)
    got = host(out)
    say("  rel. Frobenius %.2e, max-abs / max %.2e" % (np.linalg.norm(got - want) / np.linalg.norm(want),
                                                      np.abs(got - want).max() / np.abs(want).max()))
    assert np.linalg.norm(got - want) <= 2e-4 * np.linalg.norm(want)
    assert np.abs(got - want).max() <= 1e-3 * np.abs(want).max()
    np.testing.assert_allclose(host(mass), r, rtol=2e-4)


def test_zero_weight_points_drop_out(ctx, oracle):
    rng = np.random.default_rng(77)
    x, y, a, b = _rand_problem(rng, 300, 280, 3)
    b0 = b.copy()
    b0[:5] = 0.0
    eps = float(np.float32(0.3))
    g = rng.standard_normal(280).astype(np.float32)
    say("update_f with five zero target weights")
    prob = make_problem(x, y, a, b0)
    f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
    want = oracle.update_f(x[:, :], y[5:], b0[5:], eps, g[5:])
    assert np.isfinite(f_gpu).all()
    assert max_err_over_eps(f_gpu, want, eps) <= TOL


def test_full_size_lowdim_sampled_rows(ctx, oracle):
    """n = m = 262144, d = 3 in the launch configuration the bench times: one annealed solve on
    the GPU, then the last two half-steps are re-derived by the oracle on 256 sampled rows."""
    w = workloads.make("lowdim_anneal")
    say("solve lowdim_anneal FULL n=m=%d" % w.n)
    prob = binding.problem_from_workload(w)
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")
    # all but the last iteration, then the last one by hand so that the inputs of the last
    # half-steps are known float vectors
    ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    torch.cuda.synchronize()
    assert torch.isfinite(f).all() and torch.isfinite(g).all()
    eps = float(np.float32(w.eps_end))
    rng = np.random.default_rng(4242)
    rows = np.sort(rng.choice(w.n, size=256, replace=False))
    say("full size: one more f-update and g-update on the GPU, oracle on sampled rows")
    f_next = ctx.fs_update_f(prob, eps, g)
    g_next = ctx.fs_update_g(prob, eps, f_next)
    gh, fh = host(g), host(f_next)
    want_f = oracle.update_f(w.x, w.y, w.b, eps, gh, rows=rows)
    want_g = oracle.update_g(w.x, w.y, w.a, eps, fh, cols=rows)
    ef = max_err_over_eps(host(f_next)[rows], want_f, eps)
    eg = max_err_over_eps(host(g_next)[rows], want_g, eps)
    say("full size: sampled max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= TOL and eg <= TOL
    # properties that hold at any size: the column marginal is exact after a g-update
    er, ec = ctx.fs_marginal_err(prob, eps, f, g)
    say("full size: err_row=%.4e err_col=%.4e" % (er, ec))
    assert ec <= 1e-4 and 0.0 <= er < 2.0
    # sampled row marginals from the oracle agree with Prop. 3 evaluated on the GPU output
    r_or = oracle.apply_plan(w.x, w.y, w.a, w.b, eps, host(f), gh, np.ones((w.m, 1)), rows=rows)[:, 0]
    f_plus = host(ctx.fs_update_f(prob, eps, g))[rows]
    r_gpu = w.a[rows].astype(np.float64) * np.exp((host(f)[rows] - f_plus) / eps)
    np.testing.assert_allclose(r_gpu, r_or, rtol=5e-4)
    # the two plan applications of the bench step on sampled rows / columns: the gradient x - (P y)/a (three value
    # columns) and P^T U with the workload's U, and one with eleven columns (two passes, the second with three)
    fh0 = host(f)
    say("full size: plan applications on sampled rows")
    grad = host(ctx.fs_grad_x(prob, eps, f, g, 2))[rows]
    T = oracle.apply_plan(w.x, w.y, w.a, w.b, eps, fh0, gh, w.y, rows=rows)
    want_grad = w.x[rows].astype(np.float64) - T / w.a[rows].astype(np.float64)[:, None]
    scale = np.abs(w.x).max()
    eg = np.abs(grad - want_grad).max() / scale
    say("full size: gradient max abs error / max|x| = %.3e" % eg)
    assert eg <= 1e-4
    U = np.random.default_rng(77).standard_normal((w.n, 11)).astype(np.float32)
    outT, cm = ctx.fs_apply_plan_T(prob, eps, f, g, dev(U), want_mass=True)
    wantT, c_or = oracle.apply_plan_T(w.x, w.y, w.a, w.b, eps, fh0, gh, U, cols=rows, return_mass=True)
    gotT = host(outT)[rows]
    eT = np.linalg.norm(gotT - wantT) / np.linalg.norm(wantT)
    say("full size: P^T U on sampled columns, rel. Frobenius %.3e, max-abs / max %.3e"
        % (eT, np.abs(gotT - wantT).max() / np.abs(wantT).max()))
    assert eT <= 2e-4 and np.abs(gotT - wantT).max() <= 1e-3 * np.abs(wantT).max()
    np.testing.assert_allclose(host(cm)[rows], c_or, rtol=2e-4)


@pytest.mark.parametrize("n,m,d", [(1500000, 1048576 + 77, 2), (3000000, 130, 5)])
def test_million_points_sampled_rows(ctx, oracle, n, m, d):
    """Sizes well beyond the bench's: one f-update and one g-update (more than 10^12 pairs in the
    first case), checked by the oracle on 64 sampled rows and columns."""
    rng = np.random.default_rng(n + m + d)
    x = rng.random((n, d)).astype(np.float32)
    y = (rng.random((m, d)) * 0.8 + 0.1).astype(np.float32)
    a = np.full(n, 1.0 / n, dtype=np.float32)
    b = rng.random(m).astype(np.float32) + 0.5
    b /= b.sum()
    eps = float(np.float32(0.05))
    g0 = (0.1 * rng.standard_normal(m)).astype(np.float32)
    say("large sizes: update_f / update_g n=%d m=%d d=%d" % (n, m, d))
    prob = make_problem(x, y, a, b)
    f1 = ctx.fs_update_f(prob, eps, dev(g0))
    g1 = ctx.fs_update_g(prob, eps, f1)
    torch.cuda.synchronize()
    f1h = host(f1)
    rows = np.sort(rng.choice(n, size=64, replace=False))
    cols = np.sort(rng.choice(m, size=64, replace=False))
    ef = max_err_over_eps(f1h[rows], oracle.update_f(x, y, b, eps, g0, rows=rows), eps)
    eg = max_err_over_eps(host(g1)[cols], oracle.update_g(x, y, a, eps, f1h, cols=cols), eps)
    say("  sampled max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert np.isfinite(f1h).all() and ef <= TOL and eg <= TOL


@pytest.mark.parametrize("n,m,d,p", [(300, 421, 4, 1), (129, 1000, 7, 5), (1100, 260, 12, 70), (640, 700, 16, 64)])
def test_float64_scores_above_three_dimensions(ctx, oracle, n, m, d, p):
    """3 < d <= 16 with float64 scores (forced here; on its own the library takes them at small eps and
    on long runs): half-steps, both plan applications and the Hessian-vector product then run on the
    fp64 matrix-core kernels, from centred float64 records of the low-dimension prologue."""
    from oracle import hvp_dense
    rng = np.random.default_rng(5 * n + m + d)
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.5))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 30)
    f32 = (fo + 0.02 * rng.standard_normal(n)).astype(np.float32)
    g32 = go.astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    U = rng.standard_normal((n, p)).astype(np.float32)
    A = rng.standard_normal((n, d)).astype(np.float32)
    say("float64 scores forced, n=%d m=%d d=%d p=%d" % (n, m, d, p))
    prob = make_problem(x, y, a, b)
    ctx.fs_debug_set("lowd_score", 64)
    try:
        f_gpu = host(ctx.fs_update_f(prob, eps, dev(g32)))
        g_gpu = host(ctx.fs_update_g(prob, eps, dev(f32)))
        out, mass = ctx.fs_apply_plan(prob, eps, dev(f32), dev(g32), dev(V), want_mass=True)
        outT, massT = ctx.fs_apply_plan_T(prob, eps, dev(f32), dev(g32), dev(U), want_mass=True)
        fs, gs = torch.zeros(n, device="cuda:0"), torch.zeros(m, device="cuda:0")
        ctx.fs_solve_symmetric(prob, eps, 6, fs, gs)
        G, k = ctx.fs_hvp(prob, eps, dev(fo.astype(np.float32)), dev(g32), dev(A), 1e-5, 1e-6, 400)
    finally:
        ctx.fs_debug_set("lowd_score", 0)
    assert max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g32), eps) <= TOL
    assert max_err_over_eps(g_gpu, oracle.update_g(x, y, a, eps, f32), eps) <= TOL
    want, r = oracle.apply_plan(x, y, a, b, eps, f32, g32, V, return_mass=True)
    wantT, c = oracle.apply_plan_T(x, y, a, b, eps, f32, g32, U, return_mass=True)
    for got, ref in ((host(out), want), (host(outT), wantT)):
        assert np.linalg.norm(got - ref) <= 2e-4 * np.linalg.norm(ref)
        assert np.abs(got - ref).max() <= 1e-3 * np.abs(ref).max()
    np.testing.assert_allclose(host(mass), r, rtol=2e-4)
    np.testing.assert_allclose(host(massT), c, rtol=2e-4)
    fso, gso = oracle.solve_symmetric(x, y, a, b, eps, 6)
    assert max_err_over_eps(host(fs), fso, eps) <= TOL and max_err_over_eps(host(gs), gso, eps) <= TOL
    fh = fo.astype(np.float32).astype(np.float64)
    wantG = hvp_dense.hvp(x, y, a, b, eps, fh, g32.astype(np.float64), A, tau=1e-5)
    rel = np.linalg.norm(host(G) - wantG) / np.linalg.norm(wantG)
    say("  hvp: %d CG iterations, rel. error %.3e" % (k, rel))
    assert rel <= 1e-4


def test_float64_scores_above_three_dimensions_many_blocks(ctx, oracle):
    """The same kernels at a size with hundreds of row blocks and several splits (n = 30000, m = 21000,
    d = 8, float64 scores forced), checked by the oracle on sampled rows and columns."""
    rng = np.random.default_rng(77)
    n, m, d = 30000, 21000, 8
    x = rng.random((n, d)).astype(np.float32)
    y = (rng.random((m, d)) * 0.9 + 0.05).astype(np.float32)
    a = rng.random(n) + 0.5
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.5
    b = (b / b.sum()).astype(np.float32)
    eps = float(np.float32(0.05))
    g = (0.1 * rng.standard_normal(m)).astype(np.float32)
    f = (0.1 * rng.standard_normal(n)).astype(np.float32)
    rows = np.sort(rng.choice(n, 200, replace=False))
    cols = np.sort(rng.choice(m, 200, replace=False))
    say("float64 scores forced at n=%d m=%d d=%d, sampled rows" % (n, m, d))
    prob = make_problem(x, y, a, b)
    ctx.fs_debug_set("lowd_score", 64)
    try:
        f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
        g_gpu = host(ctx.fs_update_g(prob, eps, dev(f)))
        V = rng.standard_normal((m, 3)).astype(np.float32)
        out = host(ctx.fs_apply_plan(prob, eps, dev(f_gpu), dev(g), dev(V)))
    finally:
        ctx.fs_debug_set("lowd_score", 0)
    assert max_err_over_eps(f_gpu[rows], oracle.update_f(x, y, b, eps, g, rows=rows), eps) <= TOL
    assert max_err_over_eps(g_gpu[cols], oracle.update_g(x, y, a, eps, f, cols=cols), eps) <= TOL
    want = oracle.apply_plan(x, y, a, b, eps, f_gpu, g, V, rows=rows)
    assert np.linalg.norm(out[rows] - want) <= 2e-4 * np.linalg.norm(want)


@pytest.mark.parametrize("hook,value", [("lowd_splits", 1), ("lowd_splits", 7), ("lowd_precise_valu", 1)])
def test_alternative_launch_shapes_and_kernels_agree(ctx, oracle, hook, value):
    """The library's experiment switches (a forced split count of the streamed side; float64 scores on the
    vector ALU instead of the precise split records) must give the same potentials: a cross-check of the
    split merge and of the two float64-score kernels at d <= 3."""
    rng = np.random.default_rng(41)
    n, m, d = 1500, 5000, 3
    x, y, a, b = _rand_problem(rng, n, m, d)
    eps = float(np.float32(0.01))   # small enough for float64 scores
    g = (0.05 * rng.standard_normal(m)).astype(np.float32)
    f = (0.05 * rng.standard_normal(n)).astype(np.float32)
    say("update_f/update_g with the context switch %s=%s, n=%d m=%d d=%d eps=%g" % (hook, value, n, m, d, eps))
    prob = make_problem(x, y, a, b)
    ctx.fs_debug_set(hook, value)
    try:
        f_gpu = host(ctx.fs_update_f(prob, eps, dev(g)))
        g_gpu = host(ctx.fs_update_g(prob, eps, dev(f)))
    finally:
        ctx.fs_debug_set(hook, 0)
    assert max_err_over_eps(f_gpu, oracle.update_f(x, y, b, eps, g), eps) <= TOL
    assert max_err_over_eps(g_gpu, oracle.update_g(x, y, a, eps, f), eps) <= TOL
