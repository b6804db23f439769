"""GPU parity of fs_ot_value (dual objective of App. B at given potentials) against the oracle."""
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


@pytest.mark.parametrize("n,m,d,eps,iters", [(300, 421, 3, 0.25, 6), (700, 200, 2, 0.05, 30), (130, 257, 64, 1.0, 5)])
def test_value_matches_oracle_dual(ctx, oracle, n, m, d, eps, iters):
    rng = np.random.default_rng(n + 3 * m + d)
    x, y, a, b = _problem(rng, n, m, d, 1.0 if d <= 16 else 0.5)
    eps = float(np.float32(eps))
    # potentials part-way to convergence (so that the mass term eps (sum P - 1) is not zero),
    # rounded to float: the same float values go to both sides
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, iters)
    f32 = (fo + 0.01 * rng.standard_normal(n)).astype(np.float32)
    g32 = go.astype(np.float32)
    say("ot_value n=%d m=%d d=%d eps=%g" % (n, m, d, eps))
    _, dual = oracle.objectives(x, y, a, b, eps, f32.astype(np.float64), g32.astype(np.float64))
    got = ctx.fs_ot_value(make_problem(x, y, a, b), eps, dev(f32), dev(g32))
    say("  dual gpu=%.9f oracle=%.9f" % (got, dual))
    assert abs(got - dual) <= 1e-5 * (abs(dual) + eps)


def test_value_bf16_mode(ctx, oracle):
    rng = np.random.default_rng(9)
    n, m, d = 260, 300, 96
    x, y, a, b = _problem(rng, n, m, d, 0.3)
    eps = float(np.float32(1.5))
    xb, yb = workloads.to_bf16_round(x), workloads.to_bf16_round(y)
    fo, go = oracle.solve(xb, yb, a, b, eps, eps, 1, 4)
    f32, g32 = fo.astype(np.float32), (go + 0.01 * rng.standard_normal(m)).astype(np.float32)
    say("ot_value bf16 mode n=%d m=%d d=%d" % (n, m, d))
    _, dual_b = oracle.objectives(xb, yb, a, b, eps, f32.astype(np.float64), g32.astype(np.float64))
    got = ctx.fs_ot_value(make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA), eps, dev(f32), dev(g32))
    say("  dual gpu=%.9f oracle on bf16-rounded inputs=%.9f" % (got, dual_b))
    assert abs(got - dual_b) <= 2e-4 * (abs(dual_b) + eps)


def test_debiased_divergence_from_three_solves(ctx, oracle):
    """S(a, b) = OT(a, b) - OT(a, a)/2 - OT(b, b)/2 with each term the dual value after a fixed
    number of iterations from zero potentials: three fs_solve + fs_ot_value calls through the ABI,
    against the same composition of the oracle's functions."""
    rng = np.random.default_rng(21)
    n, m, d = 350, 290, 3
    x, y, a, b = _problem(rng, n, m, d, 1.0)
    eps = float(np.float32(0.2))
    iters = 40

    def gpu_value(p, q, wp, wq):
        prob = make_problem(p, q, wp, wq)
        f = torch.zeros(len(p), device="cuda:0")
        g = torch.zeros(len(q), device="cuda:0")
        ctx.fs_solve(prob, eps, eps, 1, iters, f, g)
        return ctx.fs_ot_value(prob, eps, f, g), f, g

    def oracle_value(p, q, wp, wq, f32, g32):
        # the dual value at the SAME float potentials (the solve itself is covered by the solver tests)
        return oracle.objectives(p, q, wp, wq, eps, f32.astype(np.float64), g32.astype(np.float64))[1]

    say("debiased divergence from three solves, n=%d m=%d" % (n, m))
    total_gpu, total_ref = 0.0, 0.0
    for (p, q, wp, wq, coef) in ((x, y, a, b, 1.0), (x, x, a, a, -0.5), (y, y, b, b, -0.5)):
        v, f, g = gpu_value(p, q, wp, wq)
        fo, go = oracle.solve(p, q, wp, wq, eps, eps, 1, iters)
        assert max_err_over_eps(host(f), fo, eps) <= 1e-4 and max_err_over_eps(host(g), go, eps) <= 1e-4
        ref = oracle_value(p, q, wp, wq, host(f), host(g))
        assert abs(v - ref) <= 1e-5 * (abs(ref) + eps)
        total_gpu += coef * v
        total_ref += coef * oracle.objectives(p, q, wp, wq, eps, fo, go)[1]
    say("  divergence gpu=%.8f oracle=%.8f" % (total_gpu, total_ref))
    assert total_gpu > 0.0
    assert abs(total_gpu - total_ref) <= 2e-5 * (abs(total_ref) + eps)


@pytest.mark.parametrize("n,m,d,eps,iters", [(350, 290, 3, 0.2, 40), (180, 410, 24, 0.5, 15)])
def test_divergence_entry_point(ctx, oracle, n, m, d, eps, iters):
    """fs_divergence against the oracle's three solves and dual values; called twice, the second time on
    a smaller problem, so that the buffer kept between calls is exercised."""
    rng = np.random.default_rng(5 * n + d)
    eps = float(np.float32(eps))
    for (nn, mm) in ((n, m), (n // 2 + 1, m // 3 + 2)):
        x, y, a, b = _problem(rng, nn, mm, d, 1.0 if d <= 16 else 0.4)
        say("fs_divergence n=%d m=%d d=%d eps=%g iters=%d" % (nn, mm, d, eps, iters))
        ref_terms = []
        for (p, q, wp, wq) in ((x, y, a, b), (x, x, a, a), (y, y, b, b)):
            fo, go = oracle.solve(p, q, wp, wq, eps, eps, 1, iters)
            ref_terms.append(oracle.objectives(p, q, wp, wq, eps, fo, go)[1])
            if p is x and q is y:
                f_ref, g_ref = fo, go
        ref = ref_terms[0] - 0.5 * ref_terms[1] - 0.5 * ref_terms[2]
        value, terms, f, g = ctx.fs_divergence(make_problem(x, y, a, b), eps, iters)
        say("  gpu=%.8f oracle=%.8f terms gpu=%s" % (value, ref, ["%.6f" % t for t in terms]))
        assert max_err_over_eps(host(f), f_ref, eps) <= 1e-4 and max_err_over_eps(host(g), g_ref, eps) <= 1e-4
        for t, r in zip(terms, ref_terms):
            assert abs(t - r) <= 2e-5 * (abs(r) + eps)
        assert value == terms[0] - 0.5 * terms[1] - 0.5 * terms[2]
        assert value > 0.0
        assert abs(value - ref) <= 4e-5 * (max(abs(r) for r in ref_terms) + eps)
