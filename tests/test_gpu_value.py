"""GPU parity of fs_ot_value (dual objective of App. B at given potentials) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, make_problem, say

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
