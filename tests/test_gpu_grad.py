"""GPU parity of the in-library gradient assembly (Cor. 4 and its induced-marginal and
barycentric-displacement variants) against the float64 oracle: plan application by the oracle,
assembly written out here."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, say

pytestmark = pytest.mark.gpu
BF = binding.FS_COMPUTE_BF16_MFMA


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def _problem(rng, n, m, d):
    x = (rng.standard_normal((n, d)) / np.sqrt(d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) / np.sqrt(d) + 0.3 / np.sqrt(d)).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.1
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


def _reference(oracle, xs, ys, x, y, a, b, eps, f, g):
    """mode -> (grad wrt x, grad wrt y) from the oracle's plan applications.  The plan is that of
    (xs, ys) (the points as the chosen arithmetic sees them); values and assembly use (x, y)."""
    PY, r = oracle.apply_plan(xs, ys, a, b, eps, f, g, y.astype(np.float64), return_mass=True)
    PtX, c = oracle.apply_plan_T(xs, ys, a, b, eps, f, g, x.astype(np.float64), return_mass=True)
    xd, yd, ad, bd = (v.astype(np.float64) for v in (x, y, a, b))
    return {0: (2 * (ad[:, None] * xd - PY), 2 * (bd[:, None] * yd - PtX)),
            1: (2 * (r[:, None] * xd - PY), 2 * (c[:, None] * yd - PtX)),
            2: (xd - PY / ad[:, None], yd - PtX / bd[:, None])}


@pytest.mark.parametrize("n,m,d,mode_name", [(300, 421, 3, "fp32"), (130, 700, 8, "fp32"), (257, 190, 40, "fp32"),
                                             (200, 333, 64, "fp32"), (210, 260, 200, "fp32"), (300, 500, 64, "bf16"), (260, 1100, 100, "bf16")])
def test_gradients_all_modes(ctx, oracle, n, m, d, mode_name):
    rng = np.random.default_rng(17 * n + m + d)
    x, y, a, b = _problem(rng, n, m, d)
    eps = float(np.float32(0.5 if d > 3 else 0.2))
    bf = mode_name == "bf16"
    xs, ys = (workloads.to_bf16_round(x), workloads.to_bf16_round(y)) if bf else (x, y)
    fo, go = oracle.solve(xs, ys, a, b, eps, eps, 1, 4)
    f32 = (fo + 0.02 * rng.standard_normal(n)).astype(np.float32)
    g32 = go.astype(np.float32)
    say("gradients n=%d m=%d d=%d %s" % (n, m, d, mode_name))
    prob = make_problem(x, y, a, b, compute=BF) if bf else make_problem(x, y, a, b)
    # bf16 mode: the plan is that of the rounded points, values and assembly use the points as given
    ref = _reference(oracle, xs, ys, x, y, a, b, eps, f32, g32)
    tol = 2e-2 if bf else 2e-4
    for mode in (0, 1, 2):
        gx = host(ctx.fs_grad_x(prob, eps, dev(f32), dev(g32), mode))
        gy = host(ctx.fs_grad_y(prob, eps, dev(f32), dev(g32), mode))
        ex = np.linalg.norm(gx - ref[mode][0]) / np.linalg.norm(ref[mode][0])
        ey = np.linalg.norm(gy - ref[mode][1]) / np.linalg.norm(ref[mode][1])
        say("  mode %d: grad_x %.3e  grad_y %.3e" % (mode, ex, ey))
        assert ex <= tol and ey <= tol


def test_gradient_bf16_storage(ctx, oracle):
    """Points stored as bfloat16: the other cloud is widened in the workspace before it is applied."""
    w = workloads.make("embedding", n=600, m=450, d=128)
    eps = float(np.float32(0.05))
    fo, go = oracle.solve(w.x, w.y, w.a, w.b, eps, eps, 1, 5)
    f32, g32 = fo.astype(np.float32), go.astype(np.float32)
    say("gradients bf16 storage n=%d m=%d d=%d" % (w.n, w.m, w.d))
    prob = binding.problem_from_workload(w)
    ref = _reference(oracle, w.x, w.y, w.x, w.y, w.a, w.b, eps, f32, g32)
    for mode in (0, 2):
        gx = host(ctx.fs_grad_x(prob, eps, dev(f32), dev(g32), mode))
        gy = host(ctx.fs_grad_y(prob, eps, dev(f32), dev(g32), mode))
        ex = np.linalg.norm(gx - ref[mode][0]) / np.linalg.norm(ref[mode][0])
        ey = np.linalg.norm(gy - ref[mode][1]) / np.linalg.norm(ref[mode][1])
        say("  mode %d: grad_x %.3e  grad_y %.3e" % (mode, ex, ey))
        assert ex <= 2e-2 and ey <= 2e-2
