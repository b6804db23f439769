"""Label-augmented cost (the dataset-distance application in the paper's appendix on OTDD):
    C_ij = l1 |x_i - y_j|^2 + l2 W[lx_i, ly_j],   W a V x V table of class-to-class distances.
No kernel needs to know about labels: the lookup is a contraction, W[lx, ly] = <onehot(lx), W[:, ly]>,
so with the augmented points  xa_i = [x_i, onehot(lx_i)],  ya_j = [y_j, -(l2 / 2 l1) W[:, ly_j]]
    l1 |xa_i - ya_j|^2 = C_ij + l1 (1 + |(l2 / 2 l1) W[:, ly_j]|^2) =: C_ij + l1 + v_j,
a cost that differs from C by per-point constants only, which the potentials absorb exactly:
started from g = v, every Sinkhorn iterate on the augmented clouds is (f + l1, g + v).
The test runs fs_solve on the augmented clouds (eps / l1, potentials scaled by 1 / l1) and compares
with dense log-domain Sinkhorn on the explicit label-augmented cost matrix."""
import numpy as np
import pytest
import torch

from oracle import dense_ref
from paper_2602_03067_amd import binding
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return binding.Context(0)


@pytest.mark.parametrize("n,m,d,V,mode", [(300, 260, 6, 5, "fp32"), (200, 330, 40, 10, "fp32"), (256, 300, 64, 10, "bf16")])
def test_label_augmented_cost_through_augmented_points(ctx, n, m, d, V, mode):
    rng = np.random.default_rng(n + d + V)
    scale = 1.0 if d <= 16 else 0.4
    x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    y = (rng.standard_normal((m, d)) * scale + 0.2).astype(np.float32)
    lx = rng.integers(0, V, n)
    ly = rng.integers(0, V, m)
    Wt = rng.random((V, V))
    Wt = (0.5 * (Wt + Wt.T) * (2.0 if d <= 16 else 4.0)).astype(np.float32)   # symmetric class distances
    a = np.full(n, 1.0 / n, dtype=np.float32)
    b = np.full(m, 1.0 / m, dtype=np.float32)
    l1 = l2 = 0.5
    eps = float(np.float32(0.25 if d <= 16 else 1.0))
    iters = 15
    # augmented clouds (all values float32; in bf16 mode the oracle gets the bf16-rounded ones)
    xa = np.concatenate([x, np.eye(V, dtype=np.float32)[lx]], axis=1)
    ya = np.concatenate([y, (-(l2 / (2.0 * l1)) * Wt[:, ly].T).astype(np.float32)], axis=1)
    if mode == "bf16":
        from paper_2602_03067_amd import workloads
        xo, yo = workloads.to_bf16_round(xa), workloads.to_bf16_round(ya)
        prob = make_problem(xa, ya, a, b, compute=binding.FS_COMPUTE_BF16_MFMA)
        tol = 2e-4
    else:
        xo, yo = xa, ya
        prob = make_problem(xa, ya, a, b)
        tol = 1e-4
    # dense reference on the explicit label-augmented cost of the (possibly rounded) data
    xd, yd = xo[:, :d].astype(np.float64), yo[:, :d].astype(np.float64)
    Wd = -(2.0 * l1 / l2) * yo[:, d:].astype(np.float64).T          # the table as the kernels see it: [V][m]
    C = l1 * dense_ref.cost(xd, yd) + l2 * Wd[lx, :]
    f_ref, g_ref = np.zeros(n), np.zeros(m)
    for _ in range(iters):
        f_ref = dense_ref.update_f(C, b.astype(np.float64), eps, g_ref)
        g_ref = dense_ref.update_g(C, a.astype(np.float64), eps, f_ref)
    # GPU: cost |xa - ya|^2 = (C + l1 + v) / l1 at eps / l1; start from g = v / l1
    v = l1 * (yo[:, d:].astype(np.float64) ** 2).sum(1)
    say("label-augmented cost n=%d m=%d d=%d V=%d %s mode" % (n, m, d, V, mode))
    f = torch.zeros(n, device="cuda:0")
    g = dev((v / l1).astype(np.float32))
    ctx.fs_solve(prob, eps / l1, eps / l1, 1, iters, f, g)
    f_gpu = host(f) * l1 - l1
    g_gpu = host(g) * l1 - v
    ef, eg = max_err_over_eps(f_gpu, f_ref, eps), max_err_over_eps(g_gpu, g_ref, eps)
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= tol and eg <= tol
