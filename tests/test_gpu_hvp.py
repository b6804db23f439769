"""GPU parity of fs_hvp (Thm. 5: streaming Hessian-vector product) against the dense float64
oracle (oracle/hvp_dense.py, pinned by central differences of the gradient).

The GPU works with float32 vectors inside conjugate gradients; the bar is a relative Frobenius
error of 1e-4 against the oracle at the SAME damping tau (measured: 2e-6 .. 5e-6), and entry by entry
1e-3 of the largest entry.  Against the
undamped pseudo-inverse the damping itself shows: the paper's parity protocol (n = m = 512, d = 4,
tau = 1e-5, eta = 1e-6) reports 4.6e-3 there, this implementation 3.0e-3 on its own random data."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding
from tests._gpu_common import dev, host, make_problem, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return binding.Context(0)


def _problem(rng, n, m, d):
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) * 0.8 + 0.3).astype(np.float32)
    a = rng.random(n) + 0.5
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.5
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


@pytest.mark.parametrize("n,m,d,eps,iters", [(60, 45, 2, 0.5, 200), (300, 260, 3, 0.4, 60), (512, 512, 4, 0.5, 100),
                                             (130, 700, 8, 1.0, 30),
                                             (200, 170, 20, 2.0, 40), (150, 260, 64, 6.0, 30), (70, 90, 100, 10.0, 20)])
def test_hvp_matches_dense_oracle(ctx, oracle, n, m, d, eps, iters):
    from oracle import hvp_dense
    rng = np.random.default_rng(7 * n + m + d)
    x, y, a, b = _problem(rng, n, m, d)
    eps = float(np.float32(eps))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, iters)
    f32, g32 = fo.astype(np.float32), go.astype(np.float32)
    A = rng.standard_normal((n, d)).astype(np.float32)
    tau, eta = 1e-5, 1e-6
    say("hvp n=%d m=%d d=%d eps=%g (potentials after %d iterations), tau=%g eta=%g" % (n, m, d, eps, iters, tau, eta))
    G, k = ctx.fs_hvp(make_problem(x, y, a, b), eps, dev(f32), dev(g32), dev(A), tau, eta, 400)
    want = hvp_dense.hvp(x, y, a, b, eps, f32.astype(np.float64), g32.astype(np.float64), A, tau=tau)
    rel = np.linalg.norm(host(G) - want) / np.linalg.norm(want)
    mx = np.abs(host(G) - want).max() / np.abs(want).max()
    undamped = hvp_dense.hvp(x, y, a, b, eps, f32.astype(np.float64), g32.astype(np.float64), A)
    rel0 = np.linalg.norm(host(G) - undamped) / np.linalg.norm(undamped)
    say("  CG iterations %d, rel. error vs oracle at the same tau %.3e (largest entry error / largest entry %.3e), "
        "vs the pseudo-inverse %.3e" % (k, rel, mx, rel0))
    assert rel <= 1e-4
    assert mx <= 1e-3      # entry by entry, against the largest entry (entries of T A change sign)
    assert rel0 <= 2e-2


def test_hvp_is_linear_in_the_direction(ctx, oracle):
    """T(A1 + A2) = T A1 + T A2 on the GPU (every term of the decomposition, the Hadamard-weighted
    transport included, is linear in A; CG only up to its stopping rule)."""
    rng = np.random.default_rng(3)
    n, m, d = 200, 150, 3
    x, y, a, b = _problem(rng, n, m, d)
    eps = float(np.float32(0.5))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 80)
    f, g = dev(fo.astype(np.float32)), dev(go.astype(np.float32))
    A1 = rng.standard_normal((n, d)).astype(np.float32)
    A2 = rng.standard_normal((n, d)).astype(np.float32)
    prob = make_problem(x, y, a, b)
    say("hvp linearity n=%d m=%d d=%d" % (n, m, d))
    G1, _ = ctx.fs_hvp(prob, eps, f, g, dev(A1), 1e-5, 1e-7, 400)
    G2, _ = ctx.fs_hvp(prob, eps, f, g, dev(A2), 1e-5, 1e-7, 400)
    G12, _ = ctx.fs_hvp(prob, eps, f, g, dev(A1 + A2), 1e-5, 1e-7, 400)
    err = np.linalg.norm(host(G12) - host(G1) - host(G2)) / np.linalg.norm(host(G12))
    say("  |T(A1+A2) - T A1 - T A2| / |T(A1+A2)| = %.3e" % err)
    assert err <= 1e-4


def test_hvp_refuses_what_it_does_not_cover(ctx):
    rng = np.random.default_rng(1)
    x, y, a, b = _problem(rng, 40, 30, 32)
    f = torch.zeros(40, device="cuda:0")
    g = torch.zeros(30, device="cuda:0")
    A = torch.zeros(40, 32, device="cuda:0")
    say("hvp in bf16 mode is refused")
    with pytest.raises(binding.FlashSinkError):
        ctx.fs_hvp(make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA), 0.5, f, g, A, 1e-5, 1e-6, 10)
