"""GPU parity of fs_solve_labeled: alternating Sinkhorn for the label-augmented cost of the dataset-distance application
(Section 3.1's remark on generalised costs; the appendix on that application),
    C_ij = l1 |x_i - y_j|^2 + l2 W[lx_i, ly_j],   W a V x V table of class-to-class distances (synthetic here),
against dense log-domain Sinkhorn (oracle/dense_ref.py) on the EXPLICIT n x m cost matrix.  Everything the method does
with the labels happens inside the library; the test only builds the cost matrix for the reference.

fp32-accuracy mode: 1e-4 eps.  bf16 mode: 2e-2 eps against the cost of the inputs as given, and 2e-4 eps against the cost
of the values the matrix cores see (points and table entries rounded to bfloat16; with l2 / (2 l1) = 1/2, a power of
two, rounding the scaled table entries is rounding the entries)."""
import numpy as np
import pytest
import torch

from oracle import dense_ref
from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import dev, host, make_problem, max_err_over_eps, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return binding.Context(0)


def _dense_labeled(x, y, lx, ly, Wt, a, b, l1, l2, eps, iters, g0):
    C = l1 * dense_ref.cost(x, y) + l2 * Wt.astype(np.float64)[lx][:, ly]
    f, g = np.zeros(len(x)), np.asarray(g0, dtype=np.float64).copy()
    for _ in range(iters):
        f = dense_ref.update_f(C, b.astype(np.float64), eps, g)
        g = dense_ref.update_g(C, a.astype(np.float64), eps, f)
    return f, g


@pytest.mark.parametrize("n,m,d,V,mode,l1,l2", [
    (300, 260, 2, 3, "fp32", 0.5, 0.5),      # d + V <= 16: low-dimension kernels
    (300, 260, 6, 5, "fp32", 0.5, 0.5),
    (777, 1030, 3, 12, "fp32", 1.0, 0.25),
    (200, 330, 40, 10, "fp32", 0.5, 0.5),    # fp64 matrix cores
    (150, 90, 64, 20, "fp32", 0.25, 2.0),
    (256, 300, 64, 10, "bf16", 0.5, 0.5),    # bf16 matrix cores
    (600, 520, 100, 20, "bf16", 0.5, 0.5),
])
def test_labeled_cost_matches_dense_sinkhorn_on_the_explicit_cost(ctx, n, m, d, V, mode, l1, l2):
    rng = np.random.default_rng(n + d + V)
    scale = 1.0 if d <= 16 else 0.4
    x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    y = (rng.standard_normal((m, d)) * scale + 0.2).astype(np.float32)
    lx = rng.integers(0, V, n).astype(np.int32)
    ly = rng.integers(0, V, m).astype(np.int32)
    Wt = rng.random((V, V)) * (2.0 if d <= 16 else 4.0)        # not symmetric: a transposed lookup would show
    Wt = Wt.astype(np.float32)
    a = rng.random(n) + 0.5
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.5
    b = (b / b.sum()).astype(np.float32)
    eps = float(np.float32(0.25 if d <= 16 else 1.0))
    iters = 15
    g0 = (0.1 * rng.standard_normal(m)).astype(np.float32)    # a warm start: the given g is read, the given f is not
    bf = mode == "bf16"
    prob = make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA if bf else binding.FS_COMPUTE_FP32)
    say("labelled cost n=%d m=%d d=%d V=%d %s mode l1=%g l2=%g" % (n, m, d, V, mode, l1, l2))
    f = torch.full((n,), 3.0, device="cuda:0")
    g = dev(g0)
    ctx.fs_solve_labeled(prob, dev(lx, torch.int32), dev(ly, torch.int32), dev(Wt), l1, l2, eps, iters, f, g)
    f_ref, g_ref = _dense_labeled(x, y, lx, ly, Wt, a, b, l1, l2, eps, iters, g0)
    ef, eg = max_err_over_eps(host(f), f_ref, eps), max_err_over_eps(host(g), g_ref, eps)
    say("  against the cost of the inputs as given: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    if not bf:
        assert ef <= 1e-4 and eg <= 1e-4
        return
    assert ef <= 2e-2 and eg <= 2e-2
    xr, yr, Wr = workloads.to_bf16_round(x), workloads.to_bf16_round(y), workloads.to_bf16_round(Wt)
    f_ref, g_ref = _dense_labeled(xr, yr, lx, ly, Wr, a, b, l1, l2, eps, iters, g0)
    ef, eg = max_err_over_eps(host(f), f_ref, eps), max_err_over_eps(host(g), g_ref, eps)
    say("  against the cost of the rounded values: max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= 2e-4 and eg <= 2e-4


def test_labeled_cost_with_a_zero_table_is_the_plain_solve(ctx, oracle):
    """W = 0: the labelled solve must equal the oracle's plain solve at cost l1 |x - y|^2, i.e. the squared-Euclidean
    trajectory at eps / l1 with potentials scaled by l1."""
    rng = np.random.default_rng(3)
    n, m, d, V, l1 = 400, 350, 3, 4, 0.5
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) + 0.3).astype(np.float32)
    a = np.full(n, 1.0 / n, dtype=np.float32)
    b = np.full(m, 1.0 / m, dtype=np.float32)
    eps = float(np.float32(0.2))
    say("labelled cost with W = 0, n=%d m=%d" % (n, m))
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    ctx.fs_solve_labeled(make_problem(x, y, a, b), dev(rng.integers(0, V, n), torch.int32), dev(rng.integers(0, V, m), torch.int32),
                         torch.zeros(V, V, device="cuda:0"), l1, 0.7, eps, 10, f, g)
    fo, go = oracle.solve(x, y, a, b, eps / l1, eps / l1, 1, 10)
    assert max_err_over_eps(host(f), l1 * fo, eps) <= 1e-4
    assert max_err_over_eps(host(g), l1 * go, eps) <= 1e-4


def test_labeled_cost_reports_labels_out_of_range(ctx):
    rng = np.random.default_rng(5)
    n, m, d, V = 64, 50, 3, 4
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = rng.standard_normal((m, d)).astype(np.float32)
    lx = rng.integers(0, V, n).astype(np.int32)
    ly = rng.integers(0, V, m).astype(np.int32)
    ly[7] = V          # one past the table
    lx[3] = -1
    say("labelled cost with two labels out of range")
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    with pytest.raises(binding.FlashSinkError) as ei:
        ctx.fs_solve_labeled(make_problem(x, y, None, None), dev(lx, torch.int32), dev(ly, torch.int32),
                             torch.ones(V, V, device="cuda:0"), 0.5, 0.5, 0.3, 2, f, g)
    assert ei.value.status == 1 and "2 labels" in str(ei.value)
