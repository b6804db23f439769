"""GPU parity of fs_apply_plan_hadamard (Alg. 5: Hadamard-weighted transport (P o (A y^T)) V) against the dense
float64 oracle (oracle/hvp_dense.hadamard_transport, pinned by its entry-by-entry definition), element by
element, on all three code paths it can take: d <= 3 (vector-ALU kernel), d in 4..16 (fp64 matrix cores on
centred records, or the vector-ALU kernel on fp32 scores) and d > 16 (fp64 matrix cores).

The bar is the one of the plain plan application in fp32-accuracy mode: 2e-4 relative (Frobenius) and
1e-3 of the largest entry, entry by entry.  The weights <A_i, y_j> change sign, so entries of the result can be small
next to the terms they sum; the element-wise bar is therefore relative to the largest entry of the result."""
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


def _problem(rng, n, m, d, shift):
    x = rng.standard_normal((n, d)).astype(np.float32)
    y = (rng.standard_normal((m, d)) * 0.8 + shift).astype(np.float32)
    a = rng.random(n) + 0.5
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.5
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


# sizes span several tiles of every kernel with ragged tails; the shift moves the common mean away from the origin
# (the low-d kernels centre the clouds and the mean's share of the weights is added separately)
@pytest.mark.parametrize("n,m,d,p,eps,iters,shift", [
    (300, 260, 1, 2, 0.4, 20, 0.3), (1100, 777, 2, 5, 0.5, 10, 2.0), (513, 1300, 3, 3, 0.3, 15, -1.5),
    (260, 300, 4, 4, 0.5, 20, 0.3), (700, 500, 8, 9, 1.0, 10, 1.0), (333, 410, 16, 16, 2.0, 10, 0.5),
    (200, 170, 20, 20, 2.0, 10, 0.3), (150, 260, 64, 7, 6.0, 10, 0.2), (70, 90, 100, 70, 10.0, 5, 0.1),
])
def test_hadamard_transport_matches_dense_oracle(ctx, oracle, n, m, d, p, eps, iters, shift):
    from oracle import hvp_dense
    rng = np.random.default_rng(11 * n + m + d)
    x, y, a, b = _problem(rng, n, m, d, shift)
    eps = float(np.float32(eps))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, iters)     # not converged: any potentials are allowed
    f32, g32 = fo.astype(np.float32), go.astype(np.float32)
    A = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    say("hadamard transport n=%d m=%d d=%d p=%d eps=%g shift=%g" % (n, m, d, p, eps, shift))
    got = host(ctx.fs_apply_plan_hadamard(make_problem(x, y, a, b), eps, dev(f32), dev(g32), dev(A), dev(V)))
    want = hvp_dense.hadamard_transport(x, y, a, b, eps, f32.astype(np.float64), g32.astype(np.float64), A, V)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    mx = np.abs(got - want).max() / np.abs(want).max()
    say("  rel. Frobenius %.3e, max abs / max |ref| %.3e" % (rel, mx))
    assert rel <= 2e-4
    assert mx <= 1e-3


def test_hadamard_transport_with_the_clouds_own_points_and_row_strides(ctx, oracle):
    """V = y read in place from a wider array, A and out with row strides of their own: the form Thm. 5 uses."""
    from oracle import hvp_dense
    rng = np.random.default_rng(5)
    n, m, d = 400, 333, 3
    x, y, a, b = _problem(rng, n, m, d, 0.7)
    eps = float(np.float32(0.5))
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 30)
    f32, g32 = fo.astype(np.float32), go.astype(np.float32)
    Abig = rng.standard_normal((n, d + 2)).astype(np.float32)
    prob = make_problem(x, y, a, b)
    A_dev = dev(Abig)[:, :d]                       # row stride d + 2
    say("hadamard transport, V = y in place, strided A, n=%d m=%d d=%d" % (n, m, d))
    lib = ctx.lib
    out = torch.full((n, d + 3), 7.0, dtype=torch.float32, device="cuda:0")
    import ctypes
    f_dev, g_dev = dev(f32), dev(g32)
    st = lib.fs_apply_plan_hadamard(ctx.h, ctypes.byref(prob.c), eps, ctypes.c_void_p(f_dev.data_ptr()),
                                    ctypes.c_void_p(g_dev.data_ptr()), ctypes.c_void_p(A_dev.data_ptr()), d + 2,
                                    ctypes.c_void_p(prob.y.data_ptr()), d, prob.y.stride(0),
                                    ctypes.c_void_p(out.data_ptr()), d + 3)
    assert st == 0
    torch.cuda.synchronize()
    got = host(out)
    want = hvp_dense.hadamard_transport(x, y, a, b, eps, f32.astype(np.float64), g32.astype(np.float64), Abig[:, :d])
    assert np.abs(got[:, :d] - want).max() <= 1e-3 * np.abs(want).max()
    assert np.linalg.norm(got[:, :d] - want) <= 2e-4 * np.linalg.norm(want)
    assert np.all(got[:, d:] == 7.0)               # nothing written beyond the p columns of a row


def test_hadamard_transport_refuses_what_it_does_not_cover(ctx):
    rng = np.random.default_rng(1)
    x, y, a, b = _problem(rng, 40, 30, 32, 0.0)
    f = torch.zeros(40, device="cuda:0")
    g = torch.zeros(30, device="cuda:0")
    A = torch.zeros(40, 32, device="cuda:0")
    V = torch.zeros(30, 4, device="cuda:0")
    say("hadamard transport in bf16 mode is refused")
    with pytest.raises(binding.FlashSinkError):
        ctx.fs_apply_plan_hadamard(make_problem(x, y, a, b, compute=binding.FS_COMPUTE_BF16_MFMA), 0.5, f, g, A, V)
