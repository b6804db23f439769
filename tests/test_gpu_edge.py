"""GPU edge cases of the C ABI against the float64 oracle: row strides larger than the row,
a context on a stream of its own, one context reused over problems of different sizes and paths
(workspace regrowth), very small eps in low dimension, derived copies kept across calls."""
import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding
from tests._gpu_common import dev, host, max_err_over_eps, say

pytestmark = pytest.mark.gpu
BF = binding.FS_COMPUTE_BF16_MFMA


def _cloud(rng, n, m, d, scale):
    x = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    y = (rng.standard_normal((m, d)) * scale + 0.3 * scale).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = rng.random(m) + 0.1
    b = (b / b.sum()).astype(np.float32)
    return x, y, a, b


def _strided(arr, extra):
    """Device tensor whose rows are `extra` elements apart more than their length (junk in between)."""
    rows, cols = arr.shape
    buf = torch.full((rows, cols + extra), 1.0e30, dtype=torch.float32, device="cuda:0")
    view = buf[:, :cols]
    view.copy_(torch.from_numpy(arr))
    assert view.stride(0) == cols + extra
    return view


@pytest.mark.parametrize("d,compute,tol", [(3, "fp32", 1e-4), (9, "fp32", 1e-4), (40, "fp32", 1e-4), (48, "bf16", 2e-2)])
def test_row_strides_larger_than_the_rows(oracle, d, compute, tol):
    rng = np.random.default_rng(100 + d)
    n, m, p = 333, 290, 5
    x, y, a, b = _cloud(rng, n, m, d, 1.0 / np.sqrt(d))
    eps = float(np.float32(0.3))
    g0 = (0.2 * rng.standard_normal(m)).astype(np.float32)
    V = rng.standard_normal((m, p)).astype(np.float32)
    say("strided inputs d=%d %s" % (d, compute))
    ctx = binding.Context(0)
    prob = binding.Problem(_strided(x, 3), _strided(y, 7), dev(a), dev(b), BF if compute == "bf16" else binding.FS_COMPUTE_FP32)
    f1 = ctx.fs_update_f(prob, eps, dev(g0))
    g1 = ctx.fs_update_g(prob, eps, f1)
    f1h = host(f1)
    ef = max_err_over_eps(f1h, oracle.update_f(x, y, b, eps, g0), eps)
    eg = max_err_over_eps(host(g1), oracle.update_g(x, y, a, eps, f1h.astype(np.float32)), eps)
    out = host(ctx.fs_apply_plan(prob, eps, f1, g1, _strided(V, 2)))
    want = oracle.apply_plan(x, y, a, b, eps, f1h.astype(np.float32), host(g1).astype(np.float32), V)
    ea = np.linalg.norm(out - want) / np.linalg.norm(want)
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e apply rel=%.3e" % (ef, eg, ea))
    assert ef <= tol and eg <= tol and ea <= max(tol, 2e-4)
    ctx.close()


def test_context_on_its_own_stream(oracle):
    rng = np.random.default_rng(7)
    n, m, d = 500, 400, 3
    x, y, a, b = _cloud(rng, n, m, d, 1.0)
    eps = float(np.float32(0.2))
    say("context bound to a non-default stream")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = binding.Context(0, stream)
        prob = binding.Problem(dev(x), dev(y), dev(a), dev(b))
        f = torch.zeros(n, device="cuda:0")
        g = torch.zeros(m, device="cuda:0")
        ctx.fs_solve(prob, eps, eps, 1, 7, f, g)
    stream.synchronize()
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 7)
    assert max_err_over_eps(host(f), fo, eps) <= 1e-4 and max_err_over_eps(host(g), go, eps) <= 1e-4
    ctx.close()


def test_one_context_many_problems(oracle):
    """The workspace grows and is laid out anew per call: small, large, another path, small again."""
    rng = np.random.default_rng(11)
    ctx = binding.Context(0)
    for (n, m, d, compute, tol) in ((50, 60, 3, "fp32", 1e-4), (3000, 2500, 3, "fp32", 1e-4), (300, 200, 64, "fp32", 1e-4),
                                    (600, 700, 64, "bf16", 2e-2), (40, 30, 2, "fp32", 1e-4), (900, 1000, 16, "fp32", 1e-4)):
        x, y, a, b = _cloud(rng, n, m, d, 1.0 / np.sqrt(d))
        eps = float(np.float32(0.25))
        say("same context: n=%d m=%d d=%d %s" % (n, m, d, compute))
        prob = binding.Problem(dev(x), dev(y), dev(a), dev(b), BF if compute == "bf16" else binding.FS_COMPUTE_FP32)
        f = torch.zeros(n, device="cuda:0")
        g = torch.zeros(m, device="cuda:0")
        ctx.fs_solve(prob, eps, eps, 1, 4, f, g)
        fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 4)
        ef, eg = max_err_over_eps(host(f), fo, eps), max_err_over_eps(host(g), go, eps)
        say("  max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
        assert ef <= tol and eg <= tol
    ctx.close()


@pytest.mark.parametrize("d,eps", [(3, 2e-3), (2, 5e-4), (8, 2e-3)])
def test_very_small_eps_low_dimension(oracle, d, eps):
    """Scores of several thousand (base 2): float64-score half-steps, on the matrix cores where the
    fixed grids cover the biases (d <= 3) and on the fp64 matrix cores at larger d."""
    rng = np.random.default_rng(31 + d)
    n, m = 700, 650
    x = rng.random((n, d)).astype(np.float32)
    y = rng.random((m, d)).astype(np.float32)
    a = np.full(n, 1.0 / n, dtype=np.float32)
    b = np.full(m, 1.0 / m, dtype=np.float32)
    eps = float(np.float32(eps))
    say("very small eps: d=%d eps=%g" % (d, eps))
    ctx = binding.Context(0)
    prob = binding.Problem(dev(x), dev(y), dev(a), dev(b))
    f = torch.zeros(n, device="cuda:0")
    g = torch.zeros(m, device="cuda:0")
    ctx.fs_solve(prob, eps, eps, 1, 5, f, g)
    fo, go = oracle.solve(x, y, a, b, eps, eps, 1, 5)
    ef, eg = max_err_over_eps(host(f), fo, eps), max_err_over_eps(host(g), go, eps)
    say("  max|df|/eps=%.3e max|dg|/eps=%.3e" % (ef, eg))
    assert ef <= 1e-4 and eg <= 1e-4
    ctx.close()


def test_check_weights(oracle):
    """fs_check_weights: sums in float64 of the float weights, FS_ERR_BAD_WEIGHTS for a weight that is not
    positive, and for a sum off by more than the tolerance."""
    rng = np.random.default_rng(3)
    n, m, d = 5000, 777, 3
    x = rng.random((n, d)).astype(np.float32)
    y = rng.random((m, d)).astype(np.float32)
    a = rng.random(n) + 0.1
    a = (a / a.sum()).astype(np.float32)
    b = np.full(m, 1.0 / m, dtype=np.float32)
    say("check_weights n=%d m=%d" % (n, m))
    ctx = binding.Context(0)
    sa, sb = ctx.fs_check_weights(binding.Problem(dev(x), dev(y), dev(a), dev(b)), 1e-5)
    assert abs(sa - a.astype(np.float64).sum()) <= 1e-12 and abs(sb - b.astype(np.float64).sum()) <= 1e-12
    assert ctx.fs_check_weights(binding.Problem(dev(x), dev(y), None, dev(b)), 1e-5)[0] == 1.0
    bad = a.copy()
    bad[1234] = 0.0
    with pytest.raises(binding.FlashSinkError) as e:
        ctx.fs_check_weights(binding.Problem(dev(x), dev(y), dev(bad), dev(b)), 1e-5)
    assert e.value.status == 4
    with pytest.raises(binding.FlashSinkError) as e:
        ctx.fs_check_weights(binding.Problem(dev(x), dev(y), dev(a), dev((b * 1.01).astype(np.float32))), 1e-5)
    assert e.value.status == 4
    bad[1234] = np.nan
    with pytest.raises(binding.FlashSinkError):
        ctx.fs_check_weights(binding.Problem(dev(x), dev(y), dev(bad), None), 1e-5)
    ctx.close()


def test_check_finite():
    ctx = binding.Context(0)
    v = torch.randn(100001, device="cuda:0")
    say("check_finite on %d values" % v.numel())
    assert ctx.fs_check_finite(v) == 0
    v[77] = float("nan")
    v[99999] = float("-inf")
    with pytest.raises(binding.FlashSinkError) as e:
        ctx.fs_check_finite(v)
    assert e.value.status == 8 and "2 of 100001" in str(e.value)
    ctx.close()


@pytest.mark.parametrize("d,compute", [(3, "fp32"), (2, "fp32"), (9, "fp32"), (40, "fp32"), (48, "bf16")])
def test_kept_derived_copies_change_nothing(oracle, d, compute):
    """fs_points_keep: a sequence of entry calls on one pair of clouds gives bit-identical results with and without the
    declaration (the copies are the same bytes either way); a call on other clouds in between overwrites the kept copies
    and the next call prepares them again; after fs_points_release new coordinates at the same addresses are seen."""
    rng = np.random.default_rng(500 + d)
    n, m = 700, 900
    x, y, a, b = _cloud(rng, n, m, d, 0.4)
    if compute == "bf16":   # coordinates the matrix cores see exactly (and so are their doubles further down)
        x = torch.from_numpy(x).bfloat16().float().numpy()
        y = torch.from_numpy(y).bfloat16().float().numpy()
    eps = float(np.float32(0.25))
    cm = BF if compute == "bf16" else binding.FS_COMPUTE_FP32
    xd, yd = dev(x), dev(y)
    prob = binding.Problem(xd, yd, dev(a), dev(b), cm)
    other = binding.Problem(dev(x[:300] * 2.0), dev(y[:500] * 0.5), None, None, cm)
    V = dev(rng.standard_normal((m, 5)).astype(np.float32))
    say("kept derived copies d=%d %s" % (d, compute))

    def sequence(ctx, interleave):
        f = torch.zeros(n, device="cuda:0")
        g = torch.zeros(m, device="cuda:0")
        ctx.fs_solve(prob, 2 * eps, eps, 3, 4, f, g)
        if interleave:   # another problem through the same workspace
            fo = torch.zeros(300, device="cuda:0")
            go = torch.zeros(500, device="cuda:0")
            ctx.fs_solve(other, eps, eps, 1, 2, fo, go)
        er, ec = ctx.fs_marginal_err(prob, eps, f, g)
        grad = ctx.fs_grad_x(prob, eps, f, g, 0)
        out = ctx.fs_apply_plan(prob, eps, f, g, V)
        f2 = ctx.fs_update_f(prob, eps, g)
        return [host(f), host(g), np.array([er, ec]), host(grad), host(out), host(f2)]

    ctx = binding.Context(0)
    plain = sequence(ctx, False)
    ctx.fs_points_keep(prob)
    kept = sequence(ctx, False)
    kept_again = sequence(ctx, True)
    for u, v, w in zip(plain, kept, kept_again):
        assert np.array_equal(u, v) and np.array_equal(u, w)
    # parity of the kept run against the oracle
    fo, go = oracle.solve(x, y, a, b, 2 * eps, eps, 3, 4)
    assert max_err_over_eps(kept[0], fo, eps) <= (2e-2 if compute == "bf16" else 1e-4)
    # the points change at the same addresses: with the declaration standing the OLD copies answer; after the
    # release the new coordinates do
    g_fix = dev(kept[1])
    xd.mul_(2.0)
    stale = host(ctx.fs_update_f(prob, eps, g_fix))
    assert np.array_equal(stale, plain[5])
    ctx.fs_points_release()
    fresh = host(ctx.fs_update_f(prob, eps, g_fix))
    want = oracle.update_f(host(xd), y, b, eps, kept[1])
    assert max_err_over_eps(fresh, want, eps) <= (2e-2 if compute == "bf16" else 1e-4)
    assert not np.array_equal(fresh, stale)
