"""fs_solve_noalloc (the entry point for callers that cannot allocate device memory) against fs_solve and
the float64 oracle, through the C ABI: two calls in a row on one context, the second on a smaller problem, so
that the second runs in a static scratch array that still holds the first call's data."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_03067_amd import binding, workloads
from tests._gpu_common import host, max_err_over_eps, say

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _solve(lib, h, name, prob, w, f, g):
    fn = getattr(lib, name)
    st = fn(h, ctypes.byref(prob.c), ctypes.c_float(w.eps_start), ctypes.c_float(w.eps_end), w.n_stages, w.iters,
            ctypes.c_void_p(f.data_ptr()), ctypes.c_void_p(g.data_ptr()))
    assert st == 0, (name, st, lib.fs_last_error(h))
    torch.cuda.synchronize()


def test_noalloc_solve_matches_solve_twice_in_a_row(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ctx = binding.Context(0)
    lib, h = ctx.lib, ctx.h
    # annealed low-dimension problem (several stages, both score arithmetics), then a smaller fixed-eps one
    cases = [workloads.make("lowdim_anneal", n=3000, m=2600, iters=3), workloads.make("tiny", n=700, m=900, iters=12)]
    for k, w in enumerate(cases):
        prob = binding.problem_from_workload(w)
        f0, g0 = torch.zeros(w.n, device="cuda:0"), torch.zeros(w.m, device="cuda:0")
        f1, g1 = torch.zeros(w.n, device="cuda:0"), torch.zeros(w.m, device="cuda:0")
        say("fs_solve_noalloc call %d: %s n=%d m=%d d=%d stages=%d iters=%d" % (k + 1, w.name, w.n, w.m, w.d, w.n_stages, w.iters))
        _solve(lib, h, "fs_solve_noalloc", prob, w, f1, g1)
        _solve(lib, h, "fs_solve", prob, w, f0, g0)
        eps = float(np.float32(w.eps_end))
        ef = max_err_over_eps(host(f1), host(f0), eps)
        eg = max_err_over_eps(host(g1), host(g0), eps)
        fo, go = oracle.solve(w.x, w.y, w.a, w.b, w.eps_start, w.eps_end, w.n_stages, w.iters)
        of = max_err_over_eps(host(f1), fo, eps)
        og = max_err_over_eps(host(g1), go, eps)
        say("  against fs_solve: max|df|/eps=%.3e max|dg|/eps=%.3e; against the oracle: %.3e %.3e" % (ef, eg, of, og))
        assert ef <= TOL and eg <= TOL
        assert of <= TOL and og <= TOL
    ctx.close()


def test_noalloc_solve_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ctx = binding.Context(0)
    n = 70000                      # beyond the static scratch at d = 3
    x = torch.rand(n, 3, device="cuda:0")
    f, g = torch.zeros(n, device="cuda:0"), torch.zeros(n, device="cuda:0")
    prob = binding.Problem(x, x.clone())
    say("fs_solve_noalloc refuses n=m=%d, d=3" % n)
    with pytest.raises(binding.FlashSinkError) as ei:
        ctx.fs_solve_noalloc(prob, 0.1, 0.1, 1, 1, f, g)
    assert ei.value.status == 2 and "fs_solve_noalloc" in str(ei.value)
    assert float(f.abs().max()) == 0.0 and float(g.abs().max()) == 0.0     # nothing was launched
    ctx.close()
