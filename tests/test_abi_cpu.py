"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and validates arguments on the host (through a host-only context)."""
import ctypes
import os
import re

import pytest

from paper_2602_03067_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


@pytest.fixture()
def hctx(lib):
    h = ctypes.c_void_p()
    assert lib.fs_create(ctypes.byref(h), -1, None) == 0
    yield h
    lib.fs_destroy(h)


def _declared():
    text = open(os.path.join(ROOT, "include", "flashsink.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z_A-Z0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    for required in ("fs_row_norms", "fs_update_f", "fs_update_g", "fs_solve", "fs_marginal_err",
                     "fs_apply_plan", "fs_apply_plan_T"):
        assert required in names
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.EXPORTS)
    assert lib.fs_version().decode().startswith("flashsink")


def _prob(**kw):
    base = dict(x=4096, y=8192, dtype=0, compute=0, n=10, m=12, d=3, ldx=3, ldy=3, a=None, b=None)
    base.update(kw)
    return binding.FsProblem(base["x"], base["y"], base["dtype"], base["compute"], base["n"],
                             base["m"], base["d"], base["ldx"], base["ldy"], base["a"], base["b"])


F = ctypes.c_float
P = ctypes.c_void_p


def test_status_strings(lib):
    seen = {lib.fs_status_str(s).decode() for s in range(9)}
    assert len(seen) == 9 and "ok" in seen


def test_valid_arguments_reach_the_device_stage(lib, hctx):
    p = _prob()
    st = lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), P(1 << 21))
    assert st == 7 and b"host-only" in lib.fs_last_error(hctx)


@pytest.mark.parametrize("kw,status", [
    (dict(x=None), 1), (dict(y=None), 1), (dict(dtype=5), 1), (dict(compute=9), 1),
    (dict(n=0), 2), (dict(m=-3), 2), (dict(d=0), 2), (dict(ldx=2), 2), (dict(ldy=1), 2),
    (dict(n=(1 << 24) + 1), 2), (dict(d=9000, ldx=9000, ldy=9000), 2),
    (dict(compute=1, d=8, ldx=8, ldy=8), 5),
])
def test_problem_validation(lib, hctx, kw, status):
    p = _prob(**kw)
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), P(1 << 21)) == status
    assert lib.fs_last_error(hctx) != b""
    assert lib.fs_solve(hctx, ctypes.byref(p), F(0.1), F(0.1), 1, 1, P(1 << 21), P(1 << 20)) == status


@pytest.mark.parametrize("eps", [0.0, -1.0, float("nan"), float("inf")])
def test_eps_validation(lib, hctx, eps):
    p = _prob()
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(eps), P(1 << 20), P(1 << 21)) == 3
    assert lib.fs_update_g(hctx, ctypes.byref(p), F(eps), P(1 << 20), P(1 << 21)) == 3
    assert lib.fs_solve(hctx, ctypes.byref(p), F(1.0), F(eps), 1, 1, P(1 << 21), P(1 << 20)) == 3
    assert lib.fs_solve(hctx, ctypes.byref(p), F(eps), F(0.1), 3, 1, P(1 << 21), P(1 << 20)) == 3
    e = F()
    assert lib.fs_marginal_err(hctx, ctypes.byref(p), F(eps), P(1 << 21), P(1 << 20),
                               ctypes.byref(e), ctypes.byref(e)) == 3


def test_solve_count_validation(lib, hctx):
    p = _prob()
    assert lib.fs_solve(hctx, ctypes.byref(p), F(1.0), F(0.1), 0, 1, P(1 << 21), P(1 << 20)) == 3
    assert lib.fs_solve(hctx, ctypes.byref(p), F(1.0), F(0.1), 1, -1, P(1 << 21), P(1 << 20)) == 3
    assert lib.fs_solve_symmetric(hctx, ctypes.byref(p), F(0.1), -1, P(1 << 21), P(1 << 20)) == 3
    assert lib.fs_solve_symmetric(hctx, ctypes.byref(p), F(0.0), 1, P(1 << 21), P(1 << 20)) == 3
    assert lib.fs_solve_symmetric(hctx, ctypes.byref(p), F(0.1), 1, None, P(1 << 20)) == 1
    it, er = ctypes.c_int32(), F()
    assert lib.fs_solve_tol(hctx, ctypes.byref(p), F(0.1), 0, 1, F(1e-3), P(1 << 21), P(1 << 20),
                            ctypes.byref(it), ctypes.byref(er)) == 3
    assert lib.fs_solve_tol(hctx, ctypes.byref(p), F(0.1), 5, 0, F(1e-3), P(1 << 21), P(1 << 20),
                            ctypes.byref(it), ctypes.byref(er)) == 3
    assert lib.fs_solve_tol(hctx, ctypes.byref(p), F(0.1), 5, 1, F(1e-3), P(1 << 21), P(1 << 20), None,
                            ctypes.byref(er)) == 1
    k = ctypes.c_int32()
    assert lib.fs_hvp(hctx, ctypes.byref(p), F(0.1), P(1 << 21), P(1 << 20), None, 3, F(1e-5), F(1e-6), 10,
                      P(1 << 22), 3, ctypes.byref(k)) == 1
    assert lib.fs_hvp(hctx, ctypes.byref(p), F(0.1), P(1 << 21), P(1 << 20), P(1 << 23), 2, F(1e-5), F(1e-6), 10,
                      P(1 << 22), 3, ctypes.byref(k)) == 2
    assert lib.fs_hvp(hctx, ctypes.byref(p), F(0.1), P(1 << 21), P(1 << 20), P(1 << 23), 3, F(-1.0), F(1e-6), 10,
                      P(1 << 22), 3, ctypes.byref(k)) == 3
    v = ctypes.c_double()
    assert lib.fs_ot_value(hctx, ctypes.byref(p), F(0.1), P(1 << 21), P(1 << 20), None) == 1
    assert lib.fs_ot_value(hctx, ctypes.byref(p), F(-1.0), P(1 << 21), P(1 << 20), ctypes.byref(v)) == 3


def test_noalloc_solve_checks_sizes_on_the_host(lib, hctx):
    """fs_solve_noalloc validates like fs_solve and refuses, before any launch, a problem whose workspace is beyond
    the static scratch array."""
    args = lambda p, **kw: (hctx, ctypes.byref(p), F(kw.get("e0", 0.1)), F(kw.get("e1", 0.1)), kw.get("stages", 1),
                            kw.get("iters", 1), P(1 << 32), P(1 << 33))
    small = _prob(n=50000, m=50000)
    assert lib.fs_solve_noalloc(*args(small)) == 7                     # valid: reaches device stage
    big = _prob(n=60000, m=60000)
    assert lib.fs_solve_noalloc(*args(big)) == 2 and b"fs_solve_noalloc" in lib.fs_last_error(hctx)
    assert lib.fs_solve(*args(big)) == 7                               # the allocating entry point takes it
    assert lib.fs_solve_noalloc(*args(big, iters=0)) == 2              # also with nothing to do
    assert lib.fs_solve_noalloc(*args(small, e1=-1.0)) == 3
    assert lib.fs_solve_noalloc(*args(small, stages=0)) == 3
    assert lib.fs_solve_noalloc(*args(_prob(d=0))) == 2


def test_labeled_solve_validation(lib, hctx):
    p = _prob()
    args = lambda V=4, l1=0.5, l2=0.5, eps=0.1, iters=3, lx=1 << 24, ly=1 << 25, W=1 << 26, f=1 << 21, g=1 << 22, prob=p: (
        hctx, ctypes.byref(prob), P(lx) if lx else None, P(ly) if ly else None, P(W) if W else None, V, F(l1), F(l2), F(eps),
        iters, P(f) if f else None, P(g) if g else None)
    assert lib.fs_solve_labeled(*args(lx=None)) == 1
    assert lib.fs_solve_labeled(*args(W=None)) == 1
    assert lib.fs_solve_labeled(*args(f=None)) == 1
    assert lib.fs_solve_labeled(*args(V=0)) == 2
    assert lib.fs_solve_labeled(*args(V=8190)) == 2                   # d + V beyond the supported dimension
    assert lib.fs_solve_labeled(*args(l1=0.0)) == 1
    assert lib.fs_solve_labeled(*args(l2=float("inf"))) == 1
    assert lib.fs_solve_labeled(*args(eps=0.0)) == 3
    assert lib.fs_solve_labeled(*args(iters=-1)) == 3
    assert lib.fs_solve_labeled(*args(g=(1 << 21) + 8)) == 1          # g on top of f
    assert lib.fs_solve_labeled(*args()) == 7                         # valid: reaches device stage


def test_null_and_aliasing(lib, hctx):
    p = _prob()
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), None, P(1 << 21)) == 1
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), None) == 1
    assert lib.fs_update_f(hctx, None, F(0.1), P(1 << 20), P(1 << 21)) == 1
    # output on top of x, and on top of the input potential
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), P(4096 + 8)) == 1
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), P((1 << 20) + 4)) == 1
    assert lib.fs_solve(hctx, ctypes.byref(p), F(0.1), F(0.1), 1, 1, P(1 << 21), P((1 << 21) + 8)) == 1
    assert lib.fs_update_f(None, ctypes.byref(p), F(0.1), P(1 << 20), P(1 << 21)) == 1


def test_apply_validation(lib, hctx):
    p = _prob()
    args = lambda pp, ldv, ldo, out=1 << 22: (hctx, ctypes.byref(p), F(0.1), P(1 << 21), P(1 << 20),
                                              P(1 << 23), pp, ldv, P(out), ldo, None)
    assert lib.fs_apply_plan(*args(0, 4, 4)) == 2
    assert lib.fs_apply_plan(*args(4, 3, 4)) == 2
    assert lib.fs_apply_plan_T(*args(4, 4, 2)) == 2
    assert lib.fs_apply_plan(*args(4, 4, 4, out=1 << 23)) == 1     # out aliases V
    assert lib.fs_apply_plan(*args(4, 4, 4)) == 7                  # valid: reaches device stage


def test_hadamard_validation(lib, hctx):
    p = _prob()
    args = lambda pp=4, lda=3, ldv=4, ldo=4, out=1 << 22, A=1 << 24, V=1 << 23, prob=p: (
        hctx, ctypes.byref(prob), F(0.1), P(1 << 21), P(1 << 20), P(A) if A else None, lda, P(V) if V else None, pp, ldv,
        P(out) if out else None, ldo)
    assert lib.fs_apply_plan_hadamard(*args(A=None)) == 1
    assert lib.fs_apply_plan_hadamard(*args(V=None)) == 1
    assert lib.fs_apply_plan_hadamard(*args(out=None)) == 1
    assert lib.fs_apply_plan_hadamard(*args(pp=0)) == 2
    assert lib.fs_apply_plan_hadamard(*args(lda=2)) == 2             # lda < d
    assert lib.fs_apply_plan_hadamard(*args(ldv=3)) == 2
    assert lib.fs_apply_plan_hadamard(*args(ldo=3)) == 2
    assert lib.fs_apply_plan_hadamard(*args(out=1 << 24)) == 1       # out on top of A
    assert lib.fs_apply_plan_hadamard(*args(out=1 << 23)) == 1       # out on top of V
    assert lib.fs_apply_plan_hadamard(*args(out=4096)) == 1          # out on top of x
    q = _prob(compute=1, d=32, ldx=32, ldy=32)
    assert lib.fs_apply_plan_hadamard(*args(lda=32, prob=q)) == 5    # bf16 mode is not covered
    assert lib.fs_apply_plan_hadamard(*args()) == 7                  # valid: reaches device stage


def test_grad_validation(lib, hctx):
    p = _prob()
    args = lambda mode, ldg, out=1 << 22, f=1 << 21: (hctx, ctypes.byref(p), F(0.1), P(f), P(1 << 20), mode, P(out), ldg)
    assert lib.fs_grad_x(*args(3, 3)) == 1                         # unknown mode
    assert lib.fs_grad_y(*args(-1, 3)) == 1
    assert lib.fs_grad_x(*args(0, 2)) == 2                         # ldg < d
    assert lib.fs_grad_x(*args(0, 3, out=None)) == 1
    assert lib.fs_grad_x(*args(0, 3, out=4096)) == 1               # grad on top of x
    assert lib.fs_grad_x(*args(0, 3, out=(1 << 21) + 8)) == 1      # grad on top of f
    assert lib.fs_grad_x(*args(0, 3)) == 7                         # valid: reaches device stage
    assert lib.fs_grad_y(*args(2, 5)) == 7


def test_divergence_validation(lib, hctx):
    p = _prob()
    v = ctypes.c_double()
    args = lambda iters, f=1 << 21, g=1 << 22, val=ctypes.byref(v): (hctx, ctypes.byref(p), F(0.1), iters, P(f) if f else None,
                                                                     P(g) if g else None, val, None)
    assert lib.fs_divergence(*args(0)) == 3                        # needs at least one iteration
    assert lib.fs_divergence(*args(5, val=None)) == 1
    assert lib.fs_divergence(*args(5, f=None)) == 1
    assert lib.fs_divergence(*args(5, g=(1 << 21) + 8)) == 1       # g on top of f
    assert lib.fs_divergence(*args(5, f=4096)) == 1                # f on top of x
    assert lib.fs_divergence(*args(5)) == 7                        # valid: reaches device stage


def test_debug_switches_are_per_context(lib, hctx):
    assert lib.fs_debug_set(hctx, b"lowd_score", 64) == 0
    assert lib.fs_debug_set(hctx, b"lowd_score", 0) == 0
    assert lib.fs_debug_set(hctx, b"lowd_splits", 7) == 0
    assert lib.fs_debug_set(hctx, b"lowd_precise_valu", 1) == 0
    assert lib.fs_debug_set(hctx, b"lowd_precise_any_bias", 1) == 0
    assert lib.fs_debug_set(hctx, b"lowd_precise_any_bias", 2) == 1
    assert lib.fs_debug_set(hctx, b"lowd_score", 16) == 1            # value out of range
    assert lib.fs_debug_set(hctx, b"lowd_splits", -1) == 1
    assert lib.fs_debug_set(hctx, b"no_such_switch", 1) == 1 and b"no_such_switch" in lib.fs_last_error(hctx)
    assert lib.fs_debug_set(hctx, None, 1) == 1
    assert lib.fs_debug_set(None, b"lowd_score", 0) == 1
    # the library reads no environment variable: its sources do not call getenv
    import glob
    for src in glob.glob(os.path.join(ROOT, "paper_2602_03067_amd", "csrc", "*")):
        assert "getenv" not in open(src).read(), src


def test_points_keep_validation(lib, hctx):
    """Host-only state: the declaration is validated like any problem and can be withdrawn; nothing is launched."""
    p = _prob()
    assert lib.fs_points_keep(hctx, ctypes.byref(p)) == 0
    assert lib.fs_points_release(hctx) == 0
    assert lib.fs_points_release(hctx) == 0                        # releasing twice is harmless
    assert lib.fs_points_keep(hctx, ctypes.byref(_prob(n=0))) == 2
    assert lib.fs_points_keep(hctx, ctypes.byref(_prob(x=None))) == 1
    assert lib.fs_points_keep(hctx, None) == 1
    assert lib.fs_points_keep(None, ctypes.byref(p)) == 1
    assert lib.fs_points_release(None) == 1
    # an entry call after the declaration still validates and reaches the device stage of a host-only context
    assert lib.fs_points_keep(hctx, ctypes.byref(p)) == 0
    assert lib.fs_update_f(hctx, ctypes.byref(p), F(0.1), P(1 << 20), P(1 << 21)) == 7
    assert lib.fs_points_release(hctx) == 0


def test_row_norms_validation(lib, hctx):
    assert lib.fs_row_norms(hctx, None, 0, 4, 3, 3, P(1 << 20)) == 1
    assert lib.fs_row_norms(hctx, P(4096), 0, 0, 3, 3, P(1 << 20)) == 2
    assert lib.fs_row_norms(hctx, P(4096), 0, 4, 3, 2, P(1 << 20)) == 2
    assert lib.fs_row_norms(hctx, P(4096), 0, 4, 3, 3, P(4100)) == 1
    assert lib.fs_row_norms(hctx, P(4096), 0, 4, 3, 3, P(1 << 20)) == 7


def test_no_gpu_means_loud_failure(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = ctypes.c_void_p()
    assert lib.fs_create(ctypes.byref(h), 0, None) == 7
    with pytest.raises(RuntimeError):
        binding.Context(0)


def test_check_weights_validation(lib, hctx):
    sa, sb = ctypes.c_double(), ctypes.c_double()
    p = _prob()
    assert lib.fs_check_weights(hctx, None, F(1e-5), None, None) == 1
    assert lib.fs_check_weights(hctx, ctypes.byref(p), F(-1.0), None, None) == 1
    assert lib.fs_check_weights(hctx, ctypes.byref(p), F(float("nan")), None, None) == 1
    # uniform weights on both sides: nothing to check, also without a device
    assert lib.fs_check_weights(hctx, ctypes.byref(p), F(1e-5), ctypes.byref(sa), ctypes.byref(sb)) == 0
    assert sa.value == 1.0 and sb.value == 1.0
    q = _prob(a=1 << 24)
    assert lib.fs_check_weights(hctx, ctypes.byref(q), F(1e-5), None, None) == 7   # valid: reaches device stage


def test_check_finite_validation(lib, hctx):
    bad = ctypes.c_int64()
    assert lib.fs_check_finite(None, P(1 << 20), 10, None) == 1
    assert lib.fs_check_finite(hctx, None, 10, None) == 1
    assert lib.fs_check_finite(hctx, P(1 << 20), 0, ctypes.byref(bad)) == 2
    assert lib.fs_check_finite(hctx, P(1 << 20), 10, ctypes.byref(bad)) == 7   # valid: reaches device stage


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; --gpus 2 (or a multi-rank environment) ends with a message, before
    anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
