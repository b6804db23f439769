"""Thin ctypes binding of libflashsink (argument marshalling only).

Function names match the C ABI in ``include/flashsink.h``.  Tensors are PyTorch
CUDA(ROCm) tensors used purely as device memory; every step of the method runs
inside the library's HIP kernels.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch  # loaded first so that the library binds to the same HIP runtime as torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libflashsink.so")

FS_F32, FS_BF16 = 0, 1
FS_COMPUTE_FP32, FS_COMPUTE_BF16_MFMA = 0, 1

EXPORTS = (
    "fs_create", "fs_destroy", "fs_status_str", "fs_last_error", "fs_version", "fs_row_norms",
    "fs_update_f", "fs_update_g", "fs_solve", "fs_solve_noalloc", "fs_solve_labeled", "fs_solve_symmetric", "fs_solve_tol", "fs_marginal_err", "fs_ot_value", "fs_check_weights", "fs_check_finite", "fs_divergence", "fs_apply_plan",
    "fs_apply_plan_T", "fs_apply_plan_hadamard", "fs_grad_x", "fs_grad_y", "fs_hvp", "fs_points_keep", "fs_points_release", "fs_debug_set", "fs_profile_enable", "fs_profile_read",
)


class FsProblem(ctypes.Structure):
    _fields_ = [
        ("x", ctypes.c_void_p), ("y", ctypes.c_void_p),
        ("dtype", ctypes.c_int32), ("compute", ctypes.c_int32),
        ("n", ctypes.c_int64), ("m", ctypes.c_int64), ("d", ctypes.c_int64),
        ("ldx", ctypes.c_int64), ("ldy", ctypes.c_int64),
        ("a", ctypes.c_void_p), ("b", ctypes.c_void_p),
    ]


class FlashSinkError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str):
        super().__init__("%s: status %d (%s)" % (what, status, detail))
        self.status = status


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libflashsink.so (built in-tree by ``python -m paper_2602_03067_amd.build``)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2602_03067_amd.build` "
            "(there is no fallback path)" % path)
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    PP = ctypes.POINTER(FsProblem)
    lib.fs_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp]
    lib.fs_destroy.argtypes = [vp]
    lib.fs_status_str.argtypes = [ctypes.c_int]
    lib.fs_status_str.restype = ctypes.c_char_p
    lib.fs_last_error.argtypes = [vp]
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_version.argtypes = []
    lib.fs_version.restype = ctypes.c_char_p
    lib.fs_row_norms.argtypes = [vp, vp, i32, i64, i64, i64, vp]
    lib.fs_update_f.argtypes = [vp, PP, f32, vp, vp]
    lib.fs_update_g.argtypes = [vp, PP, f32, vp, vp]
    lib.fs_solve.argtypes = [vp, PP, f32, f32, i32, i32, vp, vp]
    lib.fs_solve_noalloc.argtypes = [vp, PP, f32, f32, i32, i32, vp, vp]
    lib.fs_solve_labeled.argtypes = [vp, PP, vp, vp, vp, i32, f32, f32, f32, i32, vp, vp]
    lib.fs_solve_symmetric.argtypes = [vp, PP, f32, i32, vp, vp]
    lib.fs_solve_tol.argtypes = [vp, PP, f32, i32, i32, f32, vp, vp, ctypes.POINTER(i32), ctypes.POINTER(f32)]
    lib.fs_marginal_err.argtypes = [vp, PP, f32, vp, vp, ctypes.POINTER(f32), ctypes.POINTER(f32)]
    lib.fs_ot_value.argtypes = [vp, PP, f32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.fs_check_finite.argtypes = [vp, vp, i64, ctypes.POINTER(ctypes.c_int64)]
    lib.fs_check_weights.argtypes = [vp, PP, f32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.fs_divergence.argtypes = [vp, PP, f32, i32, vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.fs_apply_plan.argtypes = [vp, PP, f32, vp, vp, vp, i64, i64, vp, i64, vp]
    lib.fs_apply_plan_T.argtypes = [vp, PP, f32, vp, vp, vp, i64, i64, vp, i64, vp]
    lib.fs_apply_plan_hadamard.argtypes = [vp, PP, f32, vp, vp, vp, i64, vp, i64, i64, vp, i64]
    lib.fs_grad_x.argtypes = [vp, PP, f32, vp, vp, i32, vp, i64]
    lib.fs_grad_y.argtypes = [vp, PP, f32, vp, vp, i32, vp, i64]
    lib.fs_hvp.argtypes = [vp, PP, f32, vp, vp, vp, i64, f32, f32, i32, vp, i64, ctypes.POINTER(i32)]
    lib.fs_debug_set.argtypes = [vp, ctypes.c_char_p, i64]
    lib.fs_points_keep.argtypes = [vp, PP]
    lib.fs_points_release.argtypes = [vp]
    lib.fs_profile_enable.argtypes = [vp, i32]
    lib.fs_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64),
                                    ctypes.POINTER(ctypes.c_double)]
    for name in EXPORTS:
        if name not in ("fs_status_str", "fs_last_error", "fs_version"):
            getattr(lib, name).restype = ctypes.c_int
    if path == LIB_PATH:
        _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev_f32(t: torch.Tensor, name: str, shape=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 \
            or not t.is_contiguous():
        raise TypeError("%s must be a contiguous float32 tensor on the GPU" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return t


class Problem:
    """Holds the tensors of one OT problem and the matching C struct."""

    def __init__(self, x: torch.Tensor, y: torch.Tensor, a: Optional[torch.Tensor] = None,
                 b: Optional[torch.Tensor] = None, compute: int = FS_COMPUTE_FP32):
        for t, nm in ((x, "x"), (y, "y")):
            if not t.is_cuda or t.dim() != 2 or t.stride(1) != 1:
                raise TypeError("%s must be a 2-d GPU tensor with unit inner stride" % nm)
        if x.dtype != y.dtype or x.dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("x and y must both be float32 or both bfloat16")
        if x.shape[1] != y.shape[1]:
            raise ValueError("x and y differ in feature dimension")
        self.x, self.y, self.a, self.b = x, y, a, b
        if a is not None:
            _dev_f32(a, "a", (x.shape[0],))
        if b is not None:
            _dev_f32(b, "b", (y.shape[0],))
        self.n, self.m, self.d = x.shape[0], y.shape[0], x.shape[1]
        self.c = FsProblem(
            x.data_ptr(), y.data_ptr(), FS_BF16 if x.dtype == torch.bfloat16 else FS_F32,
            int(compute), self.n, self.m, self.d, x.stride(0), y.stride(0),
            None if a is None else a.data_ptr(), None if b is None else b.data_ptr())


class Context:
    """fs_ctx bound to a device and to the torch stream current at creation."""

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("flashsink needs a GPU: torch.cuda.is_available() is False")
        self.device = int(device)
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = ctypes.c_void_p()
        st = self.lib.fs_create(ctypes.byref(h), self.device, ctypes.c_void_p(self.stream.cuda_stream))
        if st != 0:
            raise FlashSinkError(st, "fs_create", self.lib.fs_status_str(st).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.fs_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int, what: str):
        if st != 0:
            detail = self.lib.fs_last_error(self.h).decode() or self.lib.fs_status_str(st).decode()
            raise FlashSinkError(st, what, detail)

    # ---- entry points (same names as the C ABI) --------------------------------------
    def fs_row_norms(self, pts: torch.Tensor) -> torch.Tensor:
        out = torch.empty(pts.shape[0], dtype=torch.float32, device=pts.device)
        dt = FS_BF16 if pts.dtype == torch.bfloat16 else FS_F32
        self._check(self.lib.fs_row_norms(self.h, _ptr(pts), dt, pts.shape[0], pts.shape[1],
                                          pts.stride(0), _ptr(out)), "fs_row_norms")
        return out

    def fs_update_f(self, prob: Problem, eps: float, g: torch.Tensor) -> torch.Tensor:
        _dev_f32(g, "g", (prob.m,))
        f = torch.empty(prob.n, dtype=torch.float32, device=g.device)
        self._check(self.lib.fs_update_f(self.h, ctypes.byref(prob.c), eps, _ptr(g), _ptr(f)),
                    "fs_update_f")
        return f

    def fs_update_g(self, prob: Problem, eps: float, f: torch.Tensor) -> torch.Tensor:
        _dev_f32(f, "f", (prob.n,))
        g = torch.empty(prob.m, dtype=torch.float32, device=f.device)
        self._check(self.lib.fs_update_g(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g)),
                    "fs_update_g")
        return g

    def fs_solve(self, prob: Problem, eps_start: float, eps_end: float, n_stages: int,
                 iters_per_stage: int, f: torch.Tensor, g: torch.Tensor) -> None:
        """In place: f, g are the starting potentials and receive the result."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        self._check(self.lib.fs_solve(self.h, ctypes.byref(prob.c), eps_start, eps_end,
                                      int(n_stages), int(iters_per_stage), _ptr(f), _ptr(g)),
                    "fs_solve")

    def fs_solve_noalloc(self, prob: Problem, eps_start: float, eps_end: float, n_stages: int,
                         iters_per_stage: int, f: torch.Tensor, g: torch.Tensor) -> None:
        """fs_solve in the library's static scratch array (no device allocation); in place like fs_solve."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        self._check(self.lib.fs_solve_noalloc(self.h, ctypes.byref(prob.c), eps_start, eps_end,
                                              int(n_stages), int(iters_per_stage), _ptr(f), _ptr(g)),
                    "fs_solve_noalloc")

    def fs_solve_labeled(self, prob: Problem, lx: torch.Tensor, ly: torch.Tensor, W: torch.Tensor, lambda1: float,
                         lambda2: float, eps: float, iters: int, f: torch.Tensor, g: torch.Tensor) -> None:
        """Alternating Sinkhorn for lambda1 |x - y|^2 + lambda2 W[lx, ly]; in place like fs_solve."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        _dev_f32(W, "W")
        if W.dim() != 2 or W.shape[0] != W.shape[1]:
            raise ValueError("W must be square")
        for t, nm, cnt in ((lx, "lx", prob.n), (ly, "ly", prob.m)):
            if not t.is_cuda or t.dtype != torch.int32 or not t.is_contiguous() or tuple(t.shape) != (cnt,):
                raise TypeError("%s must be a contiguous int32 GPU tensor of %d labels" % (nm, cnt))
        self._check(self.lib.fs_solve_labeled(self.h, ctypes.byref(prob.c), _ptr(lx), _ptr(ly), _ptr(W), W.shape[0],
                                              float(lambda1), float(lambda2), float(eps), int(iters), _ptr(f), _ptr(g)),
                    "fs_solve_labeled")

    def fs_solve_tol(self, prob: Problem, eps: float, max_iters: int, check_every: int, tol: float,
                     f: torch.Tensor, g: torch.Tensor) -> Tuple[int, float]:
        """In place like fs_solve; returns (iterations done, measured L1 row marginal error)."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        done, err = ctypes.c_int32(), ctypes.c_float()
        self._check(self.lib.fs_solve_tol(self.h, ctypes.byref(prob.c), eps, int(max_iters), int(check_every),
                                          float(tol), _ptr(f), _ptr(g), ctypes.byref(done), ctypes.byref(err)),
                    "fs_solve_tol")
        return done.value, err.value

    def fs_ot_value(self, prob: Problem, eps: float, f: torch.Tensor, g: torch.Tensor) -> float:
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        v = ctypes.c_double()
        self._check(self.lib.fs_ot_value(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g), ctypes.byref(v)),
                    "fs_ot_value")
        return v.value

    def fs_check_finite(self, v: torch.Tensor) -> int:
        """Raises (status 8) if an entry of the float tensor is NaN or infinite; returns 0 otherwise."""
        assert v.dtype == torch.float32 and v.is_contiguous()
        bad = ctypes.c_int64()
        self._check(self.lib.fs_check_finite(self.h, _ptr(v), v.numel(), ctypes.byref(bad)), "fs_check_finite")
        return bad.value

    def fs_check_weights(self, prob: Problem, tol: float = 1e-5):
        """Raises if a weight is not positive and finite or a sum is off by more than tol; returns the two sums."""
        sa, sb = ctypes.c_double(), ctypes.c_double()
        self._check(self.lib.fs_check_weights(self.h, ctypes.byref(prob.c), tol, ctypes.byref(sa), ctypes.byref(sb)),
                    "fs_check_weights")
        return sa.value, sb.value

    def fs_divergence(self, prob: Problem, eps: float, iters: int):
        """Debiased Sinkhorn divergence; returns (value, (OT(a,b), OT(a,a), OT(b,b)), f, g)."""
        f = torch.empty(prob.n, dtype=torch.float32, device=prob.x.device)
        g = torch.empty(prob.m, dtype=torch.float32, device=prob.x.device)
        v = ctypes.c_double()
        t = (ctypes.c_double * 3)()
        self._check(self.lib.fs_divergence(self.h, ctypes.byref(prob.c), eps, int(iters), _ptr(f), _ptr(g), ctypes.byref(v), t),
                    "fs_divergence")
        return v.value, (t[0], t[1], t[2]), f, g

    def fs_solve_symmetric(self, prob: Problem, eps: float, iters: int, f: torch.Tensor,
                           g: torch.Tensor) -> None:
        """In place: f, g are the starting potentials and receive the result."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        self._check(self.lib.fs_solve_symmetric(self.h, ctypes.byref(prob.c), eps, int(iters), _ptr(f), _ptr(g)),
                    "fs_solve_symmetric")

    def fs_marginal_err(self, prob: Problem, eps: float, f: torch.Tensor,
                        g: torch.Tensor) -> Tuple[float, float]:
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        er, ec = ctypes.c_float(), ctypes.c_float()
        self._check(self.lib.fs_marginal_err(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g),
                                             ctypes.byref(er), ctypes.byref(ec)), "fs_marginal_err")
        return er.value, ec.value

    def _apply(self, fn, what, prob, eps, f, g, M, rows_out, rows_in, want_mass):
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        if M.dim() != 2 or M.shape[0] != rows_in or M.dtype != torch.float32 or M.stride(1) != 1:
            raise TypeError("matrix to apply must be float32 (rows=%d, p), unit inner stride" % rows_in)
        p = M.shape[1]
        out = torch.empty((rows_out, p), dtype=torch.float32, device=M.device)
        mass = torch.empty(rows_out, dtype=torch.float32, device=M.device) if want_mass else None
        self._check(fn(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g), _ptr(M), p, M.stride(0),
                       _ptr(out), out.stride(0), _ptr(mass)), what)
        return (out, mass) if want_mass else out

    def fs_apply_plan(self, prob: Problem, eps: float, f, g, V, want_mass: bool = False):
        return self._apply(self.lib.fs_apply_plan, "fs_apply_plan", prob, eps, f, g, V, prob.n,
                           prob.m, want_mass)

    def fs_apply_plan_T(self, prob: Problem, eps: float, f, g, U, want_mass: bool = False):
        return self._apply(self.lib.fs_apply_plan_T, "fs_apply_plan_T", prob, eps, f, g, U, prob.m,
                           prob.n, want_mass)

    def fs_apply_plan_hadamard(self, prob: Problem, eps: float, f, g, A: torch.Tensor, V: torch.Tensor) -> torch.Tensor:
        """(P o (A y^T)) V (Alg. 5); A is n x d, V is m x p; returns n x p."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        _dev_f32(A, "A", (prob.n, prob.d))
        if V.dim() != 2 or V.shape[0] != prob.m or V.dtype != torch.float32 or V.stride(1) != 1:
            raise TypeError("V must be float32 (m, p) with unit inner stride")
        p = V.shape[1]
        out = torch.empty((prob.n, p), dtype=torch.float32, device=V.device)
        self._check(self.lib.fs_apply_plan_hadamard(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g), _ptr(A), A.stride(0),
                                                    _ptr(V), p, V.stride(0), _ptr(out), out.stride(0)),
                    "fs_apply_plan_hadamard")
        return out

    def _grad(self, fn, name, prob: Problem, eps: float, f, g, mode: int, rows: int) -> torch.Tensor:
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        out = torch.empty(rows, prob.d, dtype=torch.float32, device=f.device)
        self._check(fn(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g), int(mode), _ptr(out), prob.d), name)
        return out

    def fs_grad_x(self, prob: Problem, eps: float, f, g, mode: int = 0) -> torch.Tensor:
        """Gradient with respect to x (n x d); mode 0: 2(diag(a)x - Py), 1: with r = P1, 2: x - (Py)/a."""
        return self._grad(self.lib.fs_grad_x, "fs_grad_x", prob, eps, f, g, mode, prob.n)

    def fs_grad_y(self, prob: Problem, eps: float, f, g, mode: int = 0) -> torch.Tensor:
        return self._grad(self.lib.fs_grad_y, "fs_grad_y", prob, eps, f, g, mode, prob.m)

    def fs_hvp(self, prob: Problem, eps: float, f: torch.Tensor, g: torch.Tensor, A: torch.Tensor,
               tau: float, eta: float, max_cg: int) -> Tuple[torch.Tensor, int]:
        """Hessian-vector product T A (Thm. 5); returns (G [n x d], CG iterations)."""
        _dev_f32(f, "f", (prob.n,))
        _dev_f32(g, "g", (prob.m,))
        _dev_f32(A, "A", (prob.n, prob.d))
        out = torch.empty(prob.n, prob.d, dtype=torch.float32, device=f.device)
        it = ctypes.c_int32()
        self._check(self.lib.fs_hvp(self.h, ctypes.byref(prob.c), eps, _ptr(f), _ptr(g), _ptr(A), prob.d,
                                    float(tau), float(eta), int(max_cg), _ptr(out), prob.d, ctypes.byref(it)),
                    "fs_hvp")
        return out, it.value

    def fs_points_keep(self, prob: Problem) -> None:
        """Declare the clouds of `prob` unchanged until fs_points_release: later calls reuse their derived copies."""
        self._check(self.lib.fs_points_keep(self.h, ctypes.byref(prob.c)), "fs_points_keep")

    def fs_points_release(self) -> None:
        self._check(self.lib.fs_points_release(self.h), "fs_points_release")

    def fs_debug_set(self, key: str, value: int) -> None:
        """Test and experiment switches of this context (0 = the library decides)."""
        self._check(self.lib.fs_debug_set(self.h, key.encode(), int(value)), "fs_debug_set")

    def fs_profile_enable(self, on: bool) -> None:
        self._check(self.lib.fs_profile_enable(self.h, 1 if on else 0), "fs_profile_enable")

    def fs_profile_read(self):
        avg, cnt, pairs = ctypes.c_double(), ctypes.c_int64(), ctypes.c_double()
        self._check(self.lib.fs_profile_read(self.h, ctypes.byref(avg), ctypes.byref(cnt),
                                             ctypes.byref(pairs)), "fs_profile_read")
        return avg.value, cnt.value, pairs.value


def problem_from_workload(w, device="cuda:0") -> Problem:
    """Upload a ``workloads.Workload`` (host arrays) and wrap it as a Problem."""
    dev = torch.device(device)
    x = torch.from_numpy(w.x).to(dev)
    y = torch.from_numpy(w.y).to(dev)
    if w.storage == "bf16":
        x, y = x.to(torch.bfloat16), y.to(torch.bfloat16)   # exact: values are bf16-representable
    a = torch.from_numpy(w.a).to(dev)
    b = torch.from_numpy(w.b).to(dev)
    compute = FS_COMPUTE_BF16_MFMA if w.compute == "bf16_mfma" else FS_COMPUTE_FP32
    return Problem(x, y, a, b, compute)
