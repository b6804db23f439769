"""ctypes wrapper around fs_oracle.c (float64 CPU oracle; test infrastructure).

The C file is compiled with gcc on first use (or by ``build()``).  Inputs of any
float dtype are widened exactly to float64 before the call; the oracle itself
never rounds to a narrower type.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_oracle.c")
_LIB = os.path.join(_HERE, "libfs_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I64 = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile fs_oracle.c into libfs_oracle.so next to it (gcc -O2 -fopenmp)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, dbl, cint = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        lib.fso_num_threads.restype = cint
        lib.fso_num_threads.argtypes = []
        lib.fso_row_norms.argtypes = [_D, i64, i64, _D]
        lib.fso_half_step_rows.argtypes = [_D, _D, i64, i64, i64, _D, dbl, _D, _I64, i64, _D]
        lib.fso_stage_eps.restype = dbl
        lib.fso_stage_eps.argtypes = [dbl, dbl, cint, cint]
        lib.fso_solve.argtypes = [_D, _D, i64, i64, i64, _D, _D, dbl, dbl, cint, cint, _D, _D]
        lib.fso_solve_symmetric.argtypes = [_D, _D, i64, i64, i64, _D, _D, dbl, cint, _D, _D]
        lib.fso_marginals.argtypes = [_D, _D, i64, i64, i64, _D, _D, dbl, _D, _D, _D, _D]
        lib.fso_marginal_err.argtypes = [_D, _D, i64, i64, i64, _D, _D, dbl, _D, _D, _D, _D]
        lib.fso_apply_plan_rows.argtypes = [
            _D, _D, i64, i64, i64, _D, _D, dbl, _D, _D, _D, i64, _I64, i64, _D, _D]
        lib.fso_apply_plan_T_rows.argtypes = [
            _D, _D, i64, i64, i64, _D, _D, dbl, _D, _D, _D, i64, _I64, i64, _D, _D]
        lib.fso_objectives.argtypes = [_D, _D, i64, i64, i64, _D, _D, dbl, _D, _D, _D, _D]
        for name in ("fso_row_norms", "fso_half_step_rows", "fso_solve", "fso_solve_symmetric",
                     "fso_marginals", "fso_marginal_err", "fso_apply_plan_rows",
                     "fso_apply_plan_T_rows", "fso_objectives"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _f64(arr, ndim):
    out = np.ascontiguousarray(np.asarray(arr), dtype=np.float64)
    if out.ndim != ndim:
        raise ValueError("expected %d-d array, got shape %s" % (ndim, out.shape))
    return out


def _p(arr):
    return arr.ctypes.data_as(_D)


def _pts(x, y):
    x = _f64(x, 2)
    y = _f64(y, 2)
    if x.shape[1] != y.shape[1]:
        raise ValueError("x and y must have the same feature dimension")
    return x, y, x.shape[0], y.shape[0], x.shape[1]


def _idx(rows):
    if rows is None:
        return None, None
    r = np.ascontiguousarray(np.asarray(rows), dtype=np.int64)
    return r, r.ctypes.data_as(_I64)


def num_threads() -> int:
    return int(_load().fso_num_threads())


def row_norms(pts):
    pts = _f64(pts, 2)
    out = np.empty(pts.shape[0])
    _load().fso_row_norms(_p(pts), pts.shape[0], pts.shape[1], _p(out))
    return out


def half_step_rows(p, q, w, eps, pot, rows=None):
    """out_r = -eps*LSE_j[(pot_j - |p_i - q_j|^2)/eps + log w_j] for i in rows (all if None)."""
    p, q, np_, nq, d = _pts(p, q)
    w = _f64(w, 1)
    pot = _f64(pot, 1)
    assert w.shape[0] == nq and pot.shape[0] == nq
    ridx, rptr = _idx(rows)
    n_rows = np_ if ridx is None else ridx.shape[0]
    if ridx is not None and n_rows and (ridx.min() < 0 or ridx.max() >= np_):
        raise IndexError("row index out of range")
    out = np.empty(n_rows)
    _load().fso_half_step_rows(_p(p), _p(q), np_, nq, d, _p(w), float(eps), _p(pot),
                               rptr, n_rows, _p(out))
    return out


def update_f(x, y, b, eps, g, rows=None):
    """Eq. 2 of the paper: f from g (optionally for selected rows only)."""
    return half_step_rows(x, y, b, eps, g, rows)


def update_g(x, y, a, eps, f, cols=None):
    """Eq. 3 of the paper: g from f (optionally for selected columns only)."""
    return half_step_rows(y, x, a, eps, f, cols)


def stage_eps(eps_start, eps_end, n_stages, s) -> float:
    return float(_load().fso_stage_eps(float(eps_start), float(eps_end), int(n_stages), int(s)))


def solve(x, y, a, b, eps_start, eps_end, n_stages, iters, f0=None, g0=None):
    """Alternating schedule (App. B): n_stages*iters iterations of (f from g, g from new f)."""
    x, y, n, m, d = _pts(x, y)
    a = _f64(a, 1)
    b = _f64(b, 1)
    f = np.zeros(n) if f0 is None else _f64(f0, 1).copy()
    g = np.zeros(m) if g0 is None else _f64(g0, 1).copy()
    _load().fso_solve(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps_start), float(eps_end),
                      int(n_stages), int(iters), _p(f), _p(g))
    return f, g


def solve_symmetric(x, y, a, b, eps, iters, f0=None, g0=None):
    """Symmetric averaged schedule (Eq. 4-5)."""
    x, y, n, m, d = _pts(x, y)
    a = _f64(a, 1)
    b = _f64(b, 1)
    f = np.zeros(n) if f0 is None else _f64(f0, 1).copy()
    g = np.zeros(m) if g0 is None else _f64(g0, 1).copy()
    _load().fso_solve_symmetric(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), int(iters),
                                _p(f), _p(g))
    return f, g


def marginals(x, y, a, b, eps, f, g):
    x, y, n, m, d = _pts(x, y)
    a, b, f, g = _f64(a, 1), _f64(b, 1), _f64(f, 1), _f64(g, 1)
    r = np.empty(n)
    c = np.empty(m)
    _load().fso_marginals(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), _p(f), _p(g),
                          _p(r), _p(c))
    return r, c


def marginal_err(x, y, a, b, eps, f, g):
    x, y, n, m, d = _pts(x, y)
    a, b, f, g = _f64(a, 1), _f64(b, 1), _f64(f, 1), _f64(g, 1)
    er = ctypes.c_double()
    ec = ctypes.c_double()
    _load().fso_marginal_err(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), _p(f), _p(g),
                             ctypes.byref(er), ctypes.byref(ec))
    return er.value, ec.value


def apply_plan(x, y, a, b, eps, f, g, V, rows=None, return_mass=False):
    """(P V)_i = sum_j P_ij V_j with P_ij = a_i b_j exp((f_i+g_j-C_ij)/eps)."""
    x, y, n, m, d = _pts(x, y)
    a, b, f, g = _f64(a, 1), _f64(b, 1), _f64(f, 1), _f64(g, 1)
    V = _f64(V, 2)
    assert V.shape[0] == m
    ridx, rptr = _idx(rows)
    n_rows = n if ridx is None else ridx.shape[0]
    out = np.empty((n_rows, V.shape[1]))
    mass = np.empty(n_rows)
    _load().fso_apply_plan_rows(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), _p(f), _p(g),
                                _p(V), V.shape[1], rptr, n_rows, _p(out), _p(mass))
    return (out, mass) if return_mass else out


def apply_plan_T(x, y, a, b, eps, f, g, U, cols=None, return_mass=False):
    """(P^T U)_j = sum_i P_ij U_i."""
    x, y, n, m, d = _pts(x, y)
    a, b, f, g = _f64(a, 1), _f64(b, 1), _f64(f, 1), _f64(g, 1)
    U = _f64(U, 2)
    assert U.shape[0] == n
    cidx, cptr = _idx(cols)
    n_cols = m if cidx is None else cidx.shape[0]
    out = np.empty((n_cols, U.shape[1]))
    mass = np.empty(n_cols)
    _load().fso_apply_plan_T_rows(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), _p(f),
                                  _p(g), _p(U), U.shape[1], cptr, n_cols, _p(out), _p(mass))
    return (out, mass) if return_mass else out


def objectives(x, y, a, b, eps, f, g):
    """(primal, dual) of the plan induced by (f, g): Eq. 1 and the App. B Lagrangian."""
    x, y, n, m, d = _pts(x, y)
    a, b, f, g = _f64(a, 1), _f64(b, 1), _f64(f, 1), _f64(g, 1)
    pr = ctypes.c_double()
    du = ctypes.c_double()
    _load().fso_objectives(_p(x), _p(y), n, m, d, _p(a), _p(b), float(eps), _p(f), _p(g),
                           ctypes.byref(pr), ctypes.byref(du))
    return pr.value, du.value
