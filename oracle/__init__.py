"""float64 CPU oracle (test infrastructure, not part of the product path).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the GPU package.

``oracle.fs_oracle`` wraps the C implementation (``fs_oracle.c``: plain
definitions of Section 2.1 / Eq. 1-5 of the paper, float64, OpenMP over rows);
``oracle.dense_ref`` is a dense NumPy/SciPy version on explicit n x m matrices
used to cross-check the C code on tiny inputs; ``oracle.hvp_dense`` is the dense
Hessian-vector product of Thm. 5 and the Hadamard-weighted transport of Alg. 5
(small sizes), pinned by central differences of the gradient and by the
entry-by-entry definition.

Pin status (see tests/test_oracle_pins.py): every function of fs_oracle is
pinned by brute force on tiny inputs, exact special cases, invariants and the
Gaussian closed form, and so are both functions of hvp_dense; none is "parity
unpinned".
"""
from .fs_oracle import (  # noqa: F401
    apply_plan,
    apply_plan_T,
    build,
    half_step_rows,
    marginal_err,
    marginals,
    num_threads,
    objectives,
    row_norms,
    solve,
    solve_symmetric,
    stage_eps,
    update_f,
    update_g,
)
