"""Seeded synthetic point-cloud workloads (inputs only; no Sinkhorn arithmetic).

Both the GPU library's tests/bench and the CPU oracle take their inputs from
here, so that they see bit-identical arrays.  Everything is drawn from
``numpy.random.Generator(PCG64(seed))`` in float64, in the fixed order
x, y, a, b, U, and then rounded once to the storage type; the rounded arrays are
the canonical inputs.

The five named workloads follow the shapes and distributions of the benchmark
configurations; ``n``/``m`` can be overridden to get the same distribution at a
size the float64 oracle can finish.  Workload "mnist_shape" only borrows the
shape (70000 x 784) and value range of a well-known image dataset; no dataset
item is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = ["Workload", "make", "NAMES", "to_bf16_round", "bf16_bits"]


def bf16_bits(arr32: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(arr32, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def to_bf16_round(arr32: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bfloat16 (RNE)."""
    bits = bf16_bits(arr32).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).reshape(np.shape(arr32))


@dataclass
class Workload:
    name: str
    x: np.ndarray            # (n, d) float32 (values bf16-representable if storage == "bf16")
    y: np.ndarray            # (m, d) float32
    a: np.ndarray            # (n,) float32, > 0, sums to ~1
    b: np.ndarray            # (m,) float32
    eps_start: float
    eps_end: float
    n_stages: int
    iters: int               # iterations per stage
    storage: str = "f32"     # "f32" | "bf16": type the library receives x, y in
    compute: str = "fp32"    # "fp32" | "bf16_mfma"
    U: Optional[np.ndarray] = None   # (n, p) float32 for P^T U
    V: Optional[np.ndarray] = None   # (m, p) float32 for P V
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n(self):
        return self.x.shape[0]

    @property
    def m(self):
        return self.y.shape[0]

    @property
    def d(self):
        return self.x.shape[1]

    @property
    def total_iters(self):
        return self.n_stages * self.iters


NAMES = ("tiny", "lowdim_anneal", "mnist_shape", "embedding", "transport_grad")
_SEEDS = {"tiny": 1001, "lowdim_anneal": 1002, "mnist_shape": 1003, "embedding": 1004,
          "transport_grad": 1005}
_DEFAULT = {
    "tiny": (1024, 1024, 3),
    "lowdim_anneal": (262144, 262144, 3),
    "mnist_shape": (70000, 70000, 784),
    "embedding": (50000, 20000, 1024),
    "transport_grad": (16384, 16384, 64),
}


def _uniform_w(k):
    return np.full(k, 1.0 / k, dtype=np.float64).astype(np.float32)


def _dirichlet1(rng, k):
    e = rng.exponential(1.0, size=k)
    return (e / e.sum()).astype(np.float32)


def make(name: str, n: Optional[int] = None, m: Optional[int] = None, d: Optional[int] = None,
         seed: Optional[int] = None, iters: Optional[int] = None) -> Workload:
    """Build one of the named workloads, optionally scaled down."""
    if name not in _DEFAULT:
        raise KeyError("unknown workload %r (known: %s)" % (name, ", ".join(NAMES)))
    n0, m0, d0 = _DEFAULT[name]
    n = n0 if n is None else int(n)
    m = m0 if m is None else int(m)
    d = d0 if d is None else int(d)
    seed = _SEEDS[name] if seed is None else int(seed)
    rng = np.random.Generator(np.random.PCG64(seed))

    if name == "tiny":
        x = rng.standard_normal((n, d))
        y = rng.standard_normal((m, d)) + 0.5
        w = Workload(name, x.astype(np.float32), y.astype(np.float32), _uniform_w(n),
                     _uniform_w(m), 0.1, 0.1, 1, 50 if iters is None else iters, seed=seed)
    elif name == "lowdim_anneal":
        x = rng.random((n, d))
        means = rng.random((8, d))
        comp = rng.integers(0, 8, size=m)
        y = means[comp] + 0.05 * rng.standard_normal((m, d))
        w = Workload(name, x.astype(np.float32), y.astype(np.float32), _uniform_w(n),
                     _uniform_w(m), 1.0, 0.01, 20, 10 if iters is None else iters, seed=seed)
    elif name == "mnist_shape":
        x = rng.beta(0.5, 2.0, size=(n, d)).astype(np.float32)
        y = rng.beta(0.5, 2.0, size=(m, d)).astype(np.float32)
        k = 1000
        ii = rng.integers(0, n, size=k)
        jj = rng.integers(0, m, size=k)
        diff = x[ii].astype(np.float64) - y[jj].astype(np.float64)
        msd = float(np.mean(np.einsum("kd,kd->k", diff, diff)))
        eps = float(np.float32(0.05 * msd))
        w = Workload(name, x, y, _uniform_w(n), _uniform_w(m), eps, eps, 1,
                     100 if iters is None else iters, storage="f32", compute="bf16_mfma",
                     seed=seed, notes={"mean_sq_dist_sample": msd})
    elif name == "embedding":
        x = rng.standard_normal((n, d))
        y = rng.standard_normal((m, d))
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        y /= np.linalg.norm(y, axis=1, keepdims=True)
        x = to_bf16_round(x.astype(np.float32))
        y = to_bf16_round(y.astype(np.float32))
        a = _dirichlet1(rng, n)
        b = _dirichlet1(rng, m)
        w = Workload(name, x, y, a, b, 0.05, 0.05, 1, 200 if iters is None else iters,
                     storage="bf16", compute="bf16_mfma", seed=seed)
    else:  # transport_grad
        x = rng.standard_normal((n, d))
        y = rng.standard_normal((m, d)) + 1.0
        a = _uniform_w(n)
        b = _uniform_w(m)
        U = rng.standard_normal((n, 64)).astype(np.float32)
        w = Workload(name, x.astype(np.float32), y.astype(np.float32), a, b, 0.1, 0.1, 1,
                     100 if iters is None else iters, seed=seed, U=U)
        w.V = w.y  # the gradient wrt x needs P Y
    return w
