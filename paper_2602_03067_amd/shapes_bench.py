"""Timings on the shapes of the paper's synthetic benchmark tables (Section 4.1 and the appendix with
the full results): points uniform on [0,1]^d, uniform weights, eps = 0.1, fixed iteration count.

    python -m paper_2602_03067_amd.shapes_bench [--quick]

"forward" = fs_solve (10 iterations from zero potentials) + fs_ot_value; "forward+backward" adds
fs_grad_x (the plan applied to y and the assembly of Cor. 4).  Both compute modes are timed: bf16
(matrix-core scores from bf16-rounded points, the closest to the paper's TF32 setting) and fp32
(the library's fp32-accuracy mode).  Prints one line per shape; times are medians of 5 runs after
2 warm-up runs, measured with events on the library's stream.  Context for a reader who wants to
set this library next to the paper's tables; it is not the benchmark contract (that is bench.py).
"""
from __future__ import annotations

import argparse
import sys

import numpy as np
import torch

from . import binding


def _cloud(rng, n, d):
    return torch.from_numpy(rng.random((n, d), dtype=np.float32)).to("cuda:0")


def _time(fn, reps=5, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    return float(np.median(ts))


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="a few shapes only")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("shapes_bench: no GPU visible", file=sys.stderr)
        return 2
    ctx = binding.Context(0)
    rng = np.random.default_rng(2602)
    eps, iters = 0.1, 10
    square = [(10000, 10000, 64), (10000, 10000, 128), (10000, 10000, 512), (10000, 10000, 1024), (20000, 20000, 64),
              (40000, 40000, 128), (40000, 40000, 512), (50000, 50000, 64), (50000, 50000, 1024)]
    rect = [(1000, 10000, 128), (2000, 20000, 128), (10000, 1000, 128), (500, 50000, 128)]
    lowd = [(10000, 10000, 4), (50000, 50000, 4), (10000, 10000, 16)]
    shapes = [(10000, 10000, 64), (10000, 10000, 1024), (500, 50000, 128), (10000, 10000, 4)] if args.quick else square + rect + lowd
    print("%-22s %-5s %12s %12s %12s %12s" % ("n x m, d", "mode", "fwd alt ms", "fwd sym ms", "fwd+bwd ms", "ms / iter"))
    for (n, m, d) in shapes:
        x, y = _cloud(rng, n, d), _cloud(rng, m, d)
        for mode in ("bf16", "fp32"):
            if mode == "bf16" and d < 16:
                continue
            prob = binding.Problem(x, y, None, None,
                                   binding.FS_COMPUTE_BF16_MFMA if mode == "bf16" else binding.FS_COMPUTE_FP32)
            f = torch.zeros(n, device="cuda:0")
            g = torch.zeros(m, device="cuda:0")

            def fwd(sym=False, its=iters):
                f.zero_()
                g.zero_()
                if sym:
                    ctx.fs_solve_symmetric(prob, eps, its, f, g)
                else:
                    ctx.fs_solve(prob, eps, eps, 1, its, f, g)
                return ctx.fs_ot_value(prob, eps, f, g)

            def fwd_bwd():
                fwd()
                return ctx.fs_grad_x(prob, eps, f, g, 0)

            t_alt = _time(fwd)
            t_sym = _time(lambda: fwd(True))
            t_fb = _time(fwd_bwd)
            t_long = _time(lambda: fwd(False, 5 * iters), reps=3, warm=1)
            per_iter = (t_long - t_alt) / (4 * iters)
            print("%-22s %-5s %12.2f %12.2f %12.2f %12.3f" % ("%d x %d, %d" % (n, m, d), mode, t_alt, t_sym, t_fb, per_iter),
                  flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
