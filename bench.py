#!/usr/bin/env python3
"""Benchmark of the fused Sinkhorn hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--no-per-config]

One "step" is one pass of the whole hot path over the workload, inputs already resident
in HBM: fs_row_norms of both clouds, fs_solve (all stages and iterations), fs_marginal_err,
fs_grad_x (the plan applied to y and the assembly x - (P y)/a) and fs_apply_plan_T (U: the
workload's own 64 columns where it has them, else min(d, 64) seeded normal columns).
The headline workload is the large low-dimension annealed problem (n = m = 262144, d = 3,
eps 1.0 -> 0.01 over 20 stages x 10 iterations).  Prints ONE JSON line; its "per_config"
array carries the same measurement (fewer steps) for the other four workloads.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X fp32 vector peak: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.64e12 lane-operations
# per second (x 2 flop per FMA = the published 157.3 TFLOP/s).
VALU_LANE_SLOTS_PER_S = 256 * 4 * 32 * 2.4e9
PEAKS = {"bf16": 2.5e15, "f64": 78.6e12}
# HBM bytes per launch of the dominant kernel: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script on the
# default size of each workload, scaled by what the same counters read for a 1 GiB device copy in the same run.
# These are NOT measured by this run (they need the profiler); each entry names the summary under profiles/ it was
# copied from, and the figures go stale when a kernel changes without its profile being taken again.
MEASURED_TRAFFIC = {
    "lowdim_anneal": (191.79e6, "profiles/lse_lowd_split__lowdim_anneal.txt"),
    "mnist_shape": (16499.31e6, "profiles/lse_bf16__mnist_shape.txt"),
    "embedding": (4391.51e6, "profiles/lse_bf16__embedding.txt"),
    "transport_grad": (77.17e6, "profiles/pass_f64__transport_grad.txt"),
}
PER_CONFIG = ("tiny", "mnist_shape", "embedding", "transport_grad")


def algorithmic_slots_per_pair(exp_cost: float = 4.0) -> float:
    """Issue slots the method itself needs per (i, j) pair on the vector ALU: one exp2 (a
    transcendental occupies the ALU for `exp_cost` full-rate slots: quarter rate) and one
    accumulation of the sum.  The score contraction (d + 2 multiply-adds per pair) runs on the
    matrix cores, which sit far below their own peak, so the pass is bound by this ALU work."""
    return exp_cost + 1


def run_workload(name, steps, warmup, schedule="alternating", n_override=None, cpu_baseline=False,
                 calibrate_copy=False):
    """Time `steps` steps of the hot path on workload `name`; returns the fields of the JSON line."""
    import numpy as np
    import torch

    from paper_2602_03067_amd import binding, workloads

    w = workloads.make(name, n=n_override, m=n_override)
    ctx = binding.Context(0)
    prob = binding.problem_from_workload(w)
    if w.U is not None:
        U = torch.from_numpy(w.U).to("cuda:0")
    else:
        U = torch.from_numpy(np.random.Generator(np.random.PCG64(w.seed + 7)).standard_normal(
            (w.n, min(w.d, 64))).astype(np.float32)).to("cuda:0")
    f = torch.zeros(w.n, device="cuda:0")
    g = torch.zeros(w.m, device="cuda:0")

    apply_ms = {"grad_x": [], "apply_plan_T": []}

    def timed(key, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        r = fn()
        e1.record()
        apply_ms[key].append((e0, e1))
        return r

    def step():
        f.zero_()
        g.zero_()
        # one batch: the clouds stay as they are for the five entry calls of the step, so the library prepares their
        # derived copies in the first one (the solve) and reuses them; the declaration ends with the step
        ctx.fs_points_keep(prob)
        ctx.fs_row_norms(prob.x)
        ctx.fs_row_norms(prob.y)
        if schedule == "symmetric":
            ctx.fs_solve_symmetric(prob, w.eps_end, w.total_iters, f, g)
        else:
            ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
        er, ec = ctx.fs_marginal_err(prob, w.eps_end, f, g)
        # gradient with respect to x in the form the workload list asks for, x - (P y)/a: the plan
        # applied to y (d value columns) and the assembly, inside the library
        grad = timed("grad_x", lambda: ctx.fs_grad_x(prob, w.eps_end, f, g, 2))
        timed("apply_plan_T", lambda: ctx.fs_apply_plan_T(prob, w.eps_end, f, g, U))
        ctx.fs_points_release()
        return er, ec, grad

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # What a solve costs beyond its streaming passes (derived copies of both clouds, norms, first biases, and
    # the merges of one iteration): a one-iteration solve at the final eps, minus its two pass launches.
    # Outside the timed region; every timed step prepares the derived copies once (in its solve; the rate is a "cold" one).
    ctx.fs_profile_enable(True)
    ctx.fs_profile_read()
    pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pe0.record()
    ctx.fs_solve(prob, w.eps_end, w.eps_end, 1, 1, f, g)
    pe1.record()
    torch.cuda.synchronize()
    p_avg, p_launches, _ = ctx.fs_profile_read()
    ctx.fs_profile_enable(False)
    prologue_ms = pe0.elapsed_time(pe1) - p_avg * p_launches
    # The solve alone with the derived copies of the clouds already in place (the "warm" rate beside the step's cold
    # one): a second solve in a row under fs_points_keep, outside the timed region.
    ctx.fs_points_keep(prob)
    ctx.fs_solve(prob, w.eps_end, w.eps_end, 1, 1, f, g)
    f.zero_()
    g.zero_()
    se0, se1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    se0.record()
    if schedule == "symmetric":
        ctx.fs_solve_symmetric(prob, w.eps_end, w.total_iters, f, g)
    else:
        ctx.fs_solve(prob, w.eps_start, w.eps_end, w.n_stages, w.iters, f, g)
    se1.record()
    torch.cuda.synchronize()
    ctx.fs_points_release()
    solve_ms = se0.elapsed_time(se1)
    # A plan application with 64 value columns (outside the timed region too): at d <= 16 the step's own applications
    # have only d columns, and an application takes eight columns per streaming pass there.
    wide_ms = None
    if w.d <= 16:
        U64 = torch.from_numpy(np.random.Generator(np.random.PCG64(w.seed + 8)).standard_normal((w.n, 64)).astype(np.float32)).to("cuda:0")
        ctx.fs_apply_plan_T(prob, w.eps_end, f, g, U64)
        we0, we1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        we0.record()
        ctx.fs_apply_plan_T(prob, w.eps_end, f, g, U64)
        we1.record()
        torch.cuda.synchronize()
        wide_ms = we0.elapsed_time(we1)
        del U64
    if calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ctx.fs_profile_enable(True)
    ctx.fs_profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        er, ec, _ = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    avg_ms, launches, pairs = ctx.fs_profile_read()
    ctx.fs_profile_enable(False)

    # the two plan applications of a step, timed on torch's stream (the library's stream is the same one)
    apply_avg = {k: (sum(a.elapsed_time(b) for a, b in v[-steps:]) / max(1, len(v[-steps:])) if v else None)
                 for k, v in apply_ms.items()}
    ms_per_step = elapsed * 1e3 / steps
    value = w.total_iters * steps / elapsed

    # ---- roofline of the dominant kernel (the streaming LSE pass) -------------------------
    if w.compute == "bf16_mfma":
        flops = 2.0 * w.d * pairs
        roof = {"bound": "mfma", "achieved": flops / (avg_ms * 1e-3) / 1e12, "peak": PEAKS["bf16"] / 1e12,
                "unit": "TFLOP/s"}
        dtype = "bf16"
    elif w.d > 16:
        flops = 2.0 * w.d * pairs
        roof = {"bound": "mfma", "achieved": flops / (avg_ms * 1e-3) / 1e12, "peak": PEAKS["f64"] / 1e12,
                "unit": "TFLOP/s"}
        # the same rate against the fp32 vector peak (157.3 TFLOP/s), the ceiling an fp32 formulation
        # would have; fp32 scores cannot hold the 1e-4 tolerance at this size of the scores
        roof["frac_of_fp32_vector_peak"] = roof["achieved"] / 157.3
        dtype = "f64"
    else:
        slots = algorithmic_slots_per_pair() * pairs
        roof = {"bound": "alu", "achieved": slots / (avg_ms * 1e-3) / 1e12,
                "peak": VALU_LANE_SLOTS_PER_S / 1e12, "unit": "Tlane-op/s"}
        dtype = "f32"
    roof["frac"] = roof["achieved"] / roof["peak"]
    traffic = MEASURED_TRAFFIC.get(w.name) if n_override is None else None
    roof["traffic"] = traffic[0] if traffic else None
    roof["traffic_source"] = (traffic[1] + " (rocprofv3 counters of an earlier run of this command, not of this run)") \
        if traffic else None
    # the same launch in the other units the workload list asks for: pair evaluations (= exponentials) per
    # second, and the measured HBM traffic as a rate and as a fraction of the 8 TB/s peak (far from it: the
    # pass is not HBM-bound; the re-reads of the streamed cloud are served by L2 and the memory-side cache)
    rates = {"pair_evals_per_s": pairs / (avg_ms * 1e-3), "exp2_per_s": pairs / (avg_ms * 1e-3)}
    if roof["traffic"]:
        rates["hbm_GB_per_s"] = roof["traffic"] / (avg_ms * 1e-3) / 1e9
        rates["hbm_frac_of_peak"] = rates["hbm_GB_per_s"] / 8000.0
    # one half-step reads both clouds and one potential and writes the other potential
    rates["algorithmic_min_bytes"] = float((w.n + w.m) * (w.d * (2 if w.compute == "bf16_mfma" else 4) + 4))
    roof["kernel"] = "streaming LSE half-step"
    roof["avg_launch_ms"] = avg_ms
    roof["launches"] = launches
    roof["pairs_per_launch"] = pairs
    if w.n * w.m < (1 << 24):
        roof["note"] = ("an iteration at this size is four dependent launches of a few microseconds each: bound by "
                        "launch latency, the fraction says little")

    out = {
        "value": value, "unit": "iterations/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "dtype": dtype,
        "config": {"workload": w.name, "n": w.n, "m": w.m, "d": w.d, "eps_start": w.eps_start,
                   "eps_end": w.eps_end, "stages": w.n_stages, "iters_per_stage": w.iters, "schedule": schedule,
                   "step": "row_norms + solve + marginal_err + grad_x (plan applied to y + assembly) + apply_plan_T"},
        "marginal_err": {"row": er, "col": ec},
        "apply_ms": {"grad_x": apply_avg["grad_x"], "grad_x_value_columns": w.d,
                     "apply_plan_T": apply_avg["apply_plan_T"], "apply_plan_T_value_columns": int(U.shape[1]),
                     "apply_plan_T_64_columns": wide_ms},
        "solve_overhead_ms": prologue_ms,
        "solve_only_warm": {"ms": solve_ms, "iterations_per_s": w.total_iters / (solve_ms * 1e-3)},
        "roofline": roof,
        "rates": rates,
    }

    # ---- the float64 oracle on the host cores, on a bounded sample -------------------------
    if cpu_baseline:
        import oracle
        R = max(1, min(w.n, w.m, int(1.2e10 / max(w.n, w.m) / max(1.0, w.d / 8.0))))
        rows = np.arange(R)
        gz = np.zeros(w.m)
        fz = np.zeros(w.n)
        eps = float(np.float32(w.eps_end))
        t1 = time.perf_counter()
        oracle.update_f(w.x, w.y, w.b, eps, gz, rows=rows)
        tf = time.perf_counter() - t1
        t1 = time.perf_counter()
        oracle.update_g(w.x, w.y, w.a, eps, fz, cols=rows)
        tg = time.perf_counter() - t1
        it_time = tf * (w.n / R) + tg * (w.m / R)
        out["cpu_baseline"] = {
            "value": 1.0 / it_time, "unit": "iterations/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "one f half-step and one g half-step restricted to %d rows against all "
                      "columns (%.1f s), extrapolated linearly in rows to a full iteration" % (R, tf + tg),
        }
    ctx.close()
    del prob, f, g, U
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="lowdim_anneal")
    ap.add_argument("--n", type=int, default=None, help="override n = m (debugging only)")
    ap.add_argument("--schedule", choices=("alternating", "symmetric"), default="alternating",
                    help="symmetric: the averaged Jacobi schedule (Eq. 4-5) at eps_end for the same number of "
                         "iterations (no annealing); the default is the metric's alternating schedule")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="only the headline workload (the default also times the other four workloads, 2 steps each)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (outside the timed region), so that a "
                         "rocprofv3 --pmc run has a kernel of known traffic to scale its counters by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path is single-GPU; "
              "sharding over GPUs is a design note only). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    head = run_workload(args.workload, args.steps, args.warmup, args.schedule, args.n,
                        cpu_baseline=not args.no_cpu_baseline, calibrate_copy=args.calibrate_copy)
    out = {"metric": "Sinkhorn iterations/sec (fused f+g)", "value": head.pop("value"), "unit": head.pop("unit"),
           "n_gpus": 1, "steps": head.pop("steps"), "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head.pop("dtype"),
           "data": "synthetic"}
    out.update(head)
    # the other workloads, same step, same fields, fewer steps (parity of each is the tests' business; these are
    # the timings of the launch configurations the tests check at full size)
    per_config = args.workload == "lowdim_anneal" and args.n is None and args.schedule == "alternating" \
        and not args.no_per_config and not args.calibrate_copy
    if per_config:
        out["per_config"] = []
        for name in PER_CONFIG:
            r = run_workload(name, 20 if name == "tiny" else 2, 1)
            r["metric"] = out["metric"]
            out["per_config"].append(r)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
