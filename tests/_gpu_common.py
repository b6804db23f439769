"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import sys

import numpy as np
import torch

from paper_2602_03067_amd import binding


def say(msg):
    """Name the case before each GPU step, flushed, so a lost box still tells which one ran."""
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def dev(arr, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(arr)).to("cuda:0").to(dtype)


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def make_problem(x, y, a, b, compute=binding.FS_COMPUTE_FP32, bf16_storage=False):
    dt = torch.bfloat16 if bf16_storage else torch.float32
    return binding.Problem(dev(x, dt), dev(y, dt), None if a is None else dev(a),
                           None if b is None else dev(b), compute)


def max_err_over_eps(got, want, eps):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / eps)
